// bppsa_spscan: the scan of Section 3.1 over CSR transposed Jacobians, with the
// hybrid schedule of Section 5.3 (a few up-sweep levels of Algorithm 1, a linear
// scan of the block totals, the matching down-sweep levels).
//
// The array [seed, Jt[0], ..., Jt[n-1]] is cut into blocks of 2^up_levels elements.
// Inside a block the elements are the leaves of a binary tree split at powers of
// two.  The plan walks that tree on the host with symbolic operands (identity,
// vector, matrix) and records a CSR x vector or CSR x CSR step for every product
// A <> B = B A it needs:
//   total(node)   = total(left) <> total(right), formed only when asked for
//                   (up-sweep: a node of 2^(d+1) leaves is level d);
//   spread(node)  : the left child inherits the node's exclusive prefix, the right
//                   child gets prefix <> total(left)   (down-sweep, level d);
//   between blocks the prefix advances serially, prefix <> total(block).
// Totals nobody asks for (the last block's, and with it anything built on the
// last array element, which an exclusive scan never outputs) are never planned.
// The index structures of the CSR x CSR products depend only on the input
// patterns and are computed when the plan is made, ahead of the training loop
// (Section 4.3); bppsa_spscan_run then only computes values.  A
// bppsa_spscan_cache keeps those structures in device memory of its own, keyed on
// a fingerprint of the input patterns, so that a later plan for the same patterns
// reuses them without running the symbolic phase again.
#include <functional>
#include <map>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "bppsa_internal.h"
#include "sparse_common.h"

namespace {

enum SlotKind { kIdent = 0, kVec = 1, kMat = 2 };
struct Slot { int kind; int id; };

struct Product {          // C = left * right; ids < n are inputs, ids >= n are products
  int left, right;
  int rows, cols;
  int level;              // the up-sweep level that forms it
  int64_t nnz;
  int64_t madds;
  int32_t* indptr;
  int32_t* indices;
  float* data;
  int numeric_kind;       // which numeric kernel forms the values (chosen when the plan is built)
  int32_t* right_split;   // BLOCK kinds: where each row of the right operand crosses the column quarters
  int max_row;            // longest row of the product
};

struct Vec {              // id 0 is the caller's seed
  int len;
  float* buf;             // arena storage (nullptr for the seed)
  int grad_index;         // >= 0: this vector is grads[grad_index]
};

struct Op {
  int kind;               // BPPSA_STEP_SPMV or BPPSA_STEP_SPGEMM
  int mat;                // SPMV: matrix id;  SPGEMM: product id (>= n)
  int vin, vout;          // SPMV
  int phase, level;
  bool diag;              // SPMV whose matrix has exactly the entries (i, i): fused into its producer
};

}  // namespace

struct bppsa_spscan_plan {
  int n = 0;
  int up_levels = 0;
  std::vector<int32_t> in_rows, in_cols;
  std::vector<int64_t> in_nnz;
  std::vector<Product> prods;
  std::vector<Vec> vecs;
  std::vector<Op> ops;
  std::vector<int> grad_vec;      // vector id holding grads[k]
  size_t arena_used = 0;
  int64_t mm_flops = 0, mv_flops = 0;
};

namespace {

struct Arena {
  char* base;
  size_t size, used;
  void* take(size_t bytes) {
    const size_t need = bppsa_align_up(bytes, 256);
    if (used + need > size) return nullptr;
    void* p = base + used;
    used += need;
    return p;
  }
};

using AllocFn = std::function<void*(size_t)>;

// The host-side walk over the tree of every block (see the head of this file).
struct Planner {
  bppsa_spscan_plan& P;
  const int last;                 // index of the last array element (= n)
  bool ok = true;                 // false once an operand combination outside Section 3.1 shows up
  std::map<std::pair<int, int>, Slot> totals;
  std::vector<Slot> prefix_of;    // exclusive prefix of every array element
  explicit Planner(bppsa_spscan_plan& p) : P(p), last(p.n), prefix_of(p.n + 1, Slot{kIdent, -1}) {}

  int mat_rows(int id) const { return id < P.n ? P.in_rows[id] : P.prods[id - P.n].rows; }
  int mat_cols(int id) const { return id < P.n ? P.in_cols[id] : P.prods[id - P.n].cols; }

  // a <> b = b a, recorded.
  Slot combine(Slot a, Slot b, int phase, int level) {
    if (a.kind == kIdent) return b;
    if (b.kind == kIdent) return a;
    if (b.kind != kMat) {           // the right operand of <> is always a matrix (Section 3.1)
      ok = false;
      return a;
    }
    if (a.kind == kVec) {
      P.vecs.push_back(Vec{mat_rows(b.id), nullptr, -1});
      const int vout = (int)P.vecs.size() - 1;
      P.ops.push_back(Op{BPPSA_STEP_SPMV, b.id, a.id, vout, phase, level, false});
      return Slot{kVec, vout};
    }
    Product pr{};
    pr.left = b.id;
    pr.right = a.id;
    pr.rows = mat_rows(b.id);
    pr.cols = mat_cols(a.id);
    pr.level = level;
    P.prods.push_back(pr);
    const int pid = P.n + (int)P.prods.size() - 1;
    P.ops.push_back(Op{BPPSA_STEP_SPGEMM, pid, -1, -1, phase, level, false});
    return Slot{kMat, pid};
  }

  // <>-product of the elements [lo, lo + size) that exist; size is a power of two
  Slot total(int lo, int size) {
    if (size == 1) return lo == 0 ? Slot{kVec, 0} : Slot{kMat, lo - 1};
    const int half = size / 2;
    if (lo + half > last) return total(lo, half);          // nothing in the right half
    const auto key = std::make_pair(lo, size);
    const auto it = totals.find(key);
    if (it != totals.end()) return it->second;
    const Slot l = total(lo, half), r = total(lo + half, half);
    const Slot t = combine(l, r, BPPSA_PHASE_UP, __builtin_ctz((unsigned)half));
    totals[key] = t;
    return t;
  }

  void spread(int lo, int size, Slot prefix) {
    if (size == 1) {
      prefix_of[lo] = prefix;
      return;
    }
    const int half = size / 2;
    if (lo + half > last) {
      spread(lo, half, prefix);
      return;
    }
    const Slot right_prefix = combine(prefix, total(lo, half), BPPSA_PHASE_DOWN, __builtin_ctz((unsigned)half));
    spread(lo, half, prefix);
    spread(lo + half, half, right_prefix);
  }
};

bppsa_csr mat_desc(const bppsa_spscan_plan& P, const bppsa_csr* Jt, int id) {
  if (id < P.n) return Jt[id];
  const Product& pr = P.prods[id - P.n];
  return bppsa_csr{pr.rows, pr.cols, pr.nnz, pr.indptr, pr.indices, pr.data};
}

bppsa_status check_inputs(int n, const bppsa_csr* Jt, int up_levels) {
  if (n < 1 || !Jt || up_levels < 0) return BPPSA_EINVAL;
  for (int k = 0; k < n; ++k) {
    if (Jt[k].rows < 1 || Jt[k].cols < 1 || Jt[k].nnz < 0 || !Jt[k].indptr) return BPPSA_EINVAL;
    if (Jt[k].nnz > 0 && !Jt[k].indices) return BPPSA_EINVAL;
    if (Jt[k].nnz >= INT32_MAX) return BPPSA_EOVERFLOW;
    if (k + 1 < n && Jt[k].rows != Jt[k + 1].cols) return BPPSA_ESHAPE;
  }
  return BPPSA_OK;
}

// Fills in everything of the plan that needs no device: sizes, steps, operand ids.
bppsa_status plan_steps(bppsa_spscan_plan& P, int n, const bppsa_csr* Jt, int up_levels) {
  P.n = n;
  for (int k = 0; k < n; ++k) {
    P.in_rows.push_back(Jt[k].rows);
    P.in_cols.push_back(Jt[k].cols);
    P.in_nnz.push_back(Jt[k].nnz);
  }
  int depth = 0;                                    // levels of a tree over all n + 1 elements
  while ((1LL << depth) < (long long)n + 1) ++depth;
  int U = up_levels;
  if (U > depth - 1) U = depth - 1;
  if (U < 0) U = 0;
  P.up_levels = U;
  P.vecs.push_back(Vec{Jt[0].cols, nullptr, -1});   // the seed
  Planner pl(P);
  const long long block = 1LL << U;
  Slot prefix{kIdent, -1};
  int j = 0;
  for (long long lo = 0; lo <= n; lo += block, ++j) {
    pl.spread((int)lo, (int)block, prefix);
    if (lo + block <= n) prefix = pl.combine(prefix, pl.total((int)lo, (int)block), BPPSA_PHASE_CHAIN, j);
  }
  if (!pl.ok) return BPPSA_EINVAL;
  // prefixes = [I, seed, grads[0], ..., grads[n-2]]; the inclusive tail needs one more product
  P.grad_vec.assign(n, -1);
  for (int k = 0; k + 2 <= n; ++k) {
    if (pl.prefix_of[k + 2].kind != kVec) return BPPSA_EINVAL;
    P.grad_vec[k] = pl.prefix_of[k + 2].id;
  }
  {
    const int vin = (n >= 2) ? P.grad_vec[n - 2] : 0;
    P.vecs.push_back(Vec{Jt[n - 1].rows, nullptr, -1});
    const int vout = (int)P.vecs.size() - 1;
    P.ops.push_back(Op{BPPSA_STEP_SPMV, n - 1, vin, vout, BPPSA_PHASE_TAIL, 0, false});
    P.grad_vec[n - 1] = vout;
  }
  for (int k = 0; k < n; ++k) P.vecs[P.grad_vec[k]].grad_index = k;
  return BPPSA_OK;
}

// The symbolic phase: structure of every product, the choice of its numeric kernel, and which
// input matrices are diagonal.  Device memory for the structures comes from `alloc`.
bppsa_status symbolic_phase(bppsa_spscan_plan& P, const bppsa_csr* Jt, const AllocFn& alloc, hipStream_t s) {
  const int n = P.n;
  unsigned long long* d_madds = static_cast<unsigned long long*>(alloc(sizeof(unsigned long long)));
  int* d_flag = static_cast<int*>(alloc(sizeof(int)));
  if (!d_madds || !d_flag) return BPPSA_EWORKSPACE;
  for (Product& pr : P.prods) {
    const bppsa_csr L = mat_desc(P, Jt, pr.left), R = mat_desc(P, Jt, pr.right);
    if (L.cols != R.rows) return BPPSA_ESHAPE;
    pr.indptr = static_cast<int32_t*>(alloc(((size_t)pr.rows + 1) * sizeof(int32_t)));
    if (!pr.indptr) return BPPSA_EWORKSPACE;
    if (hipMemsetAsync(d_madds, 0, sizeof(unsigned long long), s) != hipSuccess) return BPPSA_EHIP;
    BPPSA_TRY(bppsa_launch_spgemm_count(L, R, pr.indptr, d_madds, s));
    BPPSA_TRY(bppsa_lengths_to_indptr(pr.indptr, pr.rows, s));
    // row pointers back to the host: nnz, and the longest row (it decides the numeric kernel)
    std::vector<int32_t> hp((size_t)pr.rows + 1);
    unsigned long long madds = 0;
    if (hipMemcpyAsync(hp.data(), pr.indptr, hp.size() * sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(&madds, d_madds, sizeof(madds), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
      return BPPSA_EHIP;
    if (hp[pr.rows] < 0) return BPPSA_EOVERFLOW;    // a row-length sum that wrapped
    pr.nnz = hp[pr.rows];
    pr.madds = (int64_t)madds;
    pr.max_row = 0;
    for (int r = 0; r < pr.rows; ++r) pr.max_row = hp[r + 1] - hp[r] > pr.max_row ? hp[r + 1] - hp[r] : pr.max_row;
    pr.indices = static_cast<int32_t*>(alloc((size_t)(pr.nnz > 0 ? pr.nnz : 1) * sizeof(int32_t)));
    if (!pr.indices) return BPPSA_EWORKSPACE;
    BPPSA_TRY(bppsa_launch_spgemm_indices(L, R, pr.indptr, pr.indices, s));
    pr.numeric_kind = bppsa_spgemm_numeric_kind(pr.madds, pr.nnz, pr.max_row, R.cols);
    pr.right_split = nullptr;
    if (pr.numeric_kind >= BPPSA_SPGEMM_BLOCK_DENSE) {
      pr.right_split = static_cast<int32_t*>(alloc((size_t)3 * R.rows * sizeof(int32_t)));
      if (!pr.right_split) return BPPSA_EWORKSPACE;
      BPPSA_TRY(bppsa_launch_row_splits(R, pr.right_split, s));
    }
    P.mm_flops += 2 * pr.madds;
  }
  // Input matrices with the pattern of the identity (the ReLU Jacobians of Appendix D.2) are
  // recognised once, here, so that a run can apply them inside the kernel that produces
  // their operand.
  for (Op& op : P.ops) {
    if (op.kind != BPPSA_STEP_SPMV || op.mat >= n) continue;
    const bppsa_csr& A = Jt[op.mat];
    if (A.rows != A.cols || A.nnz != A.rows) continue;
    int flag = 1;
    if (hipMemcpyAsync(d_flag, &flag, sizeof(int), hipMemcpyHostToDevice, s) != hipSuccess) return BPPSA_EHIP;
    BPPSA_TRY(bppsa_launch_check_diagonal(A, d_flag, s));
    if (hipMemcpyAsync(&flag, d_flag, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
      return BPPSA_EHIP;
    op.diag = flag != 0;
  }
  if (hipStreamSynchronize(s) != hipSuccess) return BPPSA_EHIP;
  for (const Op& op : P.ops) {
    if (op.kind != BPPSA_STEP_SPMV || op.phase == BPPSA_PHASE_TAIL) continue;
    P.mv_flops += 2 * (op.mat < n ? P.in_nnz[op.mat] : P.prods[op.mat - n].nnz);
  }
  return BPPSA_OK;
}

// Product values and intermediate vectors: one plan's own storage, from its arena.
bppsa_status bind_values(bppsa_spscan_plan& P, Arena& ar) {
  for (size_t v = 1; v < P.vecs.size(); ++v) {
    P.vecs[v].buf = static_cast<float*>(ar.take((size_t)P.vecs[v].len * sizeof(float)));
    if (!P.vecs[v].buf) return BPPSA_EWORKSPACE;
  }
  for (Product& pr : P.prods) {
    pr.data = static_cast<float*>(ar.take((size_t)(pr.nnz > 0 ? pr.nnz : 1) * sizeof(float)));
    if (!pr.data) return BPPSA_EWORKSPACE;
  }
  P.arena_used = ar.used;
  return BPPSA_OK;
}

struct CacheEntry {
  unsigned long long key[2];
  int up_levels_asked;
  bppsa_spscan_plan tmpl;         // structure pointers into `blocks`; no values, no vectors bound
  std::vector<void*> blocks;
  ~CacheEntry() {
    for (void* b : blocks) (void)hipFree(b);
  }
};

}  // namespace

struct bppsa_spscan_cache {
  std::mutex mu;
  int device = 0;
  unsigned long long* d_key = nullptr;
  std::vector<CacheEntry*> entries;
  int64_t hits = 0, misses = 0, symbolic_products = 0;
  size_t device_bytes = 0;
};

extern "C" bppsa_status bppsa_spscan_plan_create(int n, const bppsa_csr* Jt, int up_levels,
                                                 void* arena, size_t arena_bytes, void* stream,
                                                 bppsa_spscan_plan** plan_out) {
  if (!plan_out) return BPPSA_EINVAL;
  *plan_out = nullptr;
  if (!arena || ((uintptr_t)arena & 255)) return BPPSA_EINVAL;
  BPPSA_TRY(check_inputs(n, Jt, up_levels));
  bppsa_spscan_plan* plan = new (std::nothrow) bppsa_spscan_plan();
  if (!plan) return BPPSA_EINVAL;
  Arena ar{static_cast<char*>(arena), arena_bytes, 0};
  bppsa_status st = plan_steps(*plan, n, Jt, up_levels);
  if (st == BPPSA_OK) st = symbolic_phase(*plan, Jt, [&](size_t bytes) { return ar.take(bytes); }, (hipStream_t)stream);
  if (st == BPPSA_OK) st = bind_values(*plan, ar);
  if (st != BPPSA_OK) {
    delete plan;
    return st;
  }
  *plan_out = plan;
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_spscan_cache_create(bppsa_spscan_cache** cache_out) {
  if (!cache_out) return BPPSA_EINVAL;
  *cache_out = nullptr;
  bppsa_spscan_cache* c = new (std::nothrow) bppsa_spscan_cache();
  if (!c) return BPPSA_EINVAL;
  if (hipGetDevice(&c->device) != hipSuccess || hipMalloc((void**)&c->d_key, 2 * sizeof(unsigned long long)) != hipSuccess) {
    delete c;
    return BPPSA_EHIP;
  }
  *cache_out = c;
  return BPPSA_OK;
}

extern "C" void bppsa_spscan_cache_destroy(bppsa_spscan_cache* cache) {
  if (!cache) return;
  for (CacheEntry* e : cache->entries) delete e;
  if (cache->d_key) (void)hipFree(cache->d_key);
  delete cache;
}

extern "C" bppsa_status bppsa_spscan_cache_stats(bppsa_spscan_cache* cache, int64_t* hits, int64_t* misses,
                                                 int64_t* symbolic_products, size_t* device_bytes) {
  if (!cache) return BPPSA_EINVAL;
  std::lock_guard<std::mutex> lock(cache->mu);
  if (hits) *hits = cache->hits;
  if (misses) *misses = cache->misses;
  if (symbolic_products) *symbolic_products = cache->symbolic_products;
  if (device_bytes) *device_bytes = cache->device_bytes;
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_spscan_plan_create_cached(bppsa_spscan_cache* cache, int n, const bppsa_csr* Jt,
                                                        int up_levels, void* arena, size_t arena_bytes,
                                                        void* stream, bppsa_spscan_plan** plan_out) {
  if (!plan_out) return BPPSA_EINVAL;
  *plan_out = nullptr;
  if (!cache || !arena || ((uintptr_t)arena & 255)) return BPPSA_EINVAL;
  BPPSA_TRY(check_inputs(n, Jt, up_levels));
  hipStream_t s = (hipStream_t)stream;
  std::lock_guard<std::mutex> lock(cache->mu);
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return BPPSA_EHIP;
  if (dev != cache->device) return BPPSA_EINVAL;
  // fingerprint of all row pointers and column indices, formed on the device
  unsigned long long key[2] = {0, 0};
  if (hipMemsetAsync(cache->d_key, 0, sizeof(key), s) != hipSuccess) return BPPSA_EHIP;
  {
    bppsa_hash_batch batch;
    int filled = 0;
    auto add = [&](const int32_t* a, long long count, unsigned long long salt) -> bppsa_status {
      batch.array[filled] = a;
      batch.count[filled] = count;
      batch.salt[filled] = salt;
      if (++filled < BPPSA_HASH_BATCH) return BPPSA_OK;
      filled = 0;
      return bppsa_launch_pattern_hash(batch, BPPSA_HASH_BATCH, cache->d_key, s);
    };
    for (int k = 0; k < n; ++k) {
      BPPSA_TRY(add(Jt[k].indptr, (long long)Jt[k].rows + 1, 2ull * k + 1));
      if (Jt[k].nnz > 0) BPPSA_TRY(add(Jt[k].indices, Jt[k].nnz, 2ull * k + 2));
    }
    BPPSA_TRY(bppsa_launch_pattern_hash(batch, filled, cache->d_key, s));
  }
  if (hipMemcpyAsync(key, cache->d_key, sizeof(key), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return BPPSA_EHIP;
  CacheEntry* found = nullptr;
  for (CacheEntry* e : cache->entries) {
    if (e->key[0] != key[0] || e->key[1] != key[1] || e->tmpl.n != n || e->up_levels_asked != up_levels) continue;
    bool same = true;
    for (int k = 0; k < n && same; ++k)
      same = e->tmpl.in_rows[k] == Jt[k].rows && e->tmpl.in_cols[k] == Jt[k].cols && e->tmpl.in_nnz[k] == Jt[k].nnz;
    if (same) {
      found = e;
      break;
    }
  }
  if (found) {
    ++cache->hits;
  } else {
    ++cache->misses;
    CacheEntry* e = new (std::nothrow) CacheEntry();
    if (!e) return BPPSA_EINVAL;
    e->key[0] = key[0];
    e->key[1] = key[1];
    e->up_levels_asked = up_levels;
    size_t bytes = 0;
    bppsa_status st = plan_steps(e->tmpl, n, Jt, up_levels);
    if (st == BPPSA_OK)
      st = symbolic_phase(e->tmpl, Jt, [&](size_t want) -> void* {
        void* p = nullptr;
        if (hipMalloc(&p, want) != hipSuccess) return nullptr;
        e->blocks.push_back(p);
        bytes += want;
        return p;
      }, s);
    if (st != BPPSA_OK) {
      delete e;
      return st;
    }
    cache->symbolic_products += (int64_t)e->tmpl.prods.size();
    cache->device_bytes += bytes;
    cache->entries.push_back(e);
    found = e;
  }
  bppsa_spscan_plan* plan = new (std::nothrow) bppsa_spscan_plan(found->tmpl);
  if (!plan) return BPPSA_EINVAL;
  Arena ar{static_cast<char*>(arena), arena_bytes, 0};
  const bppsa_status st = bind_values(*plan, ar);
  if (st != BPPSA_OK) {
    delete plan;
    return st;
  }
  *plan_out = plan;
  return BPPSA_OK;
}

extern "C" void bppsa_spscan_plan_destroy(bppsa_spscan_plan* plan) { delete plan; }

extern "C" size_t bppsa_spscan_plan_arena_used(const bppsa_spscan_plan* plan) {
  return plan ? plan->arena_used : 0;
}

extern "C" int bppsa_spscan_plan_num_products(const bppsa_spscan_plan* plan) {
  return plan ? (int)plan->prods.size() : 0;
}

extern "C" bppsa_status bppsa_spscan_plan_product(const bppsa_spscan_plan* plan, int idx, bppsa_csr* out,
                                                  int* left_id, int* right_id) {
  if (!plan || !out || idx < 0 || idx >= (int)plan->prods.size()) return BPPSA_EINVAL;
  const Product& pr = plan->prods[idx];
  *out = bppsa_csr{pr.rows, pr.cols, pr.nnz, pr.indptr, pr.indices, pr.data};
  if (left_id) *left_id = pr.left;
  if (right_id) *right_id = pr.right;
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_spscan_plan_flops(const bppsa_spscan_plan* plan, int64_t* mm_flops,
                                                int64_t* mv_flops) {
  if (!plan) return BPPSA_EINVAL;
  if (mm_flops) *mm_flops = plan->mm_flops;
  if (mv_flops) *mv_flops = plan->mv_flops;
  return BPPSA_OK;
}

extern "C" int bppsa_spscan_plan_num_steps(const bppsa_spscan_plan* plan) {
  return plan ? (int)plan->ops.size() : 0;
}

extern "C" bppsa_status bppsa_spscan_plan_step_flops(const bppsa_spscan_plan* plan, int idx, bppsa_spscan_step* out) {
  if (!plan || !out || idx < 0 || idx >= (int)plan->ops.size()) return BPPSA_EINVAL;
  const Op& op = plan->ops[idx];
  out->kind = op.kind;
  out->phase = op.phase;
  out->level = op.level;
  out->matrix = op.mat;
  if (op.kind == BPPSA_STEP_SPGEMM) {
    const Product& pr = plan->prods[op.mat - plan->n];
    out->flops = 2 * pr.madds;
    out->numeric_kind = pr.numeric_kind;
  } else {
    out->flops = 2 * (op.mat < plan->n ? plan->in_nnz[op.mat] : plan->prods[op.mat - plan->n].nnz);
    out->numeric_kind = -1;
  }
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_spscan_run(const bppsa_spscan_plan* plan, const bppsa_csr* Jt,
                                         const float* seed, float* const* grads, void* stream) {
  if (!plan || !Jt || !seed || !grads) return BPPSA_EINVAL;
  const bppsa_spscan_plan& P = *plan;
  for (int k = 0; k < P.n; ++k) {
    if (Jt[k].rows != P.in_rows[k] || Jt[k].cols != P.in_cols[k] || Jt[k].nnz != P.in_nnz[k])
      return BPPSA_ESHAPE;
    if (!Jt[k].indptr || (Jt[k].nnz > 0 && (!Jt[k].indices || !Jt[k].data))) return BPPSA_EINVAL;
  }
  hipStream_t s = (hipStream_t)stream;
  auto vec_ptr = [&](int vid) -> float* {
    if (vid == 0) return const_cast<float*>(seed);
    const Vec& v = P.vecs[vid];
    if (v.grad_index >= 0 && grads[v.grad_index]) return grads[v.grad_index];
    return v.buf;
  };
  for (size_t i = 0; i < P.ops.size(); ++i) {
    const Op& op = P.ops[i];
    bppsa_status st;
    if (op.kind == BPPSA_STEP_SPGEMM) {
      const Product& pr = P.prods[op.mat - P.n];
      st = bppsa_launch_spgemm_numeric(pr.numeric_kind, mat_desc(P, Jt, pr.left), mat_desc(P, Jt, pr.right),
                                       pr.right_split, pr.indptr, pr.indices, pr.data, pr.max_row, s);
    } else {
      const bool skip_tail = !grads[P.n - 1];         // inclusive tail not requested
      if (op.phase == BPPSA_PHASE_TAIL && skip_tail) continue;
      // a diagonal matrix that consumes this product in the next step is applied in the same launch
      const size_t j = i + 1;
      const bool fuse = j < P.ops.size() && P.ops[j].kind == BPPSA_STEP_SPMV && P.ops[j].diag &&
                        P.ops[j].vin == op.vout && !(P.ops[j].phase == BPPSA_PHASE_TAIL && skip_tail);
      if (fuse) {
        st = bppsa_launch_spmv(mat_desc(P, Jt, op.mat), vec_ptr(op.vin), vec_ptr(op.vout), s,
                               Jt[P.ops[j].mat].data, vec_ptr(P.ops[j].vout));
        i = j;                                      // the diagonal step is done
      } else {
        st = bppsa_launch_spmv(mat_desc(P, Jt, op.mat), vec_ptr(op.vin), vec_ptr(op.vout), s);
      }
    }
    if (st != BPPSA_OK) return st;
  }
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_spscan(int n, const bppsa_csr* Jt, const float* seed, float* const* grads,
                                     int up_levels, void* workspace, size_t workspace_bytes, void* stream) {
  bppsa_spscan_plan* plan = nullptr;
  bppsa_status st = bppsa_spscan_plan_create(n, Jt, up_levels, workspace, workspace_bytes, stream, &plan);
  if (st != BPPSA_OK) return st;
  st = bppsa_spscan_run(plan, Jt, seed, grads, stream);
  if (st == BPPSA_OK && hipStreamSynchronize((hipStream_t)stream) != hipSuccess) st = BPPSA_EHIP;
  bppsa_spscan_plan_destroy(plan);
  return st;
}
