// bppsa_spscan: the scan of Section 3.1 over CSR transposed Jacobians, with the
// hybrid schedule of Section 5.3 (a few up-sweep levels of Algorithm 1, a linear
// scan of the block totals, the matching down-sweep levels).
//
// The schedule is static for a given (n, up_levels), so the host replays
// Algorithm 1's index arithmetic symbolically once: every array slot is the
// symbolic identity, a vector or a matrix, and each A <> B = B A becomes a
// recorded CSR x vector or CSR x CSR step.  Steps whose result reaches no
// requested gradient (e.g. anything built on the last array element, which
// Algorithm 1 reads but never outputs) are dropped.  The index structures of
// the remaining CSR x CSR products depend only on the input patterns and are
// computed here, ahead of the training loop (Section 4.3); bppsa_spscan_run
// then only computes values.
#include <new>
#include <vector>

#include "bppsa_internal.h"
#include "sparse_common.h"

namespace {

enum SlotKind { kIdent = 0, kVec = 1, kMat = 2 };
struct Slot { int kind; int id; };

struct Product {          // C = left * right; ids < n are inputs, ids >= n are products
  int left, right;
  int rows, cols;
  int64_t nnz;
  int64_t madds;
  int32_t* indptr;
  int32_t* indices;
  float* data;
  bool live;
  int numeric_kind;       // which numeric kernel forms the values (chosen when the plan is built)
  int32_t* right_split;   // BLOCK kinds: where each row of the right operand crosses the column quarters
  int max_row;            // longest row of the product
};

struct Vec {              // id 0 is the caller's seed
  int len;
  float* buf;             // arena storage (nullptr for the seed)
  int grad_index;         // >= 0: this vector is grads[grad_index]
  int producer;           // op index, -1 for the seed
};

enum OpKind { kSpmv = 0, kSpgemm = 1 };
struct Op {
  int kind;
  int mat;                // kSpmv: matrix id;  kSpgemm: product id (>= n)
  int vin, vout;          // kSpmv
  bool live;
  bool tail;              // the optional inclusive-tail product
  bool diag = false;      // kSpmv whose matrix has exactly the entries (i, i): fused into its producer
};

int ceil_log2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

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
  int live_products = 0;
  std::vector<int> live_product_ids;
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

struct Builder {
  bppsa_spscan_plan& P;
  bool ok = true;                 // false once an operand combination outside Section 3.1 shows up
  explicit Builder(bppsa_spscan_plan& p) : P(p) {}

  int mat_rows(int id) const { return id < P.n ? P.in_rows[id] : P.prods[id - P.n].rows; }
  int mat_cols(int id) const { return id < P.n ? P.in_cols[id] : P.prods[id - P.n].cols; }

  int new_vec(int len, int producer) {
    P.vecs.push_back(Vec{len, nullptr, -1, producer});
    return (int)P.vecs.size() - 1;
  }

  // a <> b = b a, recorded.
  Slot combine(Slot a, Slot b) {
    if (a.kind == kIdent) return b;
    if (b.kind == kIdent) return a;
    if (b.kind != kMat) {           // the right operand of <> is always a matrix (Section 3.1)
      ok = false;
      return a;
    }
    if (a.kind == kVec) {
      const int vout = new_vec(mat_rows(b.id), (int)P.ops.size());
      P.ops.push_back(Op{kSpmv, b.id, a.id, vout, false, false});
      return Slot{kVec, vout};
    }
    Product pr{};
    pr.left = b.id;
    pr.right = a.id;
    pr.rows = mat_rows(b.id);
    pr.cols = mat_cols(a.id);
    P.prods.push_back(pr);
    const int pid = P.n + (int)P.prods.size() - 1;
    P.ops.push_back(Op{kSpgemm, pid, -1, -1, false, false});
    return Slot{kMat, pid};
  }
};

void mark_mat_live(bppsa_spscan_plan& P, int id) {
  if (id < P.n) return;
  Product& pr = P.prods[id - P.n];
  if (pr.live) return;
  pr.live = true;
  mark_mat_live(P, pr.left);
  mark_mat_live(P, pr.right);
}

void mark_vec_live(bppsa_spscan_plan& P, int vid) {
  const int opi = P.vecs[vid].producer;
  if (opi < 0 || P.ops[opi].live) return;
  Op& op = P.ops[opi];
  op.live = true;
  mark_mat_live(P, op.mat);
  mark_vec_live(P, op.vin);
}

bppsa_csr mat_desc(const bppsa_spscan_plan& P, const bppsa_csr* Jt, int id) {
  if (id < P.n) return Jt[id];
  const Product& pr = P.prods[id - P.n];
  return bppsa_csr{pr.rows, pr.cols, pr.nnz, pr.indptr, pr.indices, pr.data};
}

}  // namespace

extern "C" bppsa_status bppsa_spscan_plan_create(int n, const bppsa_csr* Jt, int up_levels,
                                                 void* arena, size_t arena_bytes, void* stream,
                                                 bppsa_spscan_plan** plan_out) {
  if (!plan_out) return BPPSA_EINVAL;
  *plan_out = nullptr;
  if (n < 1 || !Jt || up_levels < 0 || !arena) return BPPSA_EINVAL;
  if ((uintptr_t)arena & 255) return BPPSA_EINVAL;
  for (int k = 0; k < n; ++k) {
    if (Jt[k].rows < 1 || Jt[k].cols < 1 || Jt[k].nnz < 0 || !Jt[k].indptr) return BPPSA_EINVAL;
    if (Jt[k].nnz > 0 && !Jt[k].indices) return BPPSA_EINVAL;
    if (Jt[k].nnz >= INT32_MAX) return BPPSA_EOVERFLOW;
    if (k + 1 < n && Jt[k].rows != Jt[k + 1].cols) return BPPSA_ESHAPE;
  }
  hipStream_t s = (hipStream_t)stream;
  bppsa_spscan_plan* plan = new (std::nothrow) bppsa_spscan_plan();
  if (!plan) return BPPSA_EINVAL;
  bppsa_spscan_plan& P = *plan;
  P.n = n;
  for (int k = 0; k < n; ++k) {
    P.in_rows.push_back(Jt[k].rows);
    P.in_cols.push_back(Jt[k].cols);
    P.in_nnz.push_back(Jt[k].nnz);
  }

  // ---- replay Algorithm 1's indices on slots --------------------------------
  Builder B(P);
  const int N = n;                                  // array a[0..N]
  std::vector<Slot> a(N + 1);
  P.vecs.push_back(Vec{Jt[0].cols, nullptr, -1, -1});   // seed
  a[0] = Slot{kVec, 0};
  for (int k = 1; k <= N; ++k) a[k] = Slot{kMat, k - 1};
  const int levels = ceil_log2(N + 1);
  int U = up_levels;
  if (U > levels - 1) U = levels - 1;
  if (U < 0) U = 0;
  P.up_levels = U;
  for (int d = 0; d < U; ++d) {                     // truncated up-sweep
    const int half = 1 << d, step = 1 << (d + 1);
    for (int i = 0; i <= N - half; i += step) {
      const int l = i + half - 1;
      const int r = (i + step - 1 < N) ? i + step - 1 : N;
      a[r] = B.combine(a[l], a[r]);
    }
  }
  {                                                 // linear scan of the block totals
    const int block = 1 << U;
    Slot prefix{kIdent, -1};
    for (int i = 0; i <= N; i += block) {
      const int r = (i + block - 1 < N) ? i + block - 1 : N;
      const Slot total = a[r];
      a[r] = prefix;
      if (i + block <= N) prefix = B.combine(prefix, total);
    }
  }
  for (int d = U - 1; d >= 0; --d) {                // down-sweep, operands reversed
    const int half = 1 << d, step = 1 << (d + 1);
    for (int i = 0; i <= N - half; i += step) {
      const int l = i + half - 1;
      const int r = (i + step - 1 < N) ? i + step - 1 : N;
      const Slot t = a[l];
      a[l] = a[r];
      a[r] = B.combine(a[r], t);
    }
  }
  // a = [I, seed, grads[0], ..., grads[n-2]]; the inclusive tail needs one more product
  P.grad_vec.assign(n, -1);
  if (!B.ok) { delete plan; return BPPSA_EINVAL; }
  for (int k = 0; k + 2 <= N; ++k) {
    if (a[k + 2].kind != kVec) { delete plan; return BPPSA_EINVAL; }
    P.grad_vec[k] = a[k + 2].id;
  }
  {
    const int vin = (n >= 2) ? P.grad_vec[n - 2] : 0;
    const int vout = B.new_vec(Jt[n - 1].rows, (int)P.ops.size());
    P.ops.push_back(Op{kSpmv, n - 1, vin, vout, false, true});
    P.grad_vec[n - 1] = vout;
  }
  for (int k = 0; k < n; ++k) {
    P.vecs[P.grad_vec[k]].grad_index = k;
    mark_vec_live(P, P.grad_vec[k]);
  }
  for (Op& op : P.ops)
    if (op.kind == kSpgemm) op.live = P.prods[op.mat - n].live;

  // ---- device storage and the symbolic phase of the live products ------------
  Arena ar{static_cast<char*>(arena), arena_bytes, 0};
  bppsa_status st = BPPSA_OK;
  unsigned long long* d_madds = static_cast<unsigned long long*>(ar.take(sizeof(unsigned long long)));
  if (!d_madds) st = BPPSA_EWORKSPACE;
  for (size_t v = 1; v < P.vecs.size() && st == BPPSA_OK; ++v) {
    const int opi = P.vecs[v].producer;
    if (opi >= 0 && !P.ops[opi].live) continue;
    P.vecs[v].buf = static_cast<float*>(ar.take((size_t)P.vecs[v].len * sizeof(float)));
    if (!P.vecs[v].buf) st = BPPSA_EWORKSPACE;
  }
  for (size_t i = 0; i < P.prods.size() && st == BPPSA_OK; ++i) {
    Product& pr = P.prods[i];
    if (!pr.live) continue;
    const bppsa_csr L = mat_desc(P, Jt, pr.left), R = mat_desc(P, Jt, pr.right);
    if (L.cols != R.rows) { st = BPPSA_ESHAPE; break; }
    pr.indptr = static_cast<int32_t*>(ar.take(((size_t)pr.rows + 1) * sizeof(int32_t)));
    if (!pr.indptr) { st = BPPSA_EWORKSPACE; break; }
    if (hipMemsetAsync(d_madds, 0, sizeof(unsigned long long), s) != hipSuccess) { st = BPPSA_EHIP; break; }
    st = bppsa_launch_spgemm_count(L, R, pr.indptr, d_madds, s);
    if (st != BPPSA_OK) break;
    st = bppsa_lengths_to_indptr(pr.indptr, pr.rows, s);
    if (st != BPPSA_OK) break;
    int32_t nnz32 = 0;
    unsigned long long madds = 0;
    if (hipMemcpyAsync(&nnz32, pr.indptr + pr.rows, sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(&madds, d_madds, sizeof(madds), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) { st = BPPSA_EHIP; break; }
    if (nnz32 < 0) { st = BPPSA_EOVERFLOW; break; }   // a row-length sum that wrapped
    pr.nnz = nnz32;
    pr.madds = (int64_t)madds;
    pr.indices = static_cast<int32_t*>(ar.take((size_t)(pr.nnz > 0 ? pr.nnz : 1) * sizeof(int32_t)));
    pr.data = static_cast<float*>(ar.take((size_t)(pr.nnz > 0 ? pr.nnz : 1) * sizeof(float)));
    if (!pr.indices || !pr.data) { st = BPPSA_EWORKSPACE; break; }
    st = bppsa_launch_spgemm_indices(L, R, pr.indptr, pr.indices, s);
    if (st != BPPSA_OK) break;
    // the numeric kernel depends on the longest row of the product (read back once, here)
    {
      std::vector<int32_t> hp((size_t)pr.rows + 1);
      if (hipMemcpyAsync(hp.data(), pr.indptr, hp.size() * sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess ||
          hipStreamSynchronize(s) != hipSuccess) { st = BPPSA_EHIP; break; }
      int mx = 0;
      for (int r = 0; r < pr.rows; ++r) mx = hp[r + 1] - hp[r] > mx ? hp[r + 1] - hp[r] : mx;
      pr.max_row = mx;
    }
    pr.numeric_kind = bppsa_spgemm_numeric_kind(pr.madds, pr.nnz, pr.max_row, R.cols);
    pr.right_split = nullptr;
    if (pr.numeric_kind >= BPPSA_SPGEMM_BLOCK_DENSE) {
      pr.right_split = static_cast<int32_t*>(ar.take((size_t)3 * R.rows * sizeof(int32_t)));
      if (!pr.right_split) { st = BPPSA_EWORKSPACE; break; }
      st = bppsa_launch_row_splits(R, pr.right_split, s);
      if (st != BPPSA_OK) break;
    }
    P.mm_flops += 2 * pr.madds;
    P.live_product_ids.push_back((int)i);
  }
  // Input matrices with the pattern of the identity (the ReLU Jacobians of Appendix D.2) are
  // recognised once, here, so that a run can apply them inside the kernel that produces
  // their operand.
  int* d_flag = static_cast<int*>(ar.take(sizeof(int)));
  if (!d_flag && st == BPPSA_OK) st = BPPSA_EWORKSPACE;
  for (size_t i = 0; i < P.ops.size() && st == BPPSA_OK; ++i) {
    Op& op = P.ops[i];
    if (!op.live || op.kind != kSpmv || op.mat >= n) continue;
    const bppsa_csr& A = Jt[op.mat];
    if (A.rows != A.cols || A.nnz != A.rows) continue;
    int flag = 1;
    if (hipMemcpyAsync(d_flag, &flag, sizeof(int), hipMemcpyHostToDevice, s) != hipSuccess) { st = BPPSA_EHIP; break; }
    st = bppsa_launch_check_diagonal(A, d_flag, s);
    if (st != BPPSA_OK) break;
    if (hipMemcpyAsync(&flag, d_flag, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) { st = BPPSA_EHIP; break; }
    op.diag = flag != 0;
  }
  if (st == BPPSA_OK && hipStreamSynchronize(s) != hipSuccess) st = BPPSA_EHIP;
  if (st != BPPSA_OK) { delete plan; return st; }
  for (const Op& op : P.ops) {
    if (!op.live || op.kind != kSpmv) continue;
    const int64_t nnz = op.mat < n ? P.in_nnz[op.mat] : P.prods[op.mat - n].nnz;
    if (!op.tail) P.mv_flops += 2 * nnz;
  }
  P.arena_used = ar.used;
  P.live_products = (int)P.live_product_ids.size();
  *plan_out = plan;
  return BPPSA_OK;
}

extern "C" void bppsa_spscan_plan_destroy(bppsa_spscan_plan* plan) { delete plan; }

extern "C" size_t bppsa_spscan_plan_arena_used(const bppsa_spscan_plan* plan) {
  return plan ? plan->arena_used : 0;
}

extern "C" int bppsa_spscan_plan_num_products(const bppsa_spscan_plan* plan) {
  return plan ? plan->live_products : 0;
}

extern "C" bppsa_status bppsa_spscan_plan_product(const bppsa_spscan_plan* plan, int idx, bppsa_csr* out,
                                                  int* left_id, int* right_id) {
  if (!plan || !out || idx < 0 || idx >= plan->live_products) return BPPSA_EINVAL;
  const Product& pr = plan->prods[plan->live_product_ids[idx]];
  *out = bppsa_csr{pr.rows, pr.cols, pr.nnz, pr.indptr, pr.indices, pr.data};
  // report operand ids with products renumbered over the live ones only
  auto renum = [&](int id) {
    if (id < plan->n) return id;
    for (int k = 0; k < plan->live_products; ++k)
      if (plan->live_product_ids[k] == id - plan->n) return plan->n + k;
    return -1;
  };
  if (left_id) *left_id = renum(pr.left);
  if (right_id) *right_id = renum(pr.right);
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_spscan_plan_flops(const bppsa_spscan_plan* plan, int64_t* mm_flops,
                                                int64_t* mv_flops) {
  if (!plan) return BPPSA_EINVAL;
  if (mm_flops) *mm_flops = plan->mm_flops;
  if (mv_flops) *mv_flops = plan->mv_flops;
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
    if (!op.live) continue;
    bppsa_status st;
    if (op.kind == kSpgemm) {
      const Product& pr = P.prods[op.mat - P.n];
      st = bppsa_launch_spgemm_numeric(pr.numeric_kind, mat_desc(P, Jt, pr.left), mat_desc(P, Jt, pr.right),
                                       pr.right_split, pr.indptr, pr.indices, pr.data, pr.max_row, s);
    } else {
      if (op.tail && !grads[P.n - 1]) continue;     // inclusive tail not requested
      // a diagonal matrix that consumes this product is applied in the same launch
      size_t j = i + 1;
      while (j < P.ops.size() && !P.ops[j].live) ++j;
      const bool fuse = j < P.ops.size() && P.ops[j].kind == kSpmv && P.ops[j].diag &&
                        P.ops[j].vin == op.vout && !(P.ops[j].tail && !grads[P.n - 1]);
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
