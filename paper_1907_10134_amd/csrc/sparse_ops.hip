// Sparse kernels behind the CSR form of A <> B = B A (Section 3.3): a
// row-parallel CSR x dense-vector product for everything that touches the
// gradient vector, and a row-parallel CSR x CSR product for interior up-sweep
// nodes, split into a symbolic phase (row lengths, then ascending column
// indices, both from a per-row bitmap of B's columns held in LDS) and a numeric
// phase, so that the symbolic work can be done once ahead of the training loop
// (Section 4.3).  The numeric phase adds the terms of every value in a fixed order.
#include "bppsa_internal.h"
#include "sparse_common.h"

namespace {

__global__ void __launch_bounds__(1024)
lengths_to_indptr_kernel(int32_t* __restrict__ a, int n) {
  __shared__ int wave_off[16];
  __shared__ int chunk_total;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int carry = 0;
  for (int base = 0; base < n; base += 1024) {
    const int i = base + threadIdx.x;
    const int v = (i < n) ? a[i] : 0;
    int incl = v;
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    if (lane == 63) wave_off[wave] = incl;
    __syncthreads();
    if (wave == 0) {
      const int ws = (lane < 16) ? wave_off[lane] : 0;
      int wi = ws;
      for (int off = 1; off < 16; off <<= 1) {
        const int t = __shfl_up(wi, off);
        if (lane >= off) wi += t;
      }
      if (lane < 16) wave_off[lane] = wi - ws;
      if (lane == 15) chunk_total = wi;
    }
    __syncthreads();
    if (i < n) a[i] = carry + wave_off[wave] + incl - v;
    carry += chunk_total;
    __syncthreads();
  }
  if (threadIdx.x == 0) a[n] = carry;
}

// One wave per row: lanes stride over the row's entries, then reduce.
__global__ void __launch_bounds__(256)
spmv_wave_kernel(int rows, const int32_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                 const float* __restrict__ data, const float* __restrict__ x, float* __restrict__ y,
                 const float* __restrict__ d, float* __restrict__ y2) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int s = indptr[row], e = indptr[row + 1];
  float acc = 0.f;
  for (int p = s + lane; p < e; p += 64) acc += data[p] * x[indices[p]];
  for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
  if (lane == 0) {
    y[row] = acc;
    if (y2) y2[row] = d[row] * acc;
  }
}

// One lane per row: for matrices with about one entry per row (ReLU, max-pooling).
__global__ void __launch_bounds__(256)
spmv_lane_kernel(int rows, const int32_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                 const float* __restrict__ data, const float* __restrict__ x, float* __restrict__ y,
                 const float* __restrict__ d, float* __restrict__ y2) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= rows) return;
  const int s = indptr[row], e = indptr[row + 1];
  float acc = 0.f;
  for (int p = s; p < e; ++p) acc += data[p] * x[indices[p]];
  y[row] = acc;
  if (y2) y2[row] = d[row] * acc;
}

__global__ void __launch_bounds__(256)
check_diagonal_kernel(int rows, const int32_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                      int* __restrict__ flag) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i > rows) return;
  bool ok = indptr[i] == i;
  if (i < rows) ok = ok && indices[i] == i;
  if (!ok) *flag = 0;
}

// Mark, in an LDS bitmap, every column of B reachable from row `row` of A.  Waves take
// entries of A's row, lanes take entries of the matching row of B.  Returns (to every
// thread of wave 0, lane 0 only is used) nothing; the caller syncs.
__device__ __forceinline__ unsigned long long
mark_row(int row, const int32_t* __restrict__ a_indptr, const int32_t* __restrict__ a_indices,
         const int32_t* __restrict__ b_indptr, const int32_t* __restrict__ b_indices,
         unsigned int* bitmap) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwave = blockDim.x >> 6;
  const int as = a_indptr[row], ae = a_indptr[row + 1];
  unsigned long long work = 0;
  for (int p = as + wave; p < ae; p += nwave) {
    const int k = a_indices[p];
    const int bs = b_indptr[k], be = b_indptr[k + 1];
    for (int q = bs + lane; q < be; q += 64) {
      const int col = b_indices[q];
      atomicOr(&bitmap[col >> 5], 1u << (col & 31));
    }
    if (lane == 0) work += (unsigned long long)(be - bs);
  }
  return work;
}

// MODE 0: row length -> c_indptr[row], multiply-add count -> *madds.
// MODE 1: ascending column indices -> c_indices[c_indptr[row] ...].
template <int MODE>
__global__ void __launch_bounds__(256)
spgemm_symbolic_kernel(int words, const int32_t* __restrict__ a_indptr,
                       const int32_t* __restrict__ a_indices, const int32_t* __restrict__ b_indptr,
                       const int32_t* __restrict__ b_indices, int32_t* __restrict__ c_indptr,
                       int32_t* __restrict__ c_indices, unsigned long long* __restrict__ madds) {
  extern __shared__ unsigned int bitmap[];
  __shared__ int wave_sum[4];
  __shared__ int carry_s;
  const int row = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int wd = threadIdx.x; wd < words; wd += blockDim.x) bitmap[wd] = 0u;
  __syncthreads();
  const unsigned long long work = mark_row(row, a_indptr, a_indices, b_indptr, b_indices, bitmap);
  __syncthreads();
  if (MODE == 0) {
    int cnt = 0;
    for (int wd = threadIdx.x; wd < words; wd += blockDim.x) cnt += __popc(bitmap[wd]);
    for (int m = 32; m >= 1; m >>= 1) cnt += __shfl_xor(cnt, m);
    if (lane == 0) wave_sum[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) c_indptr[row] = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
    if (lane == 0 && work) atomicAdd(madds, work);
  } else {
    int carry = c_indptr[row];
    for (int base = 0; base < words; base += 256) {
      const int wd = base + threadIdx.x;
      unsigned int bits = (wd < words) ? bitmap[wd] : 0u;
      const int v = __popc(bits);
      int incl = v;
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      if (lane == 63) wave_sum[wave] = incl;
      __syncthreads();
      int woff = 0;
      for (int k = 0; k < wave; ++k) woff += wave_sum[k];
      int pos = carry + woff + incl - v;
      while (bits) {
        const int b = __ffs(bits) - 1;
        c_indices[pos++] = wd * 32 + b;
        bits &= bits - 1u;
      }
      if (threadIdx.x == 255) carry_s = carry + woff + incl;
      __syncthreads();
      carry = carry_s;
      __syncthreads();
    }
  }
}

// ---- fingerprint of an index array ----------------------------------------------------------------
// Each element contributes two 64-bit words, bit-mixed from (position, value, salt) with the
// multiply-xorshift finaliser of the SplitMix64 generator; the words of all elements are summed
// modulo 2^64, so the result is independent of the order in which waves arrive.
__device__ __forceinline__ unsigned long long mix64(unsigned long long x) {
  x ^= x >> 30;
  x *= 0xbf58476d1ce4e5b9ull;
  x ^= x >> 27;
  x *= 0x94d049bb133111ebull;
  x ^= x >> 31;
  return x;
}

__global__ void __launch_bounds__(256)
pattern_hash_kernel(bppsa_hash_batch batch, unsigned long long* __restrict__ out) {
  const int32_t* __restrict__ a = batch.array[blockIdx.y];
  const long long count = batch.count[blockIdx.y];
  const unsigned long long salt = batch.salt[blockIdx.y];
  unsigned long long h0 = 0, h1 = 0;
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
    const unsigned long long x = ((unsigned long long)i << 32) | (unsigned int)a[i];
    h0 += mix64(x ^ (salt * 0x9e3779b97f4a7c15ull));
    h1 += mix64((x + salt) * 0xd1342543de82ef95ull + 1);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    h0 += __shfl_down(h0, off, 64);
    h1 += __shfl_down(h1, off, 64);
  }
  if ((threadIdx.x & 63) == 0 && (h0 | h1) != 0) {
    atomicAdd(out, h0);
    atomicAdd(out + 1, h1);
  }
}

// ---- numeric phase of C = A B for a known structure ---------------------------------------------
// Every value of C is formed by ONE wave, which adds the terms of an entry in an order fixed by
// the structure of A and B alone, so the values are the same bits on every run; no two waves ever
// add to the same accumulator.  Three kernels, chosen once per product when the plan is built:
//
//   single : every entry of C is exactly one product a * b (the number of multiply-adds equals
//            nnz(C): a diagonal or selection matrix on either side, i.e. every product with a ReLU
//            or pooling Jacobian).  Nothing is summed; one wave per row writes the products to
//            their places.
//   wave   : rows of C of up to kWaveRowCap entries: one wave per row stages the row's column
//            indices in LDS, walks A's row and adds each term at the slot found by binary search.
//   block  : longer rows: one workgroup per row.  The columns are cut into four equal ranges, one
//            per wave, and a table built with the plan says where each row of B crosses those
//            boundaries, so a wave reads exactly its share of every row of B and owns its share of
//            the accumulators: one per column of B, or one per entry of the longest row of C
//            plus a rank table (whichever takes less LDS), or, when neither fits kBlockLdsBytes,
//            the row itself in global memory.
constexpr int kWaveRowCap = 1024;
constexpr size_t kBlockLdsBytes = 64 * 1024;   // most LDS one workgroup of the BLOCK kinds takes

// first position in sorted idx[0..n) whose value is >= col
__device__ __forceinline__ int lower_bound_i32(const int32_t* idx, int n, int col) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (idx[mid] < col) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// split[3 k + j] = first entry of row k of B whose column is >= (j + 1) * ceil(cols / 4)
__global__ void __launch_bounds__(256)
row_splits_kernel(int rows, int cols, const int32_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                  int32_t* __restrict__ split) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= 3 * rows) return;
  const int k = t / 3, j = t - 3 * k;
  const int quarter = (cols + 3) / 4;
  const int s = indptr[k], e = indptr[k + 1];
  split[t] = s + lower_bound_i32(indices + s, e - s, (j + 1) * quarter);
}

__global__ void __launch_bounds__(256)
spgemm_numeric_single_kernel(int rows, const int32_t* __restrict__ a_indptr, const int32_t* __restrict__ a_indices,
                             const float* __restrict__ a_data, const int32_t* __restrict__ b_indptr,
                             const int32_t* __restrict__ b_indices, const float* __restrict__ b_data,
                             const int32_t* __restrict__ c_indptr, const int32_t* __restrict__ c_indices,
                             float* __restrict__ c_data) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int cs = c_indptr[row], n = c_indptr[row + 1] - cs;
  if (n == 0) return;
  const int as = a_indptr[row], ae = a_indptr[row + 1];
  if (ae - as == 1) {                            // the row of C is a scaled copy of one row of B
    const int k = a_indices[as];
    const float av = a_data[as];
    const int bs = b_indptr[k];
    for (int j = lane; j < n; j += 64) c_data[cs + j] = av * b_data[bs + j];
    return;
  }
  // one lane per entry of A's row; its (short) row of B goes to the places found by binary search
  for (int p = as + lane; p < ae; p += 64) {
    const int k = a_indices[p];
    const float av = a_data[p];
    const int bs = b_indptr[k], be = b_indptr[k + 1];
    for (int q = bs; q < be; ++q) {
      const int slot = lower_bound_i32(c_indices + cs, n, b_indices[q]);
      c_data[cs + slot] = av * b_data[q];
    }
  }
}

__global__ void __launch_bounds__(256)
spgemm_numeric_wave_kernel(int rows, const int32_t* __restrict__ a_indptr, const int32_t* __restrict__ a_indices,
                           const float* __restrict__ a_data, const int32_t* __restrict__ b_indptr,
                           const int32_t* __restrict__ b_indices, const float* __restrict__ b_data,
                           const int32_t* __restrict__ c_indptr, const int32_t* __restrict__ c_indices,
                           float* __restrict__ c_data) {
  __shared__ int32_t cidx_s[4][kWaveRowCap];
  __shared__ float acc_s[4][kWaveRowCap];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows) return;                       // no workgroup barrier below: waves are independent
  int32_t* cidx = cidx_s[wave];
  float* acc = acc_s[wave];
  const int cs = c_indptr[row], n = c_indptr[row + 1] - cs;
  if (n == 0) return;
  const int as = a_indptr[row], ae = a_indptr[row + 1];
  for (int j = lane; j < n; j += 64) {
    cidx[j] = c_indices[cs + j];
    acc[j] = 0.f;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  // Entries of A's row in storage order; the entries of one row of B have distinct columns, so
  // the lanes of one step never meet at a slot, and LDS operations of a wave complete in order.
  // Each lane first fetches one entry of A's row and the bounds of its row of B; the wave then
  // takes them four at a time so that the loads of four rows of B are in flight together.
  for (int p0 = as; p0 < ae; p0 += 64) {
    const int mine = p0 + lane;
    int bs_l = 0, be_l = 0;
    float av_l = 0.f;
    if (mine < ae) {
      const int k = a_indices[mine];
      av_l = a_data[mine];
      bs_l = b_indptr[k];
      be_l = b_indptr[k + 1];
    }
    const int cnt = (ae - p0 < 64) ? (ae - p0) : 64;
    for (int e = 0; e < cnt; e += 4) {
      int bs[4], be[4], col[4];
      float av[4], bv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int src = (e + u < cnt) ? e + u : e;
        bs[u] = __builtin_amdgcn_readlane(bs_l, src);
        be[u] = (e + u < cnt) ? __builtin_amdgcn_readlane(be_l, src) : bs[u];
        av[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, av_l), src));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int q = bs[u] + lane;
        col[u] = (q < be[u]) ? b_indices[q] : -1;
        bv[u] = (q < be[u]) ? b_data[q] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (col[u] >= 0) acc[lower_bound_i32(cidx, n, col[u])] += av[u] * bv[u];
        for (int q0 = bs[u] + 64 + lane; q0 < be[u]; q0 += 64)      // a row of B longer than one wave
          acc[lower_bound_i32(cidx, n, b_indices[q0])] += av[u] * b_data[q0];
      }
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  for (int j = lane; j < n; j += 64) c_data[cs + j] = acc[j];
}

// One workgroup of four waves per row of C; wave w owns the columns [w q, (w + 1) q), q = ceil(cols / 4),
// and with them every value of the row that falls there, so each value is summed by one wave in
// one order.
//   MODE 0: one LDS accumulator per column of B.
//   MODE 1: one LDS accumulator per entry of the row; the place of a column is its rank among the
//           row's columns, read from a table of (bits, entries before) per 32 columns.
//   MODE 2: the row stays in global memory, places by binary search; the additions are memory-side
//           add operations, all additions to one entry issued by one wave in program order.
// The wave walks A's row 64 entries at a time (one per lane: value and the bounds of its share of
// the row of B), and takes their shares in pieces of 64 entries: first pieces of all entries, then
// second pieces, and so on.  Pieces are fetched kDepth at a time and the fetch of the next kDepth
// is issued before the current ones are added, so the additions run under the memory latency.
constexpr int kDepth = 8;

struct Pieces {
  int col[kDepth];
  float bv[kDepth];
  float av[kDepth];
};

// takes up to kDepth entries out of `todo` (one bit per lane whose share has a piece number `round`)
__device__ __forceinline__ int fetch_pieces(Pieces& pc, unsigned long long& todo, int round, int lane, int bs_l,
                                            int be_l, float av_l, const int32_t* __restrict__ b_indices,
                                            const float* __restrict__ b_data) {
  int got = 0;
#pragma unroll
  for (int u = 0; u < kDepth; ++u) {
    pc.col[u] = -1;
    pc.bv[u] = 0.f;
    pc.av[u] = 0.f;
    if (todo != 0) {                                   // uniform over the wave
      const int src = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int q = __builtin_amdgcn_readlane(bs_l, src) + 64 * round + lane;
      const int e = __builtin_amdgcn_readlane(be_l, src);
      pc.av[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, av_l), src));
      if (q < e) {
        pc.col[u] = b_indices[q];
        pc.bv[u] = b_data[q];
      }
      ++got;
    }
  }
  return got;
}

template <int MODE>
__global__ void __launch_bounds__(256)
spgemm_numeric_block_kernel(int b_cols, const int32_t* __restrict__ a_indptr, const int32_t* __restrict__ a_indices,
                            const float* __restrict__ a_data, const int32_t* __restrict__ b_indptr,
                            const int32_t* __restrict__ b_indices, const float* __restrict__ b_data,
                            const int32_t* __restrict__ b_split, const int32_t* __restrict__ c_indptr,
                            const int32_t* __restrict__ c_indices, float* __restrict__ c_data) {
  extern __shared__ float lds[];
  const int row = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cs = c_indptr[row], ce = c_indptr[row + 1];
  const int n = ce - cs;
  const int as = a_indptr[row], ae = a_indptr[row + 1];
  if (n == 0) return;                            // uniform over the workgroup
  // MODE 1: rank table first (8 bytes per 32 columns), then the accumulators
  const int words = (b_cols + 31) >> 5;
  uint2* rk = reinterpret_cast<uint2*>(lds);
  float* cacc = lds + 2 * words;
  if (MODE == 0) {
    for (int p = threadIdx.x; p < n; p += blockDim.x) lds[c_indices[cs + p]] = 0.f;
  } else if (MODE == 1) {
    for (int w = threadIdx.x; w < words; w += blockDim.x) rk[w] = make_uint2(0u, 0u);
    __syncthreads();
    for (int p = threadIdx.x; p < n; p += blockDim.x) {
      const int c = c_indices[cs + p];
      atomicOr(&rk[c >> 5].x, 1u << (c & 31));   // integer: the result does not depend on the order
      if (p == 0 || (c_indices[cs + p - 1] >> 5) != (c >> 5)) rk[c >> 5].y = (unsigned)p;
      cacc[p] = 0.f;
    }
  } else {
    for (int p = cs + threadIdx.x; p < ce; p += blockDim.x) c_data[p] = 0.f;
  }
  __syncthreads();
  const int quarter = (b_cols + 3) / 4;
  int slot_lo = 0, slot_n = n;                   // MODE 2: the places of this wave's columns
  if (MODE == 2) {
    slot_lo = lower_bound_i32(c_indices + cs, n, wave * quarter);
    slot_n = lower_bound_i32(c_indices + cs, n, (wave + 1) * quarter) - slot_lo;
  }
  auto add = [&](const Pieces& pc) {
#pragma unroll
    for (int u = 0; u < kDepth; ++u) {
      const int c = pc.col[u];
      if (c >= 0) {                              // the lanes of one piece hold distinct columns
        const float t = pc.av[u] * pc.bv[u];
        if (MODE == 0) {
          lds[c] += t;
        } else if (MODE == 1) {
          const uint2 r = rk[c >> 5];
          cacc[r.y + __builtin_popcount(r.x & ((1u << (c & 31)) - 1u))] += t;
        } else {
          atomicAdd(&c_data[cs + slot_lo + lower_bound_i32(c_indices + cs + slot_lo, slot_n, c)], t);
        }
      }
    }
  };
  for (int p0 = as; p0 < ae; p0 += 64) {
    const int mine = p0 + lane;
    int bs_l = 0, be_l = 0;
    float av_l = 0.f;
    if (mine < ae) {
      const int k = a_indices[mine];
      av_l = a_data[mine];
      bs_l = wave == 0 ? b_indptr[k] : b_split[3 * k + wave - 1];
      be_l = wave == 3 ? b_indptr[k + 1] : b_split[3 * k + wave];
    }
    for (int round = 0;; ++round) {
      unsigned long long todo = __ballot(be_l - bs_l > 64 * round);
      if (todo == 0) break;
      Pieces cur, nxt;
      int have = fetch_pieces(cur, todo, round, lane, bs_l, be_l, av_l, b_indices, b_data);
      while (have > 0) {
        have = fetch_pieces(nxt, todo, round, lane, bs_l, be_l, av_l, b_indices, b_data);
        add(cur);
        cur = nxt;
      }
    }
  }
  if (MODE == 2) return;
  __syncthreads();
  if (MODE == 0) {
    for (int p = threadIdx.x; p < n; p += blockDim.x) c_data[cs + p] = lds[c_indices[cs + p]];
  } else {
    for (int p = threadIdx.x; p < n; p += blockDim.x) c_data[cs + p] = cacc[p];
  }
}

}  // namespace

bppsa_status bppsa_lengths_to_indptr(int32_t* a, int n, hipStream_t stream) {
  lengths_to_indptr_kernel<<<1, 1024, 0, stream>>>(a, n);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_launch_spmv(const bppsa_csr& A, const float* x, float* y, hipStream_t stream,
                               const float* d, float* y2) {
  if (A.rows < 1) return BPPSA_OK;
  if (A.nnz >= 4 * (int64_t)A.rows)
    spmv_wave_kernel<<<bppsa_ceil_div(A.rows, 4), 256, 0, stream>>>(A.rows, A.indptr, A.indices, A.data, x, y, d,
                                                                    y2);
  else
    spmv_lane_kernel<<<bppsa_ceil_div(A.rows, 256), 256, 0, stream>>>(A.rows, A.indptr, A.indices, A.data, x, y,
                                                                      d, y2);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_launch_check_diagonal(const bppsa_csr& A, int* flag, hipStream_t stream) {
  if (A.rows != A.cols || A.nnz != A.rows) return BPPSA_EINVAL;
  check_diagonal_kernel<<<bppsa_ceil_div(A.rows + 1, 256), 256, 0, stream>>>(A.rows, A.indptr, A.indices, flag);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

static int bitmap_words(const bppsa_csr& B) { return (B.cols + 31) / 32; }

bppsa_status bppsa_launch_spgemm_count(const bppsa_csr& A, const bppsa_csr& B, int32_t* c_indptr,
                                       unsigned long long* madds, hipStream_t stream) {
  if (B.cols > kBppsaMaxSpgemmCols) return BPPSA_ESHAPE;
  const int words = bitmap_words(B);
  const size_t lds = (size_t)words * sizeof(unsigned int);
  if (lds > 48 * 1024)
    BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)spgemm_symbolic_kernel<0>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  spgemm_symbolic_kernel<0><<<A.rows, 256, lds, stream>>>(words, A.indptr, A.indices, B.indptr, B.indices,
                                                          c_indptr, nullptr, madds);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_launch_spgemm_indices(const bppsa_csr& A, const bppsa_csr& B, const int32_t* c_indptr,
                                         int32_t* c_indices, hipStream_t stream) {
  if (B.cols > kBppsaMaxSpgemmCols) return BPPSA_ESHAPE;
  const int words = bitmap_words(B);
  const size_t lds = (size_t)words * sizeof(unsigned int);
  if (lds > 48 * 1024)
    BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)spgemm_symbolic_kernel<1>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  spgemm_symbolic_kernel<1><<<A.rows, 256, lds, stream>>>(words, A.indptr, A.indices, B.indptr, B.indices,
                                                          const_cast<int32_t*>(c_indptr), c_indices, nullptr);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_launch_pattern_hash(const bppsa_hash_batch& batch, int n, unsigned long long* out,
                                       hipStream_t stream) {
  if (n < 1) return BPPSA_OK;
  if (n > BPPSA_HASH_BATCH) return BPPSA_EINVAL;
  pattern_hash_kernel<<<dim3(64, n), 256, 0, stream>>>(batch, out);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_launch_row_splits(const bppsa_csr& B, int32_t* split, hipStream_t stream) {
  if (B.rows < 1) return BPPSA_OK;
  row_splits_kernel<<<bppsa_ceil_div(3 * B.rows, 256), 256, 0, stream>>>(B.rows, B.cols, B.indptr, B.indices, split);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

static size_t dense_lds_bytes(int b_cols) { return (size_t)b_cols * sizeof(float); }
static size_t ranked_lds_bytes(int c_max_row, int b_cols) {
  return (size_t)c_max_row * sizeof(float) + (size_t)((b_cols + 31) / 32) * 8;
}

int bppsa_spgemm_numeric_kind(int64_t madds, int64_t c_nnz, int c_max_row, int b_cols) {
  if (madds == c_nnz) return BPPSA_SPGEMM_SINGLE;
  if (c_max_row <= kWaveRowCap) return BPPSA_SPGEMM_WAVE;
  const size_t dense = dense_lds_bytes(b_cols), ranked = ranked_lds_bytes(c_max_row, b_cols);
  // one accumulator per column costs one LDS access less per term: it wins unless the rank table
  // and the row's accumulators are clearly smaller (more workgroups per compute unit)
  if (dense <= kBlockLdsBytes && (dense <= 16 * 1024 || 4 * dense <= 5 * ranked)) return BPPSA_SPGEMM_BLOCK_DENSE;
  if (ranked <= kBlockLdsBytes) return BPPSA_SPGEMM_BLOCK_STAGED;
  return BPPSA_SPGEMM_BLOCK_GLOBAL;
}

bppsa_status bppsa_launch_spgemm_numeric(int kind, const bppsa_csr& A, const bppsa_csr& B, const int32_t* b_split,
                                         const int32_t* c_indptr, const int32_t* c_indices, float* c_data,
                                         int c_max_row, hipStream_t stream) {
  if (A.rows < 1) return BPPSA_OK;
#define BPPSA_NUMERIC_ARGS A.indptr, A.indices, A.data, B.indptr, B.indices, B.data
  switch (kind) {
    case BPPSA_SPGEMM_SINGLE:
      spgemm_numeric_single_kernel<<<bppsa_ceil_div(A.rows, 4), 256, 0, stream>>>(A.rows, BPPSA_NUMERIC_ARGS, c_indptr,
                                                                                  c_indices, c_data);
      break;
    case BPPSA_SPGEMM_WAVE:
      spgemm_numeric_wave_kernel<<<bppsa_ceil_div(A.rows, 4), 256, 0, stream>>>(A.rows, BPPSA_NUMERIC_ARGS, c_indptr,
                                                                                c_indices, c_data);
      break;
    case BPPSA_SPGEMM_BLOCK_DENSE:
      if (!b_split) return BPPSA_EINVAL;
      if (dense_lds_bytes(B.cols) > kBlockLdsBytes) return BPPSA_EINVAL;
      if (dense_lds_bytes(B.cols) > 48 * 1024)
        BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)spgemm_numeric_block_kernel<0>,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBlockLdsBytes));
      spgemm_numeric_block_kernel<0><<<A.rows, 256, dense_lds_bytes(B.cols), stream>>>(B.cols, BPPSA_NUMERIC_ARGS, b_split, c_indptr,
                                                                 c_indices, c_data);
      break;
    case BPPSA_SPGEMM_BLOCK_STAGED:
      if (!b_split) return BPPSA_EINVAL;
      if (ranked_lds_bytes(c_max_row, B.cols) > kBlockLdsBytes) return BPPSA_EINVAL;
      if (ranked_lds_bytes(c_max_row, B.cols) > 48 * 1024)
        BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)spgemm_numeric_block_kernel<1>,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBlockLdsBytes));
      spgemm_numeric_block_kernel<1><<<A.rows, 256, ranked_lds_bytes(c_max_row, B.cols), stream>>>(B.cols, BPPSA_NUMERIC_ARGS, b_split, c_indptr,
                                                                 c_indices, c_data);
      break;
    case BPPSA_SPGEMM_BLOCK_GLOBAL:
      if (!b_split) return BPPSA_EINVAL;
      spgemm_numeric_block_kernel<2><<<A.rows, 256, 0, stream>>>(B.cols, BPPSA_NUMERIC_ARGS, b_split, c_indptr,
                                                                 c_indices, c_data);
      break;
    default:
      return BPPSA_EINVAL;
  }
#undef BPPSA_NUMERIC_ARGS
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_spmv(const bppsa_csr* A, const float* x, float* y, void* stream) {
  if (!A || !x || !y || !A->indptr || (A->nnz > 0 && (!A->indices || !A->data))) return BPPSA_EINVAL;
  if (A->rows < 1 || A->cols < 1 || A->nnz < 0) return BPPSA_EINVAL;
  if (A->nnz >= INT32_MAX) return BPPSA_EOVERFLOW;
  return bppsa_launch_spmv(*A, x, y, (hipStream_t)stream);
}
