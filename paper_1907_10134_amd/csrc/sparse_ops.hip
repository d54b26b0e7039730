// Sparse kernels behind the CSR form of A <> B = B A (Section 3.3): a
// row-parallel CSR x dense-vector product for everything that touches the
// gradient vector, and a row-parallel CSR x CSR product for interior up-sweep
// nodes, split into a symbolic phase (row lengths, then ascending column
// indices, both from a per-row bitmap of B's columns held in LDS) and a numeric
// phase, so that the symbolic work can be done once ahead of the training loop
// (Section 4.3).
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

// C's row is owned by one workgroup and accumulated in 48 KB of LDS (three workgroups per
// compute unit):
//   DENSE  - B has at most kNumericCap columns: one accumulator per column, products are
//            added at acc[col] with LDS atomics and the row's entries are gathered at the end;
//   !DENSE - rows of up to kNumericCap / 2 entries stage their (ascending) column indices in
//            LDS, every product finds its slot by binary search there; longer rows take the
//            same steps directly in global memory.
constexpr int kNumericCap = 12288;

template <bool DENSE>
__global__ void __launch_bounds__(256)
spgemm_numeric_kernel(int b_cols, const int32_t* __restrict__ a_indptr, const int32_t* __restrict__ a_indices,
                      const float* __restrict__ a_data, const int32_t* __restrict__ b_indptr,
                      const int32_t* __restrict__ b_indices, const float* __restrict__ b_data,
                      const int32_t* __restrict__ c_indptr, const int32_t* __restrict__ c_indices,
                      float* __restrict__ c_data) {
  __shared__ float lds[kNumericCap];
  const int row = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwave = blockDim.x >> 6;
  const int cs = c_indptr[row], ce = c_indptr[row + 1];
  const int n = ce - cs;
  const int as = a_indptr[row], ae = a_indptr[row + 1];
  if (n == 0) return;
  if (DENSE) {
    for (int p = threadIdx.x; p < n; p += blockDim.x) lds[c_indices[cs + p]] = 0.f;
    __syncthreads();
    // Each lane first fetches one entry of A's row and the bounds of the matching row of B;
    // the wave then walks those entries four at a time so that the loads of four rows of B are
    // in flight together (the rows are short, so one row per trip would leave the wave waiting
    // on memory most of the time).
    for (int p0 = as + wave * 64; p0 < ae; p0 += nwave * 64) {
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
        for (int u = 0; u < 4; ++u)
          if (col[u] >= 0) atomicAdd(&lds[col[u]], av[u] * bv[u]);
        for (int u = 0; u < 4; ++u) {             // rows of B longer than one wave: four loads in flight
          for (int q0 = bs[u] + 64 + lane; q0 < be[u]; q0 += 256) {
            int c4[4];
            float v4[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              const int q = q0 + 64 * w;
              c4[w] = (q < be[u]) ? b_indices[q] : -1;
              v4[w] = (q < be[u]) ? b_data[q] : 0.f;
            }
#pragma unroll
            for (int w = 0; w < 4; ++w)
              if (c4[w] >= 0) atomicAdd(&lds[c4[w]], av[u] * v4[w]);
          }
        }
      }
    }
    __syncthreads();
    for (int p = threadIdx.x; p < n; p += blockDim.x) c_data[cs + p] = lds[c_indices[cs + p]];
    return;
  }
  if (n <= kNumericCap / 2) {
    float* cacc = lds;
    int32_t* cidx = reinterpret_cast<int32_t*>(lds + kNumericCap / 2);
    for (int p = threadIdx.x; p < n; p += blockDim.x) {
      cidx[p] = c_indices[cs + p];
      cacc[p] = 0.f;
    }
    __syncthreads();
    for (int p = as + wave; p < ae; p += nwave) {
      const int k = a_indices[p];
      const float av = a_data[p];
      const int bs = b_indptr[k], be = b_indptr[k + 1];
      for (int q = bs + lane; q < be; q += 64) {
        const int col = b_indices[q];
        int lo = 0, hi = n - 1;
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if (cidx[mid] < col) lo = mid + 1; else hi = mid;
        }
        atomicAdd(&cacc[lo], av * b_data[q]);
      }
    }
    __syncthreads();
    for (int p = threadIdx.x; p < n; p += blockDim.x) c_data[cs + p] = cacc[p];
    return;
  }
  for (int p = cs + threadIdx.x; p < ce; p += blockDim.x) c_data[p] = 0.f;
  __syncthreads();
  for (int p = as + wave; p < ae; p += nwave) {
    const int k = a_indices[p];
    const float av = a_data[p];
    const int bs = b_indptr[k], be = b_indptr[k + 1];
    for (int q = bs + lane; q < be; q += 64) {
      const int col = b_indices[q];
      int lo = cs, hi = ce - 1;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (c_indices[mid] < col) lo = mid + 1; else hi = mid;
      }
      atomicAdd(&c_data[lo], av * b_data[q]);
    }
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

bppsa_status bppsa_launch_spgemm_numeric(const bppsa_csr& A, const bppsa_csr& B, const int32_t* c_indptr,
                                         const int32_t* c_indices, float* c_data, hipStream_t stream) {
  if (B.cols <= kNumericCap)
    spgemm_numeric_kernel<true><<<A.rows, 256, 0, stream>>>(B.cols, A.indptr, A.indices, A.data, B.indptr, B.indices,
                                                            B.data, c_indptr, c_indices, c_data);
  else
    spgemm_numeric_kernel<false><<<A.rows, 256, 0, stream>>>(B.cols, A.indptr, A.indices, A.data, B.indptr,
                                                             B.indices, B.data, c_indptr, c_indices, c_data);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_spmv(const bppsa_csr* A, const float* x, float* y, void* stream) {
  if (!A || !x || !y || !A->indptr || (A->nnz > 0 && (!A->indices || !A->data))) return BPPSA_EINVAL;
  if (A->rows < 1 || A->cols < 1 || A->nnz < 0) return BPPSA_EINVAL;
  if (A->nnz >= INT32_MAX) return BPPSA_EOVERFLOW;
  return bppsa_launch_spmv(*A, x, y, (hipStream_t)stream);
}
