// H = 128 GRU kernels: the gate pre-activations are a [rows x 128] x [128 x 384] product and
// run on the matrix cores; the Jacobians (Appendix E) are then streamed out with the three
// recurrent weight matrices held in registers.
#include "bppsa_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int H = 128;
constexpr int LS = H + 4;          // LDS row stride of the staged hidden states (bank spread)
constexpr int kBatch = 32;         // (t, b) rows per gate tile = one MFMA block of rows

__device__ __forceinline__ float sigmoidf_(float a) { return 1.0f / (1.0f + expf(-a)); }

// Gates of kBatch rows for the 32 hidden units j = 32 w + (lane % 32), computed by one wave.
//   R = W_hr h' + b_hr, Z = W_hz h' + b_hz, M = W_hn h' + b_hn   (32x32x2 fp32 MFMA, K = 128)
//   r = sigmoid(W_ir x + b_ir + R), z = sigmoid(W_iz x + b_iz + Z), n = tanh(W_in x + b_in + r M)
// hp: LDS [kBatch][LS], rows past the end zero-filled.  The weights are read straight from
// global memory (196 KB, cache resident): lane l needs W[gate row 32 w + l % 32][4 consecutive k].
// emit(row, j, r, z, n, M, h'[row][j]) is called for every valid row of the tile.
template <class F>
__device__ __forceinline__ void gru_gates_h128(int w, int lane, long long row0, long long rows, int I,
                                               const float* hp, const float* __restrict__ x,
                                               const float* __restrict__ w_ih, const float* __restrict__ w_hh,
                                               const float* __restrict__ b_ih, const float* __restrict__ b_hh,
                                               F&& emit) {
  const int l32 = lane & 31, hs = lane >> 5;
  const int j = 32 * w + l32;
  v16f acc[3];
#pragma unroll
  for (int g = 0; g < 3; ++g)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[g][v] = 0.f;
  const float* arow = hp + l32 * LS + 4 * hs;
  const float* wrow = w_hh + (size_t)j * H + 4 * hs;
#pragma unroll 4
  for (int g8 = 0; g8 < 16; ++g8) {
    const v4f a4 = *reinterpret_cast<const v4f*>(arow + 8 * g8);
    v4f b4[3];
#pragma unroll
    for (int g = 0; g < 3; ++g) b4[g] = *reinterpret_cast<const v4f*>(wrow + (size_t)g * H * H + 8 * g8);
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int g = 0; g < 3; ++g)
        acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[s], b4[g][s], acc[g], 0, 0, 0);
  }
  const float bhr = b_hh ? b_hh[j] : 0.f, bhz = b_hh ? b_hh[H + j] : 0.f, bhn = b_hh ? b_hh[2 * H + j] : 0.f;
  const float bir = b_ih ? b_ih[j] : 0.f, biz = b_ih ? b_ih[H + j] : 0.f, bin = b_ih ? b_ih[2 * H + j] : 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = 8 * (v >> 2) + 4 * hs + (v & 3);
    if (row0 + row < rows) {
      float ir = bir, iz = biz, in = bin;
      const float* xr = x + (size_t)(row0 + row) * I;
      for (int i = 0; i < I; ++i) {
        const float xv = xr[i];
        ir += w_ih[(size_t)j * I + i] * xv;
        iz += w_ih[(size_t)(H + j) * I + i] * xv;
        in += w_ih[(size_t)(2 * H + j) * I + i] * xv;
      }
      const float r = sigmoidf_(ir + (acc[0][v] + bhr));
      const float z = sigmoidf_(iz + (acc[1][v] + bhz));
      const float M = acc[2][v] + bhn;
      const float n = tanhf(in + r * M);
      emit(row, j, r, z, n, M, hp[row * LS + j]);
    }
  }
}

// Stage h'[row0 .. row0 + kBatch) into LDS, zero-filling rows past the end.
template <int THREADS>
__device__ __forceinline__ void stage_hidden(int tid, long long row0, long long rows,
                                             const float* __restrict__ h, float* hp) {
#pragma unroll
  for (int q = 0; q < kBatch * (H / 4) / THREADS; ++q) {
    const int e = tid + q * THREADS;
    const int row = e >> 5, c4 = (e & 31) * 4;
    v4f v = {0.f, 0.f, 0.f, 0.f};
    if (row0 + row < rows) v = *reinterpret_cast<const v4f*>(h + (size_t)(row0 + row) * H + c4);
    *reinterpret_cast<v4f*>(hp + row * LS + c4) = v;
  }
}

// Jt[i][j] = W_hr[j][i] a_j + W_hn[j][i] c_j + W_hz[j][i] e_j + [i == j] z_j   (Appendix E)
// Persistent workgroups of 512 threads.  Thread (i0 = tid / 32, j4 = 4 (tid % 32)) owns the
// elements (i0 + 16 q, j4 .. j4 + 3), q < 8, of every tile and keeps the matching 3 x 32 weights
// in registers, so a tile costs 16 coefficient reads from LDS, 96 multiply-adds and eight
// 16-byte streaming stores per thread.
constexpr int kJacThreads = 512;

__global__ void __launch_bounds__(kJacThreads, 2)
gru_jacobians_h128_kernel(long long rows, int I, long long nbatch, const float* __restrict__ h,
                          const float* __restrict__ x, const float* __restrict__ w_ih,
                          const float* __restrict__ w_hh, const float* __restrict__ b_ih,
                          const float* __restrict__ b_hh, float* __restrict__ Jt) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* hp = smem;                    // [kBatch][LS]
  float* coef = smem + kBatch * LS;    // [kBatch][4][H]: a, c, e, z
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int j4 = (tid & 31) * 4, i0 = tid >> 5;
  v4f wr[8], wn[8], wz[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int i = i0 + 16 * q;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      wr[q][u] = w_hh[(size_t)(j4 + u) * H + i];
      wz[q][u] = w_hh[(size_t)(H + j4 + u) * H + i];
      wn[q][u] = w_hh[(size_t)(2 * H + j4 + u) * H + i];
    }
  }
  for (long long batch = blockIdx.x; batch < nbatch; batch += gridDim.x) {
    const long long row0 = batch * kBatch;
    const int nrows = (int)((rows - row0 < kBatch) ? (rows - row0) : kBatch);
    stage_hidden<kJacThreads>(tid, row0, rows, h, hp);
    __syncthreads();
    if (wave < 4) {
      gru_gates_h128(wave, lane, row0, rows, I, hp, x, w_ih, w_hh, b_ih, b_hh,
                     [&](int row, int j, float r, float z, float n, float M, float hprev) {
                       const float dn = (1.f - z) * (1.f - n * n);
                       float* c = coef + row * 4 * H;
                       c[j] = dn * M * r * (1.f - r);
                       c[H + j] = dn * r;
                       c[2 * H + j] = (hprev - n) * z * (1.f - z);
                       c[3 * H + j] = z;
                     });
    }
    __syncthreads();
    for (int r = 0; r < nrows; ++r) {
      const float* c = coef + r * 4 * H + j4;
      const v4f ca = *reinterpret_cast<const v4f*>(c);
      const v4f cc = *reinterpret_cast<const v4f*>(c + H);
      const v4f ce = *reinterpret_cast<const v4f*>(c + 2 * H);
      const v4f cz = *reinterpret_cast<const v4f*>(c + 3 * H);
      float* dst = Jt + (size_t)(row0 + r) * H * H + j4;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int i = i0 + 16 * q;
        v4f o = wr[q] * ca + wn[q] * cc + wz[q] * ce;
#pragma unroll
        for (int u = 0; u < 4; ++u) o[u] += (i == j4 + u) ? cz[u] : 0.f;
        __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(dst + (size_t)i * H));
      }
    }
    __syncthreads();                   // hp and coef are rewritten by the next batch
  }
}

// delta[row][0..4H) = (dR, dZ, dN, dM) for every (t, b) row, given g = dL/dh[t+1]: the chain
// rule through the cell of Section 4.2 with the gates recomputed as above.
constexpr int kDeltaThreads = 256;

__global__ void __launch_bounds__(kDeltaThreads)
gru_deltas_h128_kernel(long long rows, int I, const float* __restrict__ h, const float* __restrict__ x,
                       const float* __restrict__ G, const float* __restrict__ w_ih,
                       const float* __restrict__ w_hh, const float* __restrict__ b_ih,
                       const float* __restrict__ b_hh, float* __restrict__ delta) {
  __shared__ __attribute__((aligned(16))) float hp[kBatch * LS];
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * kBatch;
  stage_hidden<kDeltaThreads>(tid, row0, rows, h, hp);
  __syncthreads();
  gru_gates_h128(tid >> 6, tid & 63, row0, rows, I, hp, x, w_ih, w_hh, b_ih, b_hh,
                 [&](int row, int j, float r, float z, float n, float M, float hprev) {
                   const float gv = G[(size_t)(row0 + row) * H + j];
                   const float dN = gv * (1.f - z) * (1.f - n * n);
                   const float dZ = gv * (hprev - n) * z * (1.f - z);
                   float* d = delta + (size_t)(row0 + row) * 4 * H;
                   d[j] = dN * M * r * (1.f - r);
                   d[H + j] = dZ;
                   d[2 * H + j] = dN;
                   d[3 * H + j] = dN * r;
                 });
}

}  // namespace

bppsa_status bppsa_build_jacobians_gru_h128(int T, int B, int I, const float* h, const float* x,
                                            const float* w_ih, const float* w_hh, const float* b_ih,
                                            const float* b_hh, float* Jt, hipStream_t stream) {
  const long long rows = (long long)T * B;
  const long long nbatch = (rows + kBatch - 1) / kBatch;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  const long long grid = nbatch < cus ? nbatch : cus;     // one 81 KB workgroup per compute unit
  const size_t lds = (size_t)(kBatch * LS + kBatch * 4 * H) * sizeof(float);
  BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)gru_jacobians_h128_kernel,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  gru_jacobians_h128_kernel<<<(int)grid, kJacThreads, lds, stream>>>(rows, I, nbatch, h, x, w_ih, w_hh, b_ih,
                                                                    b_hh, Jt);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_gru_deltas_h128(long long rows, int I, const float* h, const float* x, const float* G,
                                   const float* w_ih, const float* w_hh, const float* b_ih,
                                   const float* b_hh, float* delta, hipStream_t stream) {
  const long long nbatch = (rows + kBatch - 1) / kBatch;
  if (nbatch > 0x7fffffffLL) return BPPSA_EOVERFLOW;
  gru_deltas_h128_kernel<<<(int)nbatch, kDeltaThreads, 0, stream>>>(rows, I, h, x, G, w_ih, w_hh, b_ih, b_hh,
                                                                   delta);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
