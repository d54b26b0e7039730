// GRU variants of the Jacobian builder and of the parameter-gradient reduction.
//
// Cell (Section 4.2; Appendix E's rewrite with pre-activations R, Z, M, N):
//   r = sigmoid(R), z = sigmoid(Z), n = tanh(N), N = W_in x + b_in + r o M,
//   M = W_hn h' + b_hn, h = (1 - z) o n + z o h'.
// Appendix E's closed form for the transposed Jacobian scales column j of
// W_hr^T, W_hn^T and W_hz^T by per-sample coefficients and adds diag(z):
//   Jt[i][j] = W_hr[j][i] a_j + W_hn[j][i] c_j + W_hz[j][i] e_j + [i == j] z_j,
//   a = (1-z)(1-n^2) M r(1-r),  c = (1-z)(1-n^2) r,  e = (h' - n) z(1-z).
// The gates are not inputs: they are recomputed here from (h', x, weights) for
// all steps in parallel, as the paper does (Appendix E, last paragraph).
#include "bppsa_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kRows = 16;    // (step, sample) rows per workgroup
constexpr int kGateTile = 32;

__device__ __forceinline__ float sigmoidf_(float a) { return 1.0f / (1.0f + expf(-a)); }

// gh[r][g] = b_hh[g] + sum_k W_hh[g][k] hp[r][k] for the workgroup's rows, g in [0, 3H).
// hp: LDS [kRows][H]; gh: LDS [kRows][3H]; wt: LDS [kGateTile][H + 1].
__device__ void hidden_preactivations(int H, int nrows, const float* __restrict__ w_hh,
                                      const float* __restrict__ b_hh, const float* hp,
                                      float* gh, float* wt) {
  const int G3 = 3 * H;
  const int ld = H + 1;
  for (int g0 = 0; g0 < G3; g0 += kGateTile) {
    for (int e = threadIdx.x; e < kGateTile * H; e += kThreads) {
      const int g = e / H, k = e - g * H;
      wt[g * ld + k] = (g0 + g < G3) ? w_hh[(size_t)(g0 + g) * H + k] : 0.f;
    }
    __syncthreads();
    for (int p = threadIdx.x; p < kRows * kGateTile; p += kThreads) {
      const int r = p / kGateTile, g = p - r * kGateTile;
      if (r < nrows && g0 + g < G3) {
        float acc = b_hh ? b_hh[g0 + g] : 0.f;
        const float* a = hp + r * H;
        const float* w = wt + g * ld;
        for (int k = 0; k < H; ++k) acc += a[k] * w[k];
        gh[r * G3 + g0 + g] = acc;
      }
    }
    __syncthreads();
  }
}

struct Gates { float r, z, n, M; };

__device__ __forceinline__ Gates gates_at(int H, int I, int j, const float* __restrict__ xr,
                                          const float* __restrict__ w_ih,
                                          const float* __restrict__ b_ih, const float* ghr) {
  float ir = b_ih ? b_ih[j] : 0.f, iz = b_ih ? b_ih[H + j] : 0.f, in = b_ih ? b_ih[2 * H + j] : 0.f;
  for (int i = 0; i < I; ++i) {
    const float xv = xr[i];
    ir += w_ih[(size_t)j * I + i] * xv;
    iz += w_ih[(size_t)(H + j) * I + i] * xv;
    in += w_ih[(size_t)(2 * H + j) * I + i] * xv;
  }
  Gates g;
  g.r = sigmoidf_(ir + ghr[j]);
  g.z = sigmoidf_(iz + ghr[H + j]);
  g.M = ghr[2 * H + j];
  g.n = tanhf(in + g.r * g.M);
  return g;
}

// One workgroup materialises the Jacobians of kRows consecutive (t, b) rows.
__global__ void __launch_bounds__(kThreads)
gru_jacobians_kernel(long long rows, int H, int I,
                     const float* __restrict__ h, const float* __restrict__ x,
                     const float* __restrict__ w_ih, const float* __restrict__ w_hh,
                     const float* __restrict__ b_ih, const float* __restrict__ b_hh,
                     float* __restrict__ Jt) {
  extern __shared__ float smem[];
  const int G3 = 3 * H;
  float* hp = smem;                         // [kRows][H]
  float* gh = hp + kRows * H;               // [kRows][3H]
  float* coef = gh + kRows * G3;            // [kRows][4][H]  a, c, e, z
  float* wt = coef + kRows * 4 * H;         // max([kGateTile][H+1], 3 x [32][33])
  const long long row0 = (long long)blockIdx.x * kRows;
  const int nrows = (int)((rows - row0 < kRows) ? (rows - row0) : kRows);
  for (int e = threadIdx.x; e < nrows * H; e += kThreads) hp[e] = h[(size_t)row0 * H + e];
  __syncthreads();
  hidden_preactivations(H, nrows, w_hh, b_hh, hp, gh, wt);
  for (int p = threadIdx.x; p < nrows * H; p += kThreads) {
    const int r = p / H, j = p - r * H;
    const Gates g = gates_at(H, I, j, x + (size_t)(row0 + r) * I, w_ih, b_ih, gh + r * G3);
    const float dn = (1.f - g.z) * (1.f - g.n * g.n);
    float* c = coef + r * 4 * H;
    c[j] = dn * g.M * g.r * (1.f - g.r);
    c[H + j] = dn * g.r;
    c[2 * H + j] = (hp[p] - g.n) * g.z * (1.f - g.z);
    c[3 * H + j] = g.z;
  }
  __syncthreads();
  // Stream the matrices out tile by tile; the weight tiles are transposed through LDS so
  // that both the weight reads (along i) and the Jacobian writes (along j) are contiguous.
  float* tr = wt;              // [32 j][33]  W_hr[j0+jj][i0+ii]
  float* tn = wt + 32 * 33;    // W_hn
  float* tz = wt + 2 * 32 * 33;  // W_hz
  for (int i0 = 0; i0 < H; i0 += 32) {
    for (int j0 = 0; j0 < H; j0 += 32) {
      for (int e = threadIdx.x; e < 32 * 32; e += kThreads) {
        const int jj = e >> 5, ii = e & 31;
        const int i = i0 + ii, j = j0 + jj;
        const bool ok = (i < H) && (j < H);
        tr[jj * 33 + ii] = ok ? w_hh[(size_t)j * H + i] : 0.f;
        tz[jj * 33 + ii] = ok ? w_hh[(size_t)(H + j) * H + i] : 0.f;
        tn[jj * 33 + ii] = ok ? w_hh[(size_t)(2 * H + j) * H + i] : 0.f;
      }
      __syncthreads();
      for (int e = threadIdx.x; e < nrows * 32 * 32; e += kThreads) {
        const int r = e >> 10, ii = (e >> 5) & 31, jj = e & 31;
        const int i = i0 + ii, j = j0 + jj;
        if (i < H && j < H) {
          const float* c = coef + r * 4 * H;
          float v = tr[jj * 33 + ii] * c[j] + tn[jj * 33 + ii] * c[H + j] + tz[jj * 33 + ii] * c[2 * H + j];
          if (i == j) v += c[3 * H + j];
          Jt[((size_t)(row0 + r) * H + i) * H + j] = v;
        }
      }
      __syncthreads();
    }
  }
}

size_t jacobians_lds_bytes(int H) {
  size_t wt = (size_t)kGateTile * (H + 1);
  if (wt < 3 * 32 * 33) wt = 3 * 32 * 33;
  return ((size_t)kRows * H * (1 + 3 + 4) + wt) * sizeof(float);
}

// delta[row][0..4H) = (dR, dZ, dN, dM) for every (t, b) row, given g = dL/dh[t+1].
__global__ void __launch_bounds__(kThreads)
gru_deltas_kernel(long long rows, int H, int I,
                  const float* __restrict__ h, const float* __restrict__ x,
                  const float* __restrict__ G,
                  const float* __restrict__ w_ih, const float* __restrict__ w_hh,
                  const float* __restrict__ b_ih, const float* __restrict__ b_hh,
                  float* __restrict__ delta) {
  extern __shared__ float smem[];
  const int G3 = 3 * H;
  float* hp = smem;
  float* gh = hp + kRows * H;
  float* wt = gh + kRows * G3;
  const long long row0 = (long long)blockIdx.x * kRows;
  const int nrows = (int)((rows - row0 < kRows) ? (rows - row0) : kRows);
  for (int e = threadIdx.x; e < nrows * H; e += kThreads) hp[e] = h[(size_t)row0 * H + e];
  __syncthreads();
  hidden_preactivations(H, nrows, w_hh, b_hh, hp, gh, wt);
  for (int p = threadIdx.x; p < nrows * H; p += kThreads) {
    const int r = p / H, j = p - r * H;
    const Gates g = gates_at(H, I, j, x + (size_t)(row0 + r) * I, w_ih, b_ih, gh + r * G3);
    const float gv = G[(size_t)(row0 + r) * H + j];
    const float dN = gv * (1.f - g.z) * (1.f - g.n * g.n);
    const float dZ = gv * (hp[p] - g.n) * g.z * (1.f - g.z);
    float* d = delta + (size_t)(row0 + r) * 4 * H;
    d[j] = dN * g.M * g.r * (1.f - g.r);
    d[H + j] = dZ;
    d[2 * H + j] = dN;
    d[3 * H + j] = dN * g.r;
  }
}

// Partial sums of  D_h^T [h' | 1]  and  D_i^T [x | 1]  over a range of rows, for a tile
// of kGateTile gates.  Output layout per split: [3H][H + 1 + I + 1].
constexpr int kTileRows = 32;

template <int MAXE>
__global__ void __launch_bounds__(kThreads)
gru_param_partials_kernel(long long rows, int H, int I, int rows_per_split,
                          const float* __restrict__ h, const float* __restrict__ x,
                          const float* __restrict__ delta, float* __restrict__ part) {
  extern __shared__ float smem[];
  const int WH = H + 1, WI = I + 1, W = WH + WI;
  float* Dh = smem;                         // [kTileRows][kGateTile]
  float* Di = Dh + kTileRows * kGateTile;   // [kTileRows][kGateTile]
  float* U = Di + kTileRows * kGateTile;    // [kTileRows][W]  = [h' | 1 | x | 1]
  const int g0 = blockIdx.x * kGateTile;
  const int G3 = 3 * H;
  const long long r_begin = (long long)blockIdx.y * rows_per_split;
  long long r_end = r_begin + rows_per_split;
  if (r_end > rows) r_end = rows;
  const int E = kGateTile * W;
  float acc[MAXE];
#pragma unroll
  for (int k = 0; k < MAXE; ++k) acc[k] = 0.f;
  for (long long r0 = r_begin; r0 < r_end; r0 += kTileRows) {
    const int nr = (int)((r_end - r0 < kTileRows) ? (r_end - r0) : kTileRows);
    for (int e = threadIdx.x; e < nr * kGateTile; e += kThreads) {
      const int rr = e / kGateTile, g = g0 + (e - rr * kGateTile);
      float dh = 0.f, di = 0.f;
      if (g < G3) {
        const float* d = delta + (size_t)(r0 + rr) * 4 * H;
        di = d[g];                               // (dR, dZ, dN)
        dh = (g < 2 * H) ? d[g] : d[g + H];      // (dR, dZ, dM)
      }
      Dh[e] = dh;
      Di[e] = di;
    }
    for (int e = threadIdx.x; e < nr * W; e += kThreads) {
      const int rr = e / W, c = e - rr * W;
      float u;
      if (c < H) u = h[(size_t)(r0 + rr) * H + c];
      else if (c == H) u = 1.f;
      else if (c < WH + I) u = x[(size_t)(r0 + rr) * I + (c - WH)];
      else u = 1.f;
      U[e] = u;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < MAXE; ++k) {
      const int e = threadIdx.x + k * kThreads;
      if (e < E) {
        const int g = e / W, c = e - g * W;
        const float* D = (c < WH) ? Dh : Di;
        float a = acc[k];
        for (int rr = 0; rr < nr; ++rr) a += D[rr * kGateTile + g] * U[rr * W + c];
        acc[k] = a;
      }
    }
    __syncthreads();
  }
  float* dst = part + ((size_t)blockIdx.y * G3 + g0) * W;
#pragma unroll
  for (int k = 0; k < MAXE; ++k) {
    const int e = threadIdx.x + k * kThreads;
    if (e < E && g0 + e / W < G3) dst[e] = acc[k];
  }
}

__global__ void __launch_bounds__(kThreads)
gru_param_finish_kernel(int nsplit, int H, int I, const float* __restrict__ part,
                        float* __restrict__ dW_ih, float* __restrict__ dW_hh,
                        float* __restrict__ db_ih, float* __restrict__ db_hh) {
  const int WH = H + 1, WI = I + 1, W = WH + WI;
  const int E = 3 * H * W;
  const int lane = threadIdx.x & 63;
  const int e = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (e >= E) return;
  float s = 0.f;
  for (int k = lane; k < nsplit; k += 64) s += part[(size_t)k * E + e];
  for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m);
  if (lane != 0) return;
  const int g = e / W, c = e - g * W;
  if (c < H) dW_hh[(size_t)g * H + c] = s;
  else if (c == H) db_hh[g] = s;
  else if (c < WH + I) dW_ih[(size_t)g * I + (c - WH)] = s;
  else db_ih[g] = s;
}

int gru_splits(long long rows) {
  long long ns = (rows + 4 * kTileRows - 1) / (4 * kTileRows);
  if (ns > 128) ns = 128;
  if (ns < 1) ns = 1;
  return (int)ns;
}

size_t deltas_lds_bytes(int H) {
  return ((size_t)kRows * H * 4 + (size_t)kGateTile * (H + 1)) * sizeof(float);
}

}  // namespace

// matrix-core variants for H = 128
bppsa_status bppsa_build_jacobians_gru_h128(int T, int B, int I, const float* h, const float* x,
                                            const float* w_ih, const float* w_hh, const float* b_ih,
                                            const float* b_hh, float* Jt, hipStream_t stream);
bppsa_status bppsa_gru_deltas_h128(long long rows, int I, const float* h, const float* x, const float* G,
                                   const float* w_ih, const float* w_hh, const float* b_ih,
                                   const float* b_hh, float* delta, hipStream_t stream);
bppsa_status bppsa_gru_param_partials_h128(long long rows, int I, int nsplit, const float* h, const float* x,
                                           const float* delta, float* part, hipStream_t stream);

bppsa_status bppsa_build_jacobians_gru(int T, int B, int H, int I,
                                       const float* h, const float* x,
                                       const float* w_ih, const float* w_hh,
                                       const float* b_ih, const float* b_hh,
                                       float* Jt, hipStream_t stream) {
  if (H > 128) return BPPSA_EUNSUPPORTED;
  if (H == 128) return bppsa_build_jacobians_gru_h128(T, B, I, h, x, w_ih, w_hh, b_ih, b_hh, Jt, stream);
  const long long rows = (long long)T * B;
  const long long nblk = (rows + kRows - 1) / kRows;
  if (nblk > 0x7fffffffLL) return BPPSA_EOVERFLOW;
  const size_t lds = jacobians_lds_bytes(H);
  if (lds > 48 * 1024)
    BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)gru_jacobians_kernel,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  gru_jacobians_kernel<<<(int)nblk, kThreads, lds, stream>>>(rows, H, I, h, x, w_ih, w_hh, b_ih, b_hh, Jt);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

size_t bppsa_param_grads_gru_ws(int T, int B, int H, int I) {
  const long long rows = (long long)T * B;
  const size_t W = (size_t)H + 1 + I + 1;
  return bppsa_align_up((size_t)rows * 4 * H * sizeof(float), 256) +
         bppsa_align_up((size_t)gru_splits(rows) * 3 * H * W * sizeof(float), 256);
}

bppsa_status bppsa_param_grads_gru(int T, int B, int H, int I,
                                   const float* h, const float* x, const float* G,
                                   const float* w_ih, const float* w_hh,
                                   const float* b_ih, const float* b_hh,
                                   float* dW_ih, float* dW_hh, float* db_ih, float* db_hh,
                                   void* workspace, size_t workspace_bytes, hipStream_t stream) {
  if (H > 128) return BPPSA_EUNSUPPORTED;
  const long long rows = (long long)T * B;
  const int W = H + 1 + I + 1;
  const int E = kGateTile * W;
  if (E > 32 * kThreads) return BPPSA_EUNSUPPORTED;
  if (!workspace || workspace_bytes < bppsa_param_grads_gru_ws(T, B, H, I)) return BPPSA_EWORKSPACE;
  float* delta = static_cast<float*>(workspace);
  float* part = reinterpret_cast<float*>(static_cast<char*>(workspace) +
                                         bppsa_align_up((size_t)rows * 4 * H * sizeof(float), 256));
  const long long nblk = (rows + kRows - 1) / kRows;
  if (nblk > 0x7fffffffLL) return BPPSA_EOVERFLOW;
  size_t lds = deltas_lds_bytes(H);
  if (H == 128) {
    const bppsa_status st = bppsa_gru_deltas_h128(rows, I, h, x, G, w_ih, w_hh, b_ih, b_hh, delta, stream);
    if (st != BPPSA_OK) return st;
  } else {
    if (lds > 48 * 1024)
      BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)gru_deltas_kernel,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    gru_deltas_kernel<<<(int)nblk, kThreads, lds, stream>>>(rows, H, I, h, x, G, w_ih, w_hh, b_ih, b_hh, delta);
    BPPSA_CHECK_LAUNCH();
  }

  const int ns = gru_splits(rows);
  long long rps = (rows + ns - 1) / ns;
  rps = (rps + kTileRows - 1) / kTileRows * kTileRows;
  dim3 grid(bppsa_ceil_div(3 * H, kGateTile), ns);
  lds = ((size_t)2 * kTileRows * kGateTile + (size_t)kTileRows * W) * sizeof(float);
  if (H == 128 && I <= 4) {
    const bppsa_status st = bppsa_gru_param_partials_h128(rows, I, ns, h, x, delta, part, stream);
    if (st != BPPSA_OK) return st;
  } else {
#define BPPSA_LAUNCH_GRU_PART(M)                                                         \
  gru_param_partials_kernel<M><<<grid, kThreads, lds, stream>>>(rows, H, I, (int)rps, h, x, delta, part)
  if (E <= 2 * kThreads) BPPSA_LAUNCH_GRU_PART(2);
  else if (E <= 8 * kThreads) BPPSA_LAUNCH_GRU_PART(8);
  else if (E <= 17 * kThreads) BPPSA_LAUNCH_GRU_PART(17);
  else BPPSA_LAUNCH_GRU_PART(32);
#undef BPPSA_LAUNCH_GRU_PART
    BPPSA_CHECK_LAUNCH();
  }
  const int Etot = 3 * H * W;
  gru_param_finish_kernel<<<bppsa_ceil_div(Etot, 4), kThreads, 0, stream>>>(ns, H, I, part, dW_ih, dW_hh, db_ih, db_hh);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
