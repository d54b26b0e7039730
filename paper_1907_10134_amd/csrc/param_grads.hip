// bppsa_param_grads: Eq. 2 of Section 2.1 summed over the time steps that share
// the parameters.  Once dL/dh[t] is known for every t the terms are independent,
// so the sum is one tall-skinny contraction over the T*B (step, sample) rows:
//     [dW_hh | dW_ih | db] = sum_rows  delta_row (x) [h_prev_row | x_row | 1],
// with delta[t] = (1 - h[t]^2) o dL/dh[t] for the tanh RNN (Section 4.1).
// It reads each of G, h and x once (HBM bound).  Blocks reduce disjoint row
// ranges into fp32 partials; a second kernel adds the partials in a fixed order.
#include "bppsa_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kTileRows = 32;
constexpr int kMaxBlocks = 512;

template <int MAXE>
__global__ void __launch_bounds__(kThreads)
rnn_param_partials_kernel(long long rows, int B, int H, int I, int rows_per_block,
                          const float* __restrict__ h, const float* __restrict__ x,
                          const float* __restrict__ G, float* __restrict__ part) {
  extern __shared__ float smem[];
  const int W = H + I + 1;             // columns of the right-hand rows [h_prev | x | 1]
  float* D = smem;                     // [kTileRows][H]   delta
  float* U = smem + kTileRows * H;     // [kTileRows][W]
  const int E = H * W;
  const long long r_begin = (long long)blockIdx.x * rows_per_block;
  long long r_end = r_begin + rows_per_block;
  if (r_end > rows) r_end = rows;
  const float* hcur = h + (size_t)B * H;   // row r of hcur is h[t][b], r = (t-1)*B + b
  float acc[MAXE];
#pragma unroll
  for (int k = 0; k < MAXE; ++k) acc[k] = 0.f;

  for (long long r0 = r_begin; r0 < r_end; r0 += kTileRows) {
    const int nr = (int)((r_end - r0 < kTileRows) ? (r_end - r0) : kTileRows);
    for (int e = threadIdx.x; e < nr * H; e += kThreads) {
      const size_t g = (size_t)r0 * H + e;
      const float hc = hcur[g];
      D[e] = (1.0f - hc * hc) * G[g];
    }
    for (int e = threadIdx.x; e < nr * W; e += kThreads) {
      const int rr = e / W, c = e - rr * W;
      float u;
      if (c < H) u = h[(size_t)(r0 + rr) * H + c];
      else if (c < H + I) u = x[(size_t)(r0 + rr) * I + (c - H)];
      else u = 1.0f;
      U[e] = u;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < MAXE; ++k) {
      const int e = threadIdx.x + k * kThreads;
      if (e < E) {
        const int i = e / W, c = e - i * W;
        float a = acc[k];
        for (int rr = 0; rr < nr; ++rr) a += D[rr * H + i] * U[rr * W + c];
        acc[k] = a;
      }
    }
    __syncthreads();
  }
  float* dst = part + (size_t)blockIdx.x * E;
#pragma unroll
  for (int k = 0; k < MAXE; ++k) {
    const int e = threadIdx.x + k * kThreads;
    if (e < E) dst[e] = acc[k];
  }
}

// One wave per output element: lanes add the per-block partials in a fixed
// strided order, then the wave reduces (deterministic).
__global__ void __launch_bounds__(256)
rnn_param_finish_kernel(int nblocks, int H, int I, const float* __restrict__ part,
                        float* __restrict__ dW_ih, float* __restrict__ dW_hh,
                        float* __restrict__ db_ih, float* __restrict__ db_hh) {
  const int W = H + I + 1;
  const int E = H * W;
  const int lane = threadIdx.x & 63;
  const int e = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (e >= E) return;                       // whole wave leaves together
  float s = 0.f;
  for (int k = lane; k < nblocks; k += 64) s += part[(size_t)k * E + e];
  for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m);
  if (lane != 0) return;
  const int i = e / W, c = e - i * W;
  if (c < H) dW_hh[(size_t)i * H + c] = s;
  else if (c < H + I) dW_ih[(size_t)i * I + (c - H)] = s;
  else {
    db_ih[i] = s;
    if (db_hh) db_hh[i] = s;
  }
}

int rnn_blocks(long long rows) {
  long long nb = (rows + kTileRows - 1) / kTileRows;
  if (nb > kMaxBlocks) nb = kMaxBlocks;
  return (int)nb;
}

}  // namespace

size_t bppsa_param_grads_gru_ws(int T, int B, int H, int I);
bppsa_status bppsa_param_grads_gru(int T, int B, int H, int I,
                                   const float* h, const float* x, const float* G,
                                   const float* w_ih, const float* w_hh,
                                   const float* b_ih, const float* b_hh,
                                   float* dW_ih, float* dW_hh, float* db_ih, float* db_hh,
                                   void* workspace, size_t workspace_bytes, hipStream_t stream);

extern "C" size_t bppsa_param_grads_workspace_bytes(int cell, int T, int B, int H, int I) {
  if (T < 1 || B < 1 || H < 1 || I < 1) return 0;
  if (cell == BPPSA_GRU) return bppsa_param_grads_gru_ws(T, B, H, I);
  if (cell != BPPSA_RNN_TANH) return 0;
  const long long rows = (long long)T * B;
  return bppsa_align_up((size_t)rnn_blocks(rows) * H * (H + I + 1) * sizeof(float), 256);
}

extern "C" bppsa_status bppsa_param_grads(int cell, int T, int B, int H, int I,
                                          const float* h, const float* x, const float* G,
                                          const float* w_ih, const float* w_hh,
                                          const float* b_ih, const float* b_hh,
                                          float* dW_ih, float* dW_hh,
                                          float* db_ih, float* db_hh,
                                          void* workspace, size_t workspace_bytes,
                                          void* stream) {
  if (T < 1 || B < 1 || H < 1 || I < 1) return BPPSA_EINVAL;
  if (!h || !x || !G || !dW_ih || !dW_hh || !db_ih) return BPPSA_EINVAL;
  if (bppsa_mul_overflows((int64_t)T + 1, B, H, 1) || bppsa_mul_overflows(T, B, I, 1))
    return BPPSA_EOVERFLOW;
  hipStream_t s = (hipStream_t)stream;
  if (cell == BPPSA_GRU) {
    if (!w_ih || !w_hh || !db_hh) return BPPSA_EINVAL;
    return bppsa_param_grads_gru(T, B, H, I, h, x, G, w_ih, w_hh, b_ih, b_hh,
                                 dW_ih, dW_hh, db_ih, db_hh, workspace, workspace_bytes, s);
  }
  if (cell != BPPSA_RNN_TANH) return BPPSA_EUNSUPPORTED;
  const int W = H + I + 1;
  const int E = H * W;
  if (E > 64 * kThreads) return BPPSA_EUNSUPPORTED;
  const size_t lds = (size_t)kTileRows * (H + W) * sizeof(float);
  if (lds > 64 * 1024) return BPPSA_EUNSUPPORTED;
  const long long rows = (long long)T * B;
  const int nb = rnn_blocks(rows);
  const size_t need = bppsa_align_up((size_t)nb * E * sizeof(float), 256);
  if (!workspace || workspace_bytes < need) return BPPSA_EWORKSPACE;
  long long rpb = (rows + nb - 1) / nb;
  rpb = (rpb + kTileRows - 1) / kTileRows * kTileRows;
  float* part = static_cast<float*>(workspace);
#define BPPSA_LAUNCH_PARTIALS(M)                                                     \
  rnn_param_partials_kernel<M><<<nb, kThreads, lds, s>>>(rows, B, H, I, (int)rpb, h, x, G, part)
  if (E <= 2 * kThreads) BPPSA_LAUNCH_PARTIALS(2);
  else if (E <= 8 * kThreads) BPPSA_LAUNCH_PARTIALS(8);
  else if (E <= 32 * kThreads) BPPSA_LAUNCH_PARTIALS(32);
  else BPPSA_LAUNCH_PARTIALS(64);
#undef BPPSA_LAUNCH_PARTIALS
  BPPSA_CHECK_LAUNCH();
  // blocks past the last row range wrote zeros, so summing all nb partials is exact
  rnn_param_finish_kernel<<<bppsa_ceil_div(E, 4), 256, 0, s>>>(nb, H, I, part, dW_ih, dW_hh, db_ih, db_hh);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
