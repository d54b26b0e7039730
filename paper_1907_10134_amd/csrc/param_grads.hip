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
constexpr int kMaxBlocks = 1024;

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


// H = 20 (the paper's RNN size), up to 3 inputs: the same contraction on the matrix cores.
// The 20 x W output (W = 20 + I + 1 <= 24) is 5 x 6 blocks of 4 x 4; v_mfma_f32_4x4x1 handles 16
// blocks per issue, so two issues per (step, sample) row accumulate all of it:
// D_blk[i][j] += delta[row][4 I + i] * u[row][4 J + j], lane (blk, idx) supplying both operands
// from a tile staged in LDS.  Each wave takes every fourth row of a tile and keeps its own
// accumulators; the four waves' sums are added in a fixed order at the end.
typedef float pg_v4f __attribute__((ext_vector_type(4)));
constexpr int kMfmaRows = 64;     // rows per staged tile
constexpr int kUW = 24;           // padded width of [h_prev | x | 1 | 0]

__global__ void __launch_bounds__(kThreads)
rnn_param_partials_h20_kernel(long long rows, int B, int I, int rows_per_block,
                              const float* __restrict__ h, const float* __restrict__ x,
                              const float* __restrict__ G, float* __restrict__ part) {
  constexpr int H = 20;
  __shared__ __attribute__((aligned(16))) float D[kMfmaRows * H];
  __shared__ __attribute__((aligned(16))) float U[kMfmaRows * kUW];
  __shared__ float red[4][H * kUW];
  const int W = H + I + 1;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, blk = lane >> 2, idx = lane & 3;
  const long long r_begin = (long long)blockIdx.x * rows_per_block;
  long long r_end = r_begin + rows_per_block;
  if (r_end > rows) r_end = rows;
  const float* hcur = h + (size_t)B * H;          // row r of hcur is h[t][b], r = (t-1)*B + b
  // operand offsets of this lane for the two issues (block ids blk and 16 + blk; ids 30, 31 idle)
  int aoff[2], boff[2];
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    int id = 16 * n + blk;
    id = id < 30 ? id : 29;
    aoff[n] = 4 * (id / 6) + idx;
    boff[n] = 4 * (id % 6) + idx;
  }
  pg_v4f acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  for (long long r0 = r_begin; r0 < r_end; r0 += kMfmaRows) {
    const int nr = (int)((r_end - r0 < kMfmaRows) ? (r_end - r0) : kMfmaRows);
    // delta and h_prev in 16-byte pieces (5 per row), x and the constant column one by one
    for (int e = tid; e < nr * 5; e += kThreads) {
      const int rr = e / 5, c4 = (e - rr * 5) * 4;
      const size_t g = (size_t)(r0 + rr) * H + c4;
      const pg_v4f hc = *reinterpret_cast<const pg_v4f*>(hcur + g);
      const pg_v4f gv = *reinterpret_cast<const pg_v4f*>(G + g);
      *reinterpret_cast<pg_v4f*>(D + rr * H + c4) = (1.0f - hc * hc) * gv;
      *reinterpret_cast<pg_v4f*>(U + rr * kUW + c4) = *reinterpret_cast<const pg_v4f*>(h + g);
    }
    for (int e = tid; e < nr * 4; e += kThreads) {
      const int rr = e >> 2, c = e & 3;
      float u = 0.f;
      if (c < I) u = x[(size_t)(r0 + rr) * I + c];
      else if (c == I) u = 1.0f;
      U[rr * kUW + H + c] = u;
    }
    __syncthreads();
    for (int rr = wave; rr < nr; rr += 4) {
      const float a0 = D[rr * H + aoff[0]], b0 = U[rr * kUW + boff[0]];
      const float a1 = D[rr * H + aoff[1]], b1 = U[rr * kUW + boff[1]];
      acc[0] = __builtin_amdgcn_mfma_f32_4x4x1f32(a0, b0, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_4x4x1f32(a1, b1, acc[1], 0, 0, 0);
    }
    __syncthreads();
  }
  // accumulator register v of lane (blk, idx) is element (4 I + v, 4 J + idx) of its block
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    const int id = 16 * n + blk;
    if (id < 30) {
      const int bi = id / 6, bj = id % 6;
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][(4 * bi + v) * kUW + 4 * bj + idx] = acc[n][v];
    }
  }
  __syncthreads();
  float* dst = part + (size_t)blockIdx.x * H * W;
  for (int e = tid; e < H * W; e += kThreads) {
    const int i = e / W, c = e - i * W;
    const int o = i * kUW + c;
    dst[e] = (red[0][o] + red[1][o]) + (red[2][o] + red[3][o]);
  }
}

// Adds the per-block partials in a fixed order (deterministic).  A workgroup owns 64 consecutive
// output elements; its sixteen waves each add every sixteenth block's partial for them -
// consecutive lanes read consecutive addresses, sixteen independent loads in flight per thread -
// and the sixteen sums are added in wave order.
constexpr int kFinishWaves = 16;
__global__ void __launch_bounds__(64 * kFinishWaves)
rnn_param_finish_kernel(int nblocks, int H, int I, const float* __restrict__ part,
                        float* __restrict__ dW_ih, float* __restrict__ dW_hh,
                        float* __restrict__ db_ih, float* __restrict__ db_hh) {
  __shared__ float red[kFinishWaves][64];
  const int W = H + I + 1;
  const int E = H * W;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (e < E) {
    for (int k0 = wave; k0 < nblocks; k0 += 16 * kFinishWaves) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int k = k0 + u * kFinishWaves;
        v[u] = k < nblocks ? part[(size_t)k * E + e] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) s += v[u];
    }
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave != 0 || e >= E) return;
  float t = red[0][lane];
#pragma unroll
  for (int w = 1; w < kFinishWaves; ++w) t += red[w][lane];
  const int i = e / W, c = e - i * W;
  if (c < H) dW_hh[(size_t)i * H + c] = t;
  else if (c < H + I) dW_ih[(size_t)i * I + (c - H)] = t;
  else {
    db_ih[i] = t;
    if (db_hh) db_hh[i] = t;
  }
}

int rnn_blocks(long long rows) {
  long long nb = (rows + 2 * kTileRows - 1) / (2 * kTileRows);
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
  if (H == 20 && I <= 3) {
    long long rpb64 = (rows + nb - 1) / nb;
    rpb64 = (rpb64 + kMfmaRows - 1) / kMfmaRows * kMfmaRows;
    rnn_param_partials_h20_kernel<<<nb, kThreads, 0, s>>>(rows, B, I, (int)rpb64, h, x, G, part);
  } else {
#define BPPSA_LAUNCH_PARTIALS(M)                                                     \
  rnn_param_partials_kernel<M><<<nb, kThreads, lds, s>>>(rows, B, H, I, (int)rpb, h, x, G, part)
  if (E <= 2 * kThreads) BPPSA_LAUNCH_PARTIALS(2);
  else if (E <= 8 * kThreads) BPPSA_LAUNCH_PARTIALS(8);
  else if (E <= 32 * kThreads) BPPSA_LAUNCH_PARTIALS(32);
  else BPPSA_LAUNCH_PARTIALS(64);
#undef BPPSA_LAUNCH_PARTIALS
  }
  BPPSA_CHECK_LAUNCH();
  // blocks past the last row range wrote zeros, so summing all nb partials is exact
  rnn_param_finish_kernel<<<bppsa_ceil_div(E, 64), 64 * kFinishWaves, 0, s>>>(nb, H, I, part, dW_ih, dW_hh, db_ih, db_hh);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
