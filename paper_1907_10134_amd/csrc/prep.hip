// Workload preparation kernels: the forward recurrence that yields the hidden
// states, and the softmax cross-entropy head that yields the seed gradient.
// They run once per workload, outside the timed hot path, so they favour
// simplicity: one workgroup per sample walks the sequence.
#include "bppsa_internal.h"

namespace {

__device__ __forceinline__ float sigmoidf_(float a) { return 1.0f / (1.0f + expf(-a)); }

// RNN (Section 4.1): h[t] = tanh(W_ih x[t-1] + b_ih + W_hh h[t-1] + b_hh).
__global__ void rnn_forward_kernel(int T, int B, int H, int I,
                                   const float* __restrict__ x,
                                   const float* __restrict__ w_ih,
                                   const float* __restrict__ w_hh,
                                   const float* __restrict__ b_ih,
                                   const float* __restrict__ b_hh,
                                   float* __restrict__ h) {
  extern __shared__ float smem[];
  float* hs = smem;  // [H]
  const int b = blockIdx.x;
  const int j = threadIdx.x;
  const bool active = j < H;
  if (active) hs[j] = h[(size_t)b * H + j];
  float bias = 0.f;
  if (active) bias = (b_ih ? b_ih[j] : 0.f) + (b_hh ? b_hh[j] : 0.f);
  __syncthreads();
  for (int t = 1; t <= T; ++t) {
    float hn = 0.f;
    if (active) {
      float acc = bias;
      const float* xr = x + ((size_t)(t - 1) * B + b) * I;
      for (int i = 0; i < I; ++i) acc += w_ih[(size_t)j * I + i] * xr[i];
      const float* wr = w_hh + (size_t)j * H;
      for (int i = 0; i < H; ++i) acc += wr[i] * hs[i];
      hn = tanhf(acc);
    }
    __syncthreads();
    if (active) {
      hs[j] = hn;
      h[((size_t)t * B + b) * H + j] = hn;
    }
    __syncthreads();
  }
}

// GRU (Section 4.2), gate rows ordered r, z, n.
__global__ void gru_forward_kernel(int T, int B, int H, int I,
                                   const float* __restrict__ x,
                                   const float* __restrict__ w_ih,
                                   const float* __restrict__ w_hh,
                                   const float* __restrict__ b_ih,
                                   const float* __restrict__ b_hh,
                                   float* __restrict__ h) {
  extern __shared__ float smem[];
  float* hs = smem;           // [H]
  float* gi = smem + H;       // [3H]
  float* gh = gi + 3 * H;     // [3H]
  const int b = blockIdx.x;
  const int j = threadIdx.x;
  const int R = 3 * H;
  if (j < H) hs[j] = h[(size_t)b * H + j];
  __syncthreads();
  for (int t = 1; t <= T; ++t) {
    if (j < R) {
      float ai = b_ih ? b_ih[j] : 0.f;
      const float* xr = x + ((size_t)(t - 1) * B + b) * I;
      for (int i = 0; i < I; ++i) ai += w_ih[(size_t)j * I + i] * xr[i];
      float ah = b_hh ? b_hh[j] : 0.f;
      const float* wr = w_hh + (size_t)j * H;
      for (int i = 0; i < H; ++i) ah += wr[i] * hs[i];
      gi[j] = ai;
      gh[j] = ah;
    }
    __syncthreads();
    float hn = 0.f;
    if (j < H) {
      const float r = sigmoidf_(gi[j] + gh[j]);
      const float z = sigmoidf_(gi[H + j] + gh[H + j]);
      const float n = tanhf(gi[2 * H + j] + r * gh[2 * H + j]);
      hn = (1.f - z) * n + z * hs[j];
    }
    __syncthreads();
    if (j < H) {
      hs[j] = hn;
      h[((size_t)t * B + b) * H + j] = hn;
    }
    __syncthreads();
  }
}

// One workgroup of 64 lanes walks the batch: logits, log-sum-exp, seed.
__global__ void head_seed_kernel(int B, int H, int C,
                                 const float* __restrict__ h_last,
                                 const float* __restrict__ w_out,
                                 const float* __restrict__ b_out,
                                 const int32_t* __restrict__ labels,
                                 float* __restrict__ seed, float* __restrict__ loss) {
  __shared__ float z[64];
  __shared__ float p[64];
  const int c = threadIdx.x;
  float total = 0.f;
  const float invB = 1.0f / (float)B;
  for (int b = 0; b < B; ++b) {
    const float* hr = h_last + (size_t)b * H;
    if (c < C) {
      float acc = b_out[c];
      for (int j = 0; j < H; ++j) acc += w_out[(size_t)c * H + j] * hr[j];
      z[c] = acc;
    }
    __syncthreads();
    if (c == 0) {
      float m = z[0];
      for (int k = 1; k < C; ++k) m = fmaxf(m, z[k]);
      float s = 0.f;
      for (int k = 0; k < C; ++k) s += expf(z[k] - m);
      const float lse = m + logf(s);
      const int y = labels[b];
      total += lse - z[y];
      for (int k = 0; k < C; ++k) p[k] = (expf(z[k] - lse) - (k == y ? 1.f : 0.f)) * invB;
    }
    __syncthreads();
    for (int j = c; j < H; j += blockDim.x) {
      float acc = 0.f;
      for (int k = 0; k < C; ++k) acc += p[k] * w_out[(size_t)k * H + j];
      seed[(size_t)b * H + j] = acc;
    }
    __syncthreads();
  }
  if (c == 0 && loss) *loss = total * invB;
}

}  // namespace

extern "C" bppsa_status bppsa_forward(int cell, int T, int B, int H, int I,
                                      const float* x, const float* w_ih, const float* w_hh,
                                      const float* b_ih, const float* b_hh,
                                      float* h, void* stream) {
  if (!x || !w_ih || !w_hh || !h) return BPPSA_EINVAL;
  if (T < 1 || B < 1 || H < 1 || I < 1) return BPPSA_EINVAL;
  if (bppsa_mul_overflows((int64_t)T + 1, B, H, 1) || bppsa_mul_overflows(T, B, I, 1))
    return BPPSA_EOVERFLOW;
  hipStream_t s = (hipStream_t)stream;
  if (cell == BPPSA_RNN_TANH) {
    if (H > 1024) return BPPSA_ESHAPE;
    const int nt = bppsa_ceil_div(H, 64) * 64;
    rnn_forward_kernel<<<B, nt, H * sizeof(float), s>>>(T, B, H, I, x, w_ih, w_hh, b_ih, b_hh, h);
  } else if (cell == BPPSA_GRU) {
    if (3 * H > 1024) return BPPSA_ESHAPE;
    const int nt = bppsa_ceil_div(3 * H, 64) * 64;
    gru_forward_kernel<<<B, nt, 7 * H * sizeof(float), s>>>(T, B, H, I, x, w_ih, w_hh, b_ih, b_hh, h);
  } else {
    return BPPSA_EUNSUPPORTED;
  }
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_head_seed(int B, int H, int C,
                                        const float* h_last, const float* w_out,
                                        const float* b_out, const int32_t* labels,
                                        float* seed, float* loss, void* stream) {
  if (!h_last || !w_out || !b_out || !labels || !seed) return BPPSA_EINVAL;
  if (B < 1 || H < 1 || C < 1) return BPPSA_EINVAL;
  if (C > 64) return BPPSA_ESHAPE;
  head_seed_kernel<<<1, 64, 0, (hipStream_t)stream>>>(B, H, C, h_last, w_out, b_out, labels, seed, loss);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
