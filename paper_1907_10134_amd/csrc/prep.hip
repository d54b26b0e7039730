// Workload preparation kernels: the forward recurrence that yields the hidden
// states, and the softmax cross-entropy head that yields the seed gradient.
// They run once per workload, outside the timed hot path, so they favour
// simplicity: one workgroup per sample walks the sequence.
#include "bppsa_internal.h"

// the GRU recurrence for H = 128 and at most 8 input features (weights in registers)
bppsa_status bppsa_gru_forward_h128(int T, int B, int I, const float* x, const float* w_ih, const float* w_hh,
                                    const float* b_ih, const float* b_hh, float* h, hipStream_t stream);

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

// The same recurrence for H = 20 and a few input features (the sizes of Section 4.1), where
// the walk over time is the whole cost of a training iteration's forward pass: one wave per
// sample, so no workgroup barrier is needed: lane j keeps row j of W_hh in registers, the state
// goes through LDS (one write, five broadcast reads per step), and the inputs of 64 steps are
// fetched at once.
constexpr int kFwdMaxI = 4;

// tanh for the walk over time, where it sits on the dependency chain of every step: an odd
// polynomial (the Maclaurin series to a^7) below 0.1, where 1 - 2 / (e^{2a} + 1) would cancel, and
// that expression above, on the hardware's base-2 exponential and reciprocal.  The absolute error
// stays near 1e-7, the relative error below 1e-6.
__device__ __forceinline__ float tanh_chain(float a) {
  const float t = fabsf(a);
  const float a2 = a * a;
  const float small = a * (1.0f + a2 * (-0.33333334f + a2 * (0.13333334f + a2 * -0.053968254f)));
  const float e = __builtin_amdgcn_exp2f(fminf(t, 20.0f) * 2.8853901f);      // e^{2t}
  const float big = copysignf(1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f), a);
  return t < 0.1f ? small : big;
}

__global__ void __launch_bounds__(64)
rnn_forward_h20_kernel(int T, int B, int I, const float* __restrict__ x, const float* __restrict__ w_ih,
                       const float* __restrict__ w_hh, const float* __restrict__ b_ih,
                       const float* __restrict__ b_hh, float* __restrict__ h) {
  constexpr int H = 20;
  typedef float f4 __attribute__((ext_vector_type(4)));
  __shared__ __attribute__((aligned(16))) float hs[2][H];   // the state, double-buffered
  const int b = blockIdx.x, lane = threadIdx.x;
  const int j = lane < H ? lane : H - 1;            // idle lanes mirror the last row
  f4 w[H / 4];
  float wi[kFwdMaxI];
#pragma unroll
  for (int i = 0; i < H / 4; ++i)
    w[i] = f4{w_hh[j * H + 4 * i], w_hh[j * H + 4 * i + 1], w_hh[j * H + 4 * i + 2], w_hh[j * H + 4 * i + 3]};
#pragma unroll
  for (int i = 0; i < kFwdMaxI; ++i) wi[i] = i < I ? w_ih[j * I + i] : 0.f;
  const float bias = (b_ih ? b_ih[j] : 0.f) + (b_hh ? b_hh[j] : 0.f);
  if (lane < H) hs[0][lane] = h[(size_t)b * H + lane];
  int cur = 0;
  for (int t0 = 0; t0 < T; t0 += 64) {
    float xs[kFwdMaxI];
#pragma unroll
    for (int i = 0; i < kFwdMaxI; ++i)
      xs[i] = (i < I && t0 + lane < T) ? x[((size_t)(t0 + lane) * B + b) * I + i] : 0.f;
    const int n = T - t0 < 64 ? T - t0 : 64;
    for (int s = 0; s < n; ++s) {
      // the 20 values of the state come back as five broadcast reads of 16 bytes; the writes of
      // the previous step are this wave's own and complete in order before them
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const f4* hv = reinterpret_cast<const f4*>(hs[cur]);
      f4 p[H / 4];
#pragma unroll
      for (int i = 0; i < H / 4; ++i) p[i] = hv[i];
      float a0 = bias, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
      for (int i = 0; i < kFwdMaxI; ++i)
        a1 += wi[i] * __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, xs[i]), s));
#pragma unroll
      for (int i = 0; i < H / 4; ++i) {
        a0 += w[i][0] * p[i][0];
        a1 += w[i][1] * p[i][1];
        a2 += w[i][2] * p[i][2];
        a3 += w[i][3] * p[i][3];
      }
      const float y = tanh_chain((a0 + a1) + (a2 + a3));
      cur ^= 1;
      if (lane < H) {
        hs[cur][lane] = y;
        h[((size_t)(t0 + s + 1) * B + b) * H + lane] = y;
      }
    }
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
    if (H == 20 && I <= kFwdMaxI) {
      rnn_forward_h20_kernel<<<B, 64, 0, s>>>(T, B, I, x, w_ih, w_hh, b_ih, b_hh, h);
    } else {
      const int nt = bppsa_ceil_div(H, 64) * 64;
      rnn_forward_kernel<<<B, nt, H * sizeof(float), s>>>(T, B, H, I, x, w_ih, w_hh, b_ih, b_hh, h);
    }
  } else if (cell == BPPSA_GRU) {
    if (3 * H > 1024) return BPPSA_ESHAPE;
    if (H == 128 && I <= 8) return bppsa_gru_forward_h128(T, B, I, x, w_ih, w_hh, b_ih, b_hh, h, s);
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
