// One training iteration of the tanh RNN of Section 4.1 on a mini-batch, as one call: forward
// recurrence, softmax cross-entropy head, the backward pass as a scan (Section 3.1) with its
// parameter gradients (Eq. 2), and an Adam update of every parameter (learning rate 1e-5 in the
// paper's runs).  The call only chains the library's own entry points on the caller's stream and
// adds the two kernels they lack: the head's parameter gradients and the optimiser step.
#include <cmath>

#include "bppsa_internal.h"

namespace {

// Softmax cross-entropy head with all its gradients.  One workgroup; wave w takes samples w,
// w + nwaves, ...: logits, log-sum-exp and the per-sample dL/dz (kept in LDS) with wave
// reductions, and the seed dL/dh_T = dz W_out.  After a barrier the parameter gradients
// dW_out = dz^T h_T and db_out = sum_b dz are summed over the batch in index order by one thread
// per entry, so they are the same bits on every run.
constexpr int kHeadThreads = 1024;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__global__ void __launch_bounds__(kHeadThreads)
head_backward_kernel(int B, int H, int C, const float* __restrict__ h_last, const float* __restrict__ w_out,
                     const float* __restrict__ b_out, const int32_t* __restrict__ labels,
                     float* __restrict__ seed, float* __restrict__ loss, float* __restrict__ dW_out,
                     float* __restrict__ db_out) {
  extern __shared__ float lds[];
  float* dz = lds;                  // [B][C]
  float* lb = lds + (size_t)B * C;  // [B] per-sample loss
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const float invB = 1.0f / (float)B;
  for (int b = wave; b < B; b += nwaves) {
    const float* hr = h_last + (size_t)b * H;
    float z = -INFINITY;
    if (lane < C) {
      float acc = b_out[lane];
      for (int j = 0; j < H; ++j) acc += w_out[(size_t)lane * H + j] * hr[j];
      z = acc;
    }
    const float m = wave_max(z);
    const float s = wave_sum(lane < C ? expf(z - m) : 0.f);
    const float lse = m + logf(s);
    const int y = labels[b];
    float p = 0.f;
    if (lane < C) {
      p = (expf(z - lse) - (lane == y ? 1.f : 0.f)) * invB;
      dz[(size_t)b * C + lane] = p;
    }
    const float zy = __shfl(z, y, 64);
    if (lane == 0) lb[b] = lse - zy;
    for (int j0 = 0; j0 < H; j0 += 64) {            // every lane takes part in the lane reads
      const int j = j0 + lane;
      float acc = 0.f;
      for (int k = 0; k < C; ++k) acc += __shfl(p, k, 64) * (j < H ? w_out[(size_t)k * H + j] : 0.f);
      if (j < H) seed[(size_t)b * H + j] = acc;
    }
  }
  __syncthreads();
  if (dW_out) {
    for (int e = threadIdx.x; e < C * H; e += blockDim.x) {
      const int c = e / H, j = e - c * H;
      float acc = 0.f;
      for (int b = 0; b < B; ++b) acc += dz[(size_t)b * C + c] * h_last[(size_t)b * H + j];
      dW_out[e] = acc;
    }
  }
  if (db_out && threadIdx.x < C) {
    float acc = 0.f;
    for (int b = 0; b < B; ++b) acc += dz[(size_t)b * C + threadIdx.x];
    db_out[threadIdx.x] = acc;
  }
  if (loss && threadIdx.x == 0) {
    float acc = 0.f;
    for (int b = 0; b < B; ++b) acc += lb[b];
    *loss = acc * invB;
  }
}

// Adam (Kingma & Ba, Algorithm 1).  1 - beta and the bias corrections c1 = 1 / (1 - beta1^t),
// c2 = 1 / (1 - beta2^t) are formed on the host in double precision and rounded once.
__global__ void __launch_bounds__(256)
adam_kernel(int n, float* __restrict__ theta, const float* __restrict__ g, float* __restrict__ m,
            float* __restrict__ v, float lr, float beta1, float one_minus_beta1, float beta2,
            float one_minus_beta2, float eps, float c1, float c2) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float gi = g[i];
  const float mi = beta1 * m[i] + one_minus_beta1 * gi;
  const float vi = beta2 * v[i] + one_minus_beta2 * gi * gi;
  m[i] = mi;
  v[i] = vi;
  theta[i] -= lr * (mi * c1) / (sqrtf(vi * c2) + eps);
}

}  // namespace

extern "C" bppsa_status bppsa_head_backward(int B, int H, int C, const float* h_last, const float* w_out,
                                            const float* b_out, const int32_t* labels, float* seed, float* loss,
                                            float* dW_out, float* db_out, void* stream) {
  if (!h_last || !w_out || !b_out || !labels || !seed) return BPPSA_EINVAL;
  if (B < 1 || H < 1 || C < 1) return BPPSA_EINVAL;
  if (C > 64) return BPPSA_ESHAPE;
  const size_t lds = ((size_t)B * C + (size_t)B) * sizeof(float);
  if (lds > 48 * 1024) return BPPSA_ESHAPE;
  head_backward_kernel<<<1, kHeadThreads, lds, (hipStream_t)stream>>>(B, H, C, h_last, w_out, b_out, labels, seed,
                                                                      loss, dW_out, db_out);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_adam_step(int64_t n, float* theta, const float* grad, float* m, float* v, int step,
                                        double lr, double beta1, double beta2, double eps, void* stream) {
  if (!theta || !grad || !m || !v) return BPPSA_EINVAL;
  if (n < 1 || step < 1 || n > INT32_MAX - 256) return BPPSA_EINVAL;
  if (!(beta1 >= 0. && beta1 < 1.) || !(beta2 >= 0. && beta2 < 1.)) return BPPSA_EINVAL;
  const float c1 = (float)(1.0 / (1.0 - std::pow(beta1, (double)step)));
  const float c2 = (float)(1.0 / (1.0 - std::pow(beta2, (double)step)));
  adam_kernel<<<bppsa_ceil_div((int)n, 256), 256, 0, (hipStream_t)stream>>>(
      (int)n, theta, grad, m, v, (float)lr, (float)beta1, (float)(1.0 - beta1), (float)beta2, (float)(1.0 - beta2),
      (float)eps, c1, c2);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" size_t bppsa_rnn_param_count(int H, int I, int C) {
  if (H < 1 || I < 1 || C < 1) return 0;
  return (size_t)H * I + (size_t)H * H + 2 * (size_t)H + (size_t)C * H + (size_t)C;
}

// The scan's part comes first and stays untouched by the later calls, so its error word (the
// first four bytes, H = 20) can still be read after the iteration.
static size_t train_scan_ws_bytes(int T, int B, int H) { return bppsa_align_up(bppsa_scan_workspace_bytes(T, B, H), 256); }

extern "C" size_t bppsa_rnn_train_workspace_bytes(int T, int B, int H, int I) {
  return train_scan_ws_bytes(T, B, H) + bppsa_param_grads_workspace_bytes(BPPSA_RNN_TANH, T, B, H, I);
}

extern "C" bppsa_status bppsa_rnn_train_step(int T, int B, int H, int I, int C, const float* x,
                                             const int32_t* labels, const bppsa_rnn_train_state* st, int step,
                                             double lr, double beta1, double beta2, double eps, void* stream) {
  if (!x || !labels || !st) return BPPSA_EINVAL;
  if (!st->params || !st->grads || !st->adam_m || !st->adam_v || !st->h || !st->G || !st->seed || !st->workspace)
    return BPPSA_EINVAL;
  if (T < 1 || B < 1 || H < 1 || I < 1 || C < 1 || step < 1) return BPPSA_EINVAL;
  if (st->workspace_bytes < bppsa_rnn_train_workspace_bytes(T, B, H, I)) return BPPSA_EWORKSPACE;
  // the flat layout: W_ih | W_hh | b_ih | b_hh | W_out | b_out
  const size_t o_whh = (size_t)H * I, o_bih = o_whh + (size_t)H * H, o_bhh = o_bih + H, o_wout = o_bhh + H,
               o_bout = o_wout + (size_t)C * H;
  const float* p = st->params;
  float* g = st->grads;
  const size_t scan_bytes = train_scan_ws_bytes(T, B, H);
  void* pg_ws = static_cast<char*>(st->workspace) + scan_bytes;
  const size_t pg_bytes = st->workspace_bytes - scan_bytes;
  BPPSA_TRY(bppsa_forward(BPPSA_RNN_TANH, T, B, H, I, x, p, p + o_whh, p + o_bih, p + o_bhh, st->h, stream));
  BPPSA_TRY(bppsa_head_backward(B, H, C, st->h + (size_t)T * B * H, p + o_wout, p + o_bout, labels, st->seed,
                                st->loss, g + o_wout, g + o_bout, stream));
  // the backward pass over the T steps as a scan; the seed is dL/dh_T (Eq. 5)
  if (st->Jt) {
    BPPSA_TRY(bppsa_build_jacobians(BPPSA_RNN_TANH, T, B, H, I, st->h, nullptr, nullptr, p + o_whh, nullptr,
                                    nullptr, st->Jt, stream));
    BPPSA_TRY(bppsa_scan(T, B, H, st->Jt, st->seed, st->G, nullptr, st->workspace, scan_bytes, stream));
  } else {
    BPPSA_TRY(bppsa_rnn_scan_fused(T, B, H, st->h, p + o_whh, st->seed, st->G, nullptr, st->workspace, scan_bytes,
                                   stream));
  }
  BPPSA_TRY(bppsa_param_grads(BPPSA_RNN_TANH, T, B, H, I, st->h, x, st->G, nullptr, nullptr, nullptr, nullptr, g,
                              g + o_whh, g + o_bih, g + o_bhh, pg_ws, pg_bytes, stream));
  return bppsa_adam_step((int64_t)bppsa_rnn_param_count(H, I, C), st->params, st->grads, st->adam_m, st->adam_v,
                         step, lr, beta1, beta2, eps, stream);
}
