// bppsa_build_jacobians: materialise Jt[t][b] = (d h[t+1] / d h[t])^T, the
// matrix entries of the scan's input array (Section 3.1, Eq. 5).
//
// RNN (Section 4.1): d h[t+1][j] / d h[t][i] = (1 - h[t+1][j]^2) W_hh[j][i], so
// the transposed Jacobian is W_hh^T with column j scaled by 1 - h[t+1][j]^2.
// The kernel is a pure streaming write (4 H^2 bytes out per 4 H bytes in), so
// each lane produces one 16-byte piece of a row and consecutive lanes write
// consecutive addresses; W_hh^T sits in LDS.
#include "bppsa_internal.h"

namespace {

template <int VEC>
__global__ void __launch_bounds__(256)
rnn_jacobians_kernel(long long n_vec, int B, int H,
                     const float* __restrict__ h, const float* __restrict__ w_hh,
                     float* __restrict__ Jt, int w_in_lds) {
  extern __shared__ float wt[];  // wt[i*H + j] = W_hh[j][i]
  if (w_in_lds) {
    for (int e = threadIdx.x; e < H * H; e += blockDim.x) {
      const int j = e / H, i = e - j * H;
      wt[i * H + j] = w_hh[e];
    }
    __syncthreads();
  }
  const int hv = H / VEC;            // vectors per row
  const long long mv = (long long)hv * H;  // vectors per matrix
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < n_vec; e += stride) {
    const long long m = e / mv;                 // matrix index t*B + b
    const int rem = (int)(e - m * mv);
    const int i = rem / hv;
    const int j = (rem - i * hv) * VEC;
    const float* hr = h + (size_t)(m + B) * H + j;  // h[t+1][b][j..]
    float out[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const float hj = hr[v];
      const float w = w_in_lds ? wt[i * H + j + v] : w_hh[(size_t)(j + v) * H + i];
      out[v] = w * (1.0f - hj * hj);
    }
    float* dst = Jt + (size_t)e * VEC;
    if (VEC == 4) {
      *reinterpret_cast<float4*>(dst) = make_float4(out[0], out[1], out[2], out[3]);
    } else {
#pragma unroll
      for (int v = 0; v < VEC; ++v) dst[v] = out[v];
    }
  }
}

// H = 20 (the paper's RNN size): a tile is 100 pieces of 16 bytes.  A thread keeps one fixed
// piece position (row i, columns j4..j4+3), so its four weights live in registers, and walks
// over tiles: per tile it reads 16 bytes of h, multiplies and issues one 16-byte store.
// 500 of the 512 threads of a workgroup cover five tiles per pass.
constexpr int kH20Threads = 512;
constexpr int kH20TilesPerPass = 5;

typedef float bj_v4f __attribute__((ext_vector_type(4)));

template <bool STREAM>
__global__ void __launch_bounds__(kH20Threads)
rnn_jacobians_h20_kernel(int tiles, int B, const float* __restrict__ h, const float* __restrict__ w_hh,
                         float* __restrict__ Jt) {
  constexpr int H = 20;
  const int tid = threadIdx.x;
  const int slot = tid / 100, p = tid - slot * 100;
  if (slot >= kH20TilesPerPass) return;
  const int i = p / 5, j4 = (p - i * 5) * 4;
  bj_v4f w;
#pragma unroll
  for (int u = 0; u < 4; ++u) w[u] = w_hh[(j4 + u) * H + i];
  const int step = gridDim.x * kH20TilesPerPass;
  // Eight tiles per trip: the eight 16-byte reads of h are issued before the first result is
  // formed, so a thread waits for memory once per eight stores instead of once per store.
  constexpr int kTrip = 8;
  for (int m0 = blockIdx.x * kH20TilesPerPass + slot; m0 < tiles; m0 += kTrip * step) {
    bj_v4f hv[kTrip];
#pragma unroll
    for (int u = 0; u < kTrip; ++u) {
      const int m = m0 + u * step;
      hv[u] = bj_v4f{0.f, 0.f, 0.f, 0.f};
      if (m < tiles) hv[u] = *reinterpret_cast<const bj_v4f*>(h + (size_t)(m + B) * H + j4);   // h[t+1][b][j4..]
    }
#pragma unroll
    for (int u = 0; u < kTrip; ++u) {
      const int m = m0 + u * step;
      if (m < tiles) {
        // 1 - h^2 as one fused multiply-add, spelled out: the fused scan forms the same tile and
        // must get the same bits whatever the compiler would contract
        bj_v4f o;
#pragma unroll
        for (int c = 0; c < 4; ++c) o[c] = w[c] * __builtin_fmaf(-hv[u][c], hv[u][c], 1.0f);
        bj_v4f* dst = reinterpret_cast<bj_v4f*>(Jt + (size_t)m * H * H + p * 4);
        if (STREAM) __builtin_nontemporal_store(o, dst);   // far larger than the caches: do not allocate
        else *dst = o;                                     // small enough to be read back from cache
      }
    }
  }
}

}  // namespace

bppsa_status bppsa_build_jacobians_gru(int T, int B, int H, int I,
                                       const float* h, const float* x,
                                       const float* w_ih, const float* w_hh,
                                       const float* b_ih, const float* b_hh,
                                       float* Jt, hipStream_t stream);

extern "C" bppsa_status bppsa_build_jacobians(int cell, int T, int B, int H, int I,
                                              const float* h, const float* x,
                                              const float* w_ih, const float* w_hh,
                                              const float* b_ih, const float* b_hh,
                                              float* Jt, void* stream) {
  if (!h || !w_hh || !Jt) return BPPSA_EINVAL;
  if (T < 1 || B < 1 || H < 1) return BPPSA_EINVAL;
  if (bppsa_mul_overflows(T, B, H, H)) return BPPSA_EOVERFLOW;
  hipStream_t s = (hipStream_t)stream;
  if (cell == BPPSA_GRU) {
    if (!x || !w_ih || I < 1) return BPPSA_EINVAL;
    return bppsa_build_jacobians_gru(T, B, H, I, h, x, w_ih, w_hh, b_ih, b_hh, Jt, s);
  }
  if (cell != BPPSA_RNN_TANH) return BPPSA_EUNSUPPORTED;

  if (H == 20 && (long long)T * B < 0x7fffffffLL - 65536) {
    const int tiles = T * B;
    int grid = bppsa_ceil_div(tiles, kH20TilesPerPass);
    if (grid > 512) grid = 512;
    if ((size_t)tiles * 1600 > ((size_t)128 << 20))
      rnn_jacobians_h20_kernel<true><<<grid, kH20Threads, 0, s>>>(tiles, B, h, w_hh, Jt);
    else
      rnn_jacobians_h20_kernel<false><<<grid, kH20Threads, 0, s>>>(tiles, B, h, w_hh, Jt);
    BPPSA_CHECK_LAUNCH();
    return BPPSA_OK;
  }
  const long long n_elem = (long long)T * B * H * H;
  const int w_in_lds = (size_t)H * H * sizeof(float) <= 64 * 1024;
  const size_t lds = w_in_lds ? (size_t)H * H * sizeof(float) : 0;
  const int vec = (H % 4 == 0) ? 4 : 1;
  const long long n_vec = n_elem / vec;
  long long blocks = (n_vec + 256 * 8 - 1) / (256 * 8);
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  if (vec == 4)
    rnn_jacobians_kernel<4><<<(int)blocks, 256, lds, s>>>(n_vec, B, H, h, w_hh, Jt, w_in_lds);
  else
    rnn_jacobians_kernel<1><<<(int)blocks, 256, lds, s>>>(n_vec, B, H, h, w_hh, Jt, w_in_lds);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
