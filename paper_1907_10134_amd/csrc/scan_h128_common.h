// Shared by the H = 128 kernels: tile constants, segment bounds, and the pieces of a GRU transposed
// Jacobian generated from per-step coefficient vectors (Appendix E) instead of read from memory.
#pragma once

#include "bppsa_internal.h"
#include "scan_plan.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int H = 128;
constexpr int HH = H * H;
constexpr int LS = H + 4;            // LDS row stride in floats: rows 8 apart share a bank, so the
                                     // 16-byte reads of 8 consecutive rows tile all 32 banks
constexpr int kThreads = 256;
constexpr int kChunks = HH / 4 / kThreads;   // 16-byte pieces of a tile per thread (16)

__device__ __forceinline__ void seg_bounds(int T, int t_min, int S, int seg, int& lo, int& hi) {
  lo = t_min + seg * S;
  hi = min(lo + S, T) - 1;
}

// GRU transposed Jacobians generated in place of being read (Appendix E):
//   Jt[i][j] = W_hr[j][i] a_j + W_hn[j][i] c_j + W_hz[j][i] e_j + [i == j] z_j
// with the per-step coefficient vectors (a, c, e, z) of bppsa_gru_coefs_h128 and the three
// recurrent matrices transposed, wT[g][i][j] (g = r, n, z).  The 256-thread kernels give thread
// tid the 16-byte pieces e = tid + 256 q of a tile, i.e. rows tid / 32 + 8 q and columns
// 4 (tid % 32) .. + 3: the same places in every tile, so the thread keeps its 3 x 16 pieces of
// the weights in registers for the whole segment.  Where the tile itself is needed (the A
// operand of a matrix-matrix step) it costs the thread four coefficient reads and 192
// multiply-adds instead of 256 bytes from HBM; where only its product with a vector is needed,
// the three weight matrices are applied to the vector scaled by a, c and e and no tile is formed.
struct GruWeights {
  v4f r[kChunks], n[kChunks], z[kChunks];
};
struct GruCoef {
  v4f a, c, e, z;
};

__device__ __forceinline__ void load_gru_weights(const float* __restrict__ wT, int tid, GruWeights& w) {
#pragma unroll
  for (int q = 0; q < kChunks; ++q) {
    const int e = tid + q * kThreads;
    w.r[q] = reinterpret_cast<const v4f*>(wT)[e];
    w.n[q] = reinterpret_cast<const v4f*>(wT + HH)[e];
    w.z[q] = reinterpret_cast<const v4f*>(wT + 2 * HH)[e];
  }
}
__device__ __forceinline__ GruCoef load_gru_coef(const float* __restrict__ coef, size_t row, int tid) {
  const v4f* c = reinterpret_cast<const v4f*>(coef + row * 4 * H) + (tid & 31);
  return GruCoef{c[0], c[H / 4], c[2 * (H / 4)], c[3 * (H / 4)]};
}
__device__ __forceinline__ v4f gru_piece(const GruWeights& w, const GruCoef& cf, int tid, int q) {
  v4f o = w.r[q] * cf.a + w.n[q] * cf.c + w.z[q] * cf.e;
  const int d = (tid >> 5) + 8 * q - 4 * (tid & 31);      // row minus first column of the piece
#pragma unroll
  for (int u = 0; u < 4; ++u) o[u] += (d == u) ? cf.z[u] : 0.f;
  return o;
}

}  // namespace
