// Host-side planning shared by the workspace query and the scan launcher.
#pragma once

#include "bppsa_internal.h"

// Segment length of the generic segmented scan.
static inline int bppsa_generic_segment(int H) {
  (void)H;
  return 64;
}

// Workspace of the generic scan: per recursion level, the chain of segment
// totals [nseg-1, B, H, H] and their incoming vectors [nseg-1, B, H].
static inline size_t bppsa_generic_scan_ws(int T, int B, int H, int want_g0) {
  size_t total = 0;
  int t_min = want_g0 ? 0 : 1;
  for (;;) {
    const int n = T - t_min;
    const int S = bppsa_generic_segment(H);
    if (n <= S) break;
    const int T2 = bppsa_ceil_div(n, S) - 1;
    total += bppsa_align_up((size_t)T2 * B * H * H * sizeof(float), 256);
    total += bppsa_align_up((size_t)T2 * B * H * sizeof(float), 256);
    T = T2;
    t_min = 1;
  }
  return total;
}

// ---- single-pass path for H = 20 --------------------------------------------------------
#define BPPSA_H20_SEGMENT 32
#define BPPSA_H20_AGG_STRIDE 416   /* floats: a 20x20 total padded to 13 cache lines */
#define BPPSA_H20_INC_STRIDE 32    /* floats: a 20-vector padded to one cache line */
#define BPPSA_H20_HEADER_BYTES 4096

// Workspace of the single-pass scan: header, one status word and one hop count per (unit,
// sample), one published total and one published inclusive vector per (unit, sample), and the
// transposed weights of the fused form.  Sized for units of one half (the larger case).
static inline size_t bppsa_h20_scan_ws(int T, int B) {
  const size_t nblk = (size_t)bppsa_ceil_div(T, BPPSA_H20_SEGMENT) * B;
  return BPPSA_H20_HEADER_BYTES + 2 * bppsa_align_up(nblk * sizeof(int), 256) +
         nblk * (BPPSA_H20_AGG_STRIDE + BPPSA_H20_INC_STRIDE) * sizeof(float) + 20 * 20 * sizeof(float);
}

// skip_dies (bit mask of compute dies whose workgroups stand aside) and unit_halves (0 = chosen
// from the sizes, 1 or 2 = forced) are 0 except in the diagnostic call.
bppsa_status bppsa_scan_h20(int T, int B, const float* Jt, const float* seed, float* G, float* g0,
                            void* workspace, hipStream_t stream, const float* h = nullptr,
                            const float* w_hh = nullptr, int skip_dies = 0, int unit_halves = 0);

bppsa_status bppsa_scan_h20_hops(int T, int B, int want_g0, int unit_halves, const void* workspace,
                                 long long* out, hipStream_t stream);

// GRU transposed Jacobians (H = 128) given by what generates them instead of as tiles: coef
// [T*B][4][H] = the per-step vectors (a, c, e, z) of Appendix E's closed form, wT [3][H][H] =
// W_hr^T, W_hn^T, W_hz^T.  With such a source the top level of the scan reads no Jt.
struct bppsa_gru_tiles {
  const float* coef;
  const float* wT;
};

bppsa_status bppsa_scan_generic(int T, int B, int H, const float* Jt, const float* seed,
                                float* G, float* g0, void* workspace, hipStream_t stream,
                                const bppsa_gru_tiles* gen = nullptr);

// ---- matrix-core kernels for H = 128 (used by the generic scan's reduce and apply steps) ----
bppsa_status bppsa_reduce_h128(int T, int B, int t_min, int S, int seg_begin, int seg_count,
                               const float* Jt, float* tot, hipStream_t s, const bppsa_gru_tiles* gen = nullptr);
// The same totals with the tiles generated (gen is not null); called by bppsa_reduce_h128.
bppsa_status bppsa_reduce_h128_gen(int T, int B, int t_min, int S, int seg_begin, int seg_count, float* tot,
                                   hipStream_t s, const bppsa_gru_tiles* gen);
bppsa_status bppsa_apply_h128(int T, int B, int t_min, int S, int seg_begin, int seg_count,
                              const float* Jt, const float* vin, int vin_is_seed, float* G, float* g0,
                              float* v_out, hipStream_t s, const bppsa_gru_tiles* gen = nullptr);

// coef and wT of bppsa_gru_tiles from the hidden states, inputs and weights (gates recomputed).
bppsa_status bppsa_gru_coefs_h128(long long rows, int I, const float* h, const float* x, const float* w_ih,
                                  const float* w_hh, const float* b_ih, const float* b_hh, float* coef,
                                  float* wT, hipStream_t stream);
