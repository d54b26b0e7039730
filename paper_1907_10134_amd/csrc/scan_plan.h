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

// H = 128: the slab of segments farthest from the seed may be cut into shorter segments (see
// bppsa_h128_plan); their totals and incoming vectors, at most this many, have room of their own.
#define BPPSA_H128_FINE_SEGMENTS 32
static inline size_t bppsa_h128_fine_ws(int T, int B, int want_g0) {
  if (T - (want_g0 ? 0 : 1) <= bppsa_generic_segment(128)) return 0;
  return bppsa_align_up((size_t)BPPSA_H128_FINE_SEGMENTS * B * 128 * 128 * sizeof(float), 256) +
         bppsa_align_up((size_t)BPPSA_H128_FINE_SEGMENTS * B * 128 * sizeof(float), 256);
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

// ---- schedule of a long H = 128 chain ---------------------------------------------------
// The chain is cut into segments of bppsa_generic_segment steps, counted from the far end (the
// last one, nearest the seed, may be shorter).  At this size a step of the matrix-matrix side
// costs 128 times the arithmetic of a matrix-vector step, so the hybrid schedule of Section 5.3
// is taken one step further: the `chain_segments` segments nearest the seed are walked by one
// serial matrix-vector chain per sample, on a compute unit of its own, while the totals of the
// other segments are formed on the matrix cores in slabs of `slab` segments; behind the chain and
// each slab's totals come the slab's matrix-vector passes.  chain_segments = 0: the two-level
// form without the serial chain (used when the batch alone fills the device); chain_segments =
// all segments: no matrix-matrix product at all.
#define BPPSA_H128_MAX_SLABS 32
struct bppsa_h128_plan {
  int chain_segments;
  int slab;
  int slabs;
  int last_steps;       // segment length inside the slab farthest from the seed (S, S/2 or S/4): a
                        // slab that would fill less than half of the device is cut finer, which
                        // shortens its products in proportion
  double model_us;      // the estimate the choice was made on
};

// One slab of the walk below the serial chain, shared by the cost model and the launcher:
// segments [lo, hi] of S steps, totals for [rlo, hi].
struct bppsa_h128_slab {
  int lo, hi, rlo;
};
static inline bppsa_h128_slab bppsa_h128_next_slab(int hi, int slab) {
  int lo = hi - slab + 1;
  if (lo <= 1) lo = 0;                        // segment 0 has no total: it rides with the last slab
  return bppsa_h128_slab{lo, hi, lo < 1 ? 1 : lo};
}

// The schedule of the cost model below, or the one the caller forces (force_chain >= 0; force_slab
// and force_last 0 = not forced).  Times in microseconds, measured on MI355X: a step of the serial
// chain (1024 threads, one compute unit per sample; bound by what one unit draws from memory, or
// by its vector ALUs when the Jacobians are generated), a step of a segment's running product on
// the matrix cores with the other units full, a step of the chain over a slab's totals, and the
// matrix-vector pass of a slab (HBM-bound on stored Jacobians, ALU-bound on generated ones).
static inline bppsa_h128_plan bppsa_plan_h128(int n, int B, int cus, bool generated, int force_chain = -1,
                                              int force_slab = 0, int force_last = 0) {
  const int S = bppsa_generic_segment(128);
  const int nseg = bppsa_ceil_div(n, S);
  bppsa_h128_plan best = {0, 0, 0, S, 0.0};
  if (cus < 2 * B || nseg < 2) return best;
  // the search below is O(segments x slabs): a training loop asks for the same sizes every
  // iteration, so each host thread remembers its last answer
  struct Memo {
    int n, B, cus, generated, force_chain, force_slab, force_last;
    bppsa_h128_plan plan;
  };
  static thread_local Memo memo = {-1, 0, 0, 0, 0, 0, 0, {0, 0, 0, 0, 0.0}};
  if (memo.n == n && memo.B == B && memo.cus == cus && memo.generated == (int)generated &&
      memo.force_chain == force_chain && memo.force_slab == force_slab && memo.force_last == force_last)
    return memo.plan;
  const double chain_step = generated ? 0.70 : 1.40, product_step = generated ? 8.8 : 8.3, totals_step = 1.2;
  const int top_steps = n - (nseg - 1) * S;
  const int free_units = cus - B;                       // the serial chains keep B units to themselves
  double best_us = 1e300;
  const int k_lo = force_chain >= 0 ? (force_chain < 1 ? 1 : force_chain > nseg ? nseg : force_chain) : 1;
  const int k_hi = force_chain >= 0 ? k_lo : nseg;
  for (int K = k_lo; K <= k_hi; ++K)
    for (int last = S; last >= S / 4; last /= 2) {
      if (K < nseg ? (force_last > 0 && last != force_last) : last != S) continue;   // no slab: nothing to cut
      double cur = (double)(top_steps + (K - 1) * S) * chain_step;
      int slab = 0, slabs = 0;
      bool valid = true;
      if (K < nseg) {
        const int R = nseg - K;                         // segments R-1 .. 0 lie below the chain
        slab = force_slab > 0 ? force_slab : free_units / B;
        if (slab < 1) slab = 1;
        if (bppsa_ceil_div(R, slab) > BPPSA_H128_MAX_SLABS) slab = bppsa_ceil_div(R, BPPSA_H128_MAX_SLABS);
        // first pass: when the totals of all slabs are done; second pass: the second stream
        double reduce_all = 0.0;
        for (int pass = 0; pass < 2 && valid; ++pass) {
          double reduce_end = 0.0;
          slabs = 0;
          for (int hi = R - 1; hi >= 0;) {
            const bppsa_h128_slab sl = bppsa_h128_next_slab(hi, slab);
            int steps = S, totals = sl.hi >= sl.rlo ? sl.hi - sl.rlo + 1 : 0, segs = sl.hi - sl.lo + 1;
            if (sl.lo == 0 && last < S) {               // the slab farthest from the seed, cut finer
              segs *= S / last;
              totals = segs - 1;
              steps = last;
              if (segs > BPPSA_H128_FINE_SEGMENTS) valid = false;
            }
            if (totals > 0) reduce_end += (steps - 1) * product_step * bppsa_ceil_div(totals * B, free_units);
            if (pass == 1) {
              double start = (cur > reduce_end ? cur : reduce_end) + totals * totals_step;
              // Beside the matrix-core kernel the matrix-vector pass on stored Jacobians gets a
              // fraction of its speed; the pass on generated ones (242 registers) does not fit on a
              // compute unit beside the totals kernel of that form (313) and waits for it.
              const bool beside = start < reduce_all;
              if (generated && beside) start = reduce_all;
              const double apply_us = generated ? steps * 1.1 * bppsa_ceil_div(segs * B, cus)
                                                : (double)segs * B * steps * (128.0 * 128.0 * 4.0) / 5.3e6 *
                                                      (beside ? 2.8 : 1.0);
              cur = start + apply_us;
            }
            ++slabs;
            hi = sl.lo - 1;
          }
          reduce_all = reduce_end;
        }
      }
      if (valid && cur < best_us) {
        best_us = cur;
        best = {K, slab, slabs, last, cur};
      }
    }
  memo = Memo{n, B, cus, (int)generated, force_chain, force_slab, force_last, best};
  return best;
}

// plan (H = 128 only): null = chosen by bppsa_plan_h128; otherwise the schedule to use
bppsa_status bppsa_scan_generic(int T, int B, int H, const float* Jt, const float* seed,
                                float* G, float* g0, void* workspace, hipStream_t stream,
                                const bppsa_gru_tiles* gen = nullptr, const bppsa_h128_plan* plan = nullptr);

// ---- matrix-core kernels for H = 128 (used by the generic scan's reduce and apply steps) ----
bppsa_status bppsa_reduce_h128(int T, int B, int t_min, int S, int seg_begin, int seg_count,
                               const float* Jt, float* tot, hipStream_t s, const bppsa_gru_tiles* gen = nullptr);
// The same totals with the tiles generated (gen is not null); called by bppsa_reduce_h128.
bppsa_status bppsa_reduce_h128_gen(int T, int B, int t_min, int S, int seg_begin, int seg_count, float* tot,
                                   hipStream_t s, const bppsa_gru_tiles* gen);
bppsa_status bppsa_apply_h128(int T, int B, int t_min, int S, int seg_begin, int seg_count,
                              const float* Jt, const float* vin, int vin_is_seed, float* G, float* g0,
                              float* v_out, hipStream_t s, const bppsa_gru_tiles* gen = nullptr);

// One serial chain per sample over steps hi..lo (seeded by seed [B, H]); g[t] goes to G[t-1] (g0 for
// t = 0, which must not be null if lo = 0), the last vector to v_out [B, H] if not null.
bppsa_status bppsa_chain_h128(int B, int lo, int hi, const float* Jt, const float* seed, float* G, float* g0,
                              float* v_out, hipStream_t s, const bppsa_gru_tiles* gen = nullptr);

// coef and wT of bppsa_gru_tiles from the hidden states, inputs and weights (gates recomputed).
bppsa_status bppsa_gru_coefs_h128(long long rows, int I, const float* h, const float* x, const float* w_ih,
                                  const float* w_hh, const float* b_ih, const float* b_hh, float* coef,
                                  float* wT, hipStream_t stream);
