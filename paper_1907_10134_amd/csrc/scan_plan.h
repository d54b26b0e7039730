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

bppsa_status bppsa_scan_generic(int T, int B, int H, const float* Jt, const float* seed,
                                float* G, float* g0, void* workspace, hipStream_t stream);
