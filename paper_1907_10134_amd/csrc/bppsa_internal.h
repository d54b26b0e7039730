// Internal helpers shared by the HIP translation units of libbppsa (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "bppsa.h"

#define BPPSA_WAVE 64

// Returns BPPSA_EHIP from the enclosing function if the last launch failed.
#define BPPSA_CHECK_LAUNCH()                                  \
  do {                                                        \
    if (hipGetLastError() != hipSuccess) return BPPSA_EHIP;   \
  } while (0)

#define BPPSA_TRY(expr)                                       \
  do {                                                        \
    const bppsa_status st__ = (expr);                         \
    if (st__ != BPPSA_OK) return st__;                        \
  } while (0)

#define BPPSA_HIP_TRY(expr)                                   \
  do {                                                        \
    if ((expr) != hipSuccess) return BPPSA_EHIP;              \
  } while (0)

static inline size_t bppsa_align_up(size_t n, size_t a) { return (n + a - 1) / a * a; }

static inline int bppsa_ceil_div(int a, int b) { return (a + b - 1) / b; }

// A product of sizes that must fit a signed 64-bit element count and whose
// per-array element count must stay below 2^40 (far above 288 GB of fp32).
static inline bool bppsa_mul_overflows(int64_t a, int64_t b, int64_t c, int64_t d) {
  const int64_t lim = (int64_t)1 << 40;
  if (a <= 0 || b <= 0 || c <= 0 || d <= 0) return true;
  if (a > lim / b) return true;
  int64_t ab = a * b;
  if (ab > lim / c) return true;
  int64_t abc = ab * c;
  if (abc > lim / d) return true;
  return false;
}

// Compute units of the current device (256 on an MI355X); queried from the runtime on every
// call, so nothing is remembered across devices.  Falls back to 256 if the query fails.
static inline int bppsa_compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  return cus;
}
