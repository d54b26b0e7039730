// bppsa_scan entry point: validation, workspace accounting and kernel choice.
#include <mutex>

#include "bppsa_internal.h"
#include "scan_plan.h"

namespace {
constexpr int kMaxGenericH = 128;  // two H x H fp32 tiles must fit the 160 KB LDS

// Scratch of bppsa_scan_static: a fixed array inside the library's code object, so each GPU the
// library runs on holds its own copy until the process ends.  In host code the name is only a
// handle; the device address of the current GPU's copy comes from hipGetSymbolAddress.
constexpr size_t kStaticScratchBytes = BPPSA_SCAN_STATIC_SCRATCH_BYTES;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device; looked up once per device.
void* static_scratch() {
  constexpr int kMaxDevices = 64;
  static void* table[kMaxDevices];
  static std::mutex lock;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(lock);
  if (!table[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    table[dev] = ptr;
  }
  return table[dev];
}

size_t scan_ws_bytes(int T, int B, int H) {
  const size_t a = bppsa_generic_scan_ws(T, B, H, 0);
  const size_t b = bppsa_generic_scan_ws(T, B, H, 1);
  size_t need = (a > b ? a : b) + 256;
  if (H == 128) need += bppsa_h128_fine_ws(T, B, 1);
  if (H == 20) {
    const size_t c = bppsa_h20_scan_ws(T, B);
    if (c > need) need = c;
  }
  return need;
}
}  // namespace

extern "C" size_t bppsa_scan_workspace_bytes(int T, int B, int H) {
  if (T < 1 || B < 1 || H < 1 || H > kMaxGenericH) return 0;
  if (bppsa_mul_overflows(T, B, H, H)) return 0;
  return scan_ws_bytes(T, B, H);
}

extern "C" bppsa_status bppsa_scan(int T, int B, int H,
                                   const float* Jt, const float* seed,
                                   float* G, float* g0,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  if (T < 1 || B < 1 || H < 1) return BPPSA_EINVAL;
  if (!Jt || !seed || !G) return BPPSA_EINVAL;
  if (bppsa_mul_overflows(T, B, H, H)) return BPPSA_EOVERFLOW;
  if (B > 65535) return BPPSA_ESHAPE;            // batch rides on gridDim.y
  if (H > kMaxGenericH) return BPPSA_EUNSUPPORTED;
  const size_t need = scan_ws_bytes(T, B, H);
  if (need > 256 && (!workspace || workspace_bytes < need)) return BPPSA_EWORKSPACE;
  if (workspace && ((uintptr_t)workspace & 255)) return BPPSA_EINVAL;
  if (H == 20) return bppsa_scan_h20(T, B, Jt, seed, G, g0, workspace, (hipStream_t)stream);
  return bppsa_scan_generic(T, B, H, Jt, seed, G, g0, workspace, (hipStream_t)stream);
}

extern "C" bppsa_status bppsa_scan_h20_diag(int T, int B, const float* Jt, const float* seed, float* G, float* g0,
                                            void* workspace, size_t workspace_bytes, void* stream,
                                            int absent_dies, int unit_halves, int64_t* lookback_stats) {
  if (T < 1 || B < 1) return BPPSA_EINVAL;
  if (!Jt || !seed || !G) return BPPSA_EINVAL;
  if (bppsa_mul_overflows(T, B, 20, 20)) return BPPSA_EOVERFLOW;
  if (unit_halves < 0 || unit_halves > 2 || absent_dies < 0 || absent_dies > 0xff) return BPPSA_EINVAL;
  const size_t need = scan_ws_bytes(T, B, 20);
  if (!workspace || workspace_bytes < need) return BPPSA_EWORKSPACE;
  if ((uintptr_t)workspace & 255) return BPPSA_EINVAL;
  bppsa_status st = bppsa_scan_h20(T, B, Jt, seed, G, g0, workspace, (hipStream_t)stream, nullptr, nullptr,
                                   absent_dies, unit_halves);
  if (st != BPPSA_OK || !lookback_stats) return st;
  return bppsa_scan_h20_hops(T, B, g0 != nullptr, unit_halves, workspace,
                             reinterpret_cast<long long*>(lookback_stats), (hipStream_t)stream);
}

// Matrix-matrix products of the two-level form (every interior segment of every level reduced).
static long long two_level_products(int n, int B) {
  const int S = bppsa_generic_segment(128);
  long long total = 0;
  while (n > S) {
    const int nseg = bppsa_ceil_div(n, S);
    if (nseg > 2) total += (long long)(nseg - 2) * (S - 1) * B;
    n = nseg - 2;                                  // the chain of totals, its first element being the seed side
  }
  return total;
}

extern "C" bppsa_status bppsa_scan_h128_schedule(int T, int B, int want_g0, int generated,
                                                 bppsa_h128_schedule* out) {
  if (T < 1 || B < 1 || !out) return BPPSA_EINVAL;
  const int S = bppsa_generic_segment(128);
  const int n = T - (want_g0 ? 0 : 1);
  const int nseg = n > 0 ? bppsa_ceil_div(n, S) : 0;
  *out = bppsa_h128_schedule{};
  out->segment_steps = S;
  out->segments = nseg;
  if (n <= S) {                                    // one matrix-vector pass
    out->chain_steps = n > 0 ? n : 0;
    return BPPSA_OK;
  }
  const bppsa_h128_plan plan = bppsa_plan_h128(n, B, bppsa_compute_units(), generated != 0);
  const int top = n - (nseg - 1) * S;
  if (plan.chain_segments == 0) {
    out->chain_steps = top;
    out->matrix_products = two_level_products(n, B);
    return BPPSA_OK;
  }
  out->chain_steps = top + (plan.chain_segments - 1) * S;
  if (plan.chain_segments < nseg) {
    out->slab_segments = plan.slab;
    out->slabs = plan.slabs;
    out->last_slab_steps = plan.last_steps;
    // every segment below the chain but the farthest has a total; where the last slab is cut
    // finer, each of its segments of S steps becomes S / last_steps segments
    const int R = nseg - plan.chain_segments;
    long long products = 0;
    for (int hi = R - 1; hi >= 0;) {
      const bppsa_h128_slab sl = bppsa_h128_next_slab(hi, plan.slab);
      if (sl.lo == 0 && plan.last_steps < S)
        products += (long long)((sl.hi + 1) * (S / plan.last_steps) - 1) * (plan.last_steps - 1);
      else if (sl.hi >= sl.rlo)
        products += (long long)(sl.hi - sl.rlo + 1) * (S - 1);
      hi = sl.lo - 1;
    }
    out->matrix_products = products * B;
  }
  out->model_us = plan.model_us;
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_scan_h128_diag(int T, int B, const float* Jt, const float* seed, float* G, float* g0,
                                             void* workspace, size_t workspace_bytes, void* stream,
                                             int chain_segments, int slab_segments, int last_slab_steps) {
  if (T < 1 || B < 1 || chain_segments < 0 || slab_segments < 0) return BPPSA_EINVAL;
  if (last_slab_steps != 0 && last_slab_steps != 16 && last_slab_steps != 32 && last_slab_steps != 64)
    return BPPSA_EINVAL;
  if (!Jt || !seed || !G) return BPPSA_EINVAL;
  if (bppsa_mul_overflows(T, B, 128, 128)) return BPPSA_EOVERFLOW;
  if (B > 65535) return BPPSA_ESHAPE;
  const size_t need = scan_ws_bytes(T, B, 128);
  if (need > 256 && (!workspace || workspace_bytes < need)) return BPPSA_EWORKSPACE;
  if (workspace && ((uintptr_t)workspace & 255)) return BPPSA_EINVAL;
  const int n = T - (g0 ? 0 : 1);
  bppsa_h128_plan plan = {0, 0, 0, bppsa_generic_segment(128), 0.0};
  if (chain_segments > 0) {
    // the serial chain needs a compute unit per sample beside the matrix-core work
    if (bppsa_compute_units() < 2 * B) return BPPSA_EUNSUPPORTED;
    plan = bppsa_plan_h128(n, B, bppsa_compute_units(), false, chain_segments, slab_segments, last_slab_steps);
    if (plan.chain_segments == 0) return BPPSA_ESHAPE;   // no schedule of that kind fits these sizes
  }
  return bppsa_scan_generic(T, B, 128, Jt, seed, G, g0, workspace, (hipStream_t)stream, nullptr, &plan);
}

extern "C" bppsa_status bppsa_scan_static(int T, int B, int H, const float* Jt, const float* seed,
                                          float* G, float* g0, void* stream) {
  if (T < 1 || B < 1 || H < 1) return BPPSA_EINVAL;
  if (!Jt || !seed || !G) return BPPSA_EINVAL;
  if (bppsa_mul_overflows(T, B, H, H)) return BPPSA_EOVERFLOW;
  if (B > 65535) return BPPSA_ESHAPE;
  if (H > kMaxGenericH) return BPPSA_EUNSUPPORTED;
  if (scan_ws_bytes(T, B, H) > kStaticScratchBytes) return BPPSA_EWORKSPACE;   // beyond the fixed maximum
  void* ws = static_scratch();
  if (!ws) return BPPSA_EHIP;
  return bppsa_scan(T, B, H, Jt, seed, G, g0, ws, kStaticScratchBytes, stream);
}

extern "C" bppsa_status bppsa_rnn_scan_fused(int T, int B, int H, const float* h, const float* w_hh,
                                             const float* seed, float* G, float* g0, void* workspace,
                                             size_t workspace_bytes, void* stream) {
  if (T < 1 || B < 1 || H < 1) return BPPSA_EINVAL;
  if (!h || !w_hh || !seed || !G) return BPPSA_EINVAL;
  if (bppsa_mul_overflows(T, B, H, H)) return BPPSA_EOVERFLOW;
  if (H != 20) return BPPSA_EUNSUPPORTED;        // the single-pass kernel exists for this size only
  const size_t need = scan_ws_bytes(T, B, H);
  if (!workspace || workspace_bytes < need) return BPPSA_EWORKSPACE;
  if ((uintptr_t)workspace & 255) return BPPSA_EINVAL;
  return bppsa_scan_h20(T, B, nullptr, seed, G, g0, workspace, (hipStream_t)stream, h, w_hh);
}

// Layout of the fused GRU scan's workspace: coefficient vectors, transposed weights, then the
// workspace of the scan itself.
static size_t gru_fused_coef_bytes(int T, int B, int H) { return bppsa_align_up((size_t)T * B * 4 * H * sizeof(float), 256); }
static size_t gru_fused_wt_bytes(int H) { return bppsa_align_up((size_t)3 * H * H * sizeof(float), 256); }

extern "C" size_t bppsa_gru_scan_fused_workspace_bytes(int T, int B, int H) {
  if (T < 1 || B < 1 || H != 128) return 0;
  if (bppsa_mul_overflows(T, B, H, H)) return 0;
  return gru_fused_coef_bytes(T, B, H) + gru_fused_wt_bytes(H) + scan_ws_bytes(T, B, H);
}

extern "C" bppsa_status bppsa_gru_scan_fused(int T, int B, int H, int I, const float* h, const float* x,
                                             const float* w_ih, const float* w_hh, const float* b_ih,
                                             const float* b_hh, const float* seed, float* G, float* g0,
                                             void* workspace, size_t workspace_bytes, void* stream) {
  if (T < 1 || B < 1 || H < 1 || I < 1) return BPPSA_EINVAL;
  if (!h || !x || !w_ih || !w_hh || !seed || !G) return BPPSA_EINVAL;
  if (bppsa_mul_overflows(T, B, H, H)) return BPPSA_EOVERFLOW;
  if (B > 65535) return BPPSA_ESHAPE;
  if (H != 128) return BPPSA_EUNSUPPORTED;       // the generating kernels exist for this size only
  const size_t need = bppsa_gru_scan_fused_workspace_bytes(T, B, H);
  if (!workspace || workspace_bytes < need) return BPPSA_EWORKSPACE;
  if ((uintptr_t)workspace & 255) return BPPSA_EINVAL;
  char* ws = static_cast<char*>(workspace);
  float* coef = reinterpret_cast<float*>(ws);
  float* wT = reinterpret_cast<float*>(ws + gru_fused_coef_bytes(T, B, H));
  void* scan_ws = ws + gru_fused_coef_bytes(T, B, H) + gru_fused_wt_bytes(H);
  hipStream_t s = (hipStream_t)stream;
  BPPSA_TRY(bppsa_gru_coefs_h128((long long)T * B, I, h, x, w_ih, w_hh, b_ih, b_hh, coef, wT, s));
  const bppsa_gru_tiles gen{coef, wT};
  return bppsa_scan_generic(T, B, H, nullptr, seed, G, g0, scan_ws, s, &gen);
}
