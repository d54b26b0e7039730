// Generic (any H <= 128) segmented scan for bppsa_scan.
//
// The time axis is cut into segments of S steps.  This is the hybrid schedule
// the paper itself uses when n is much larger than the number of workers
// (Section 5.3: a truncated up-sweep, a scan of the partial results, then the
// down-sweep; Section 3.6: step complexity n/p + log p):
//   reduce : every interior segment multiplies its S transposed Jacobians into
//            one H x H total (the matrix-matrix side of the up-sweep);
//   top    : the segment that touches the seed only ever needs matrix-vector
//            products (Section 3.1: A may be a vector), so it is applied
//            directly and hands its last vector on as the next level's seed;
//   recurse: the totals form a shorter chain of the same kind - scan it;
//   apply  : every other segment walks its steps with matrix-vector products
//            from its incoming vector (the down-sweep side).
// Any bracketing gives the same gradients up to rounding (Section 3.5).
#include <mutex>

#include "bppsa_internal.h"
#include "scan_plan.h"

namespace {

constexpr int kThreads = 256;

// Segment `seg` covers time steps [lo, hi]; it consumes g[hi+1] and yields g[lo..hi].
__device__ __forceinline__ void seg_bounds(int T, int t_min, int S, int seg, int& lo, int& hi) {
  lo = t_min + seg * S;
  hi = min(lo + S, T) - 1;
}

// Total[seg][b] = Jt[lo] Jt[lo+1] ... Jt[hi], built by left-multiplying from hi down.
template <int MAXE>
__global__ void __launch_bounds__(kThreads)
reduce_segments_kernel(int T, int B, int H, int t_min, int S, int seg_begin,
                       const float* __restrict__ Jt, float* __restrict__ tot) {
  extern __shared__ float smem[];
  const int HH = H * H;
  float* P = smem;
  float* J = smem + HH;
  const int seg = seg_begin + blockIdx.x;
  const int b = blockIdx.y;
  int lo, hi;
  seg_bounds(T, t_min, S, seg, lo, hi);
  const float* src = Jt + ((size_t)hi * B + b) * HH;
  for (int e = threadIdx.x; e < HH; e += kThreads) P[e] = src[e];
  for (int t = hi - 1; t >= lo; --t) {
    src = Jt + ((size_t)t * B + b) * HH;
    for (int e = threadIdx.x; e < HH; e += kThreads) J[e] = src[e];
    __syncthreads();
    float acc[MAXE];
#pragma unroll
    for (int k = 0; k < MAXE; ++k) {
      const int e = threadIdx.x + k * kThreads;
      acc[k] = 0.f;
      if (e < HH) {
        const int i = e / H, j = e - i * H;
        float a = 0.f;
        for (int q = 0; q < H; ++q) a += J[i * H + q] * P[q * H + j];
        acc[k] = a;
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < MAXE; ++k) {
      const int e = threadIdx.x + k * kThreads;
      if (e < HH) P[e] = acc[k];
    }
    __syncthreads();
  }
  __syncthreads();
  float* dst = tot + ((size_t)seg * B + b) * HH;
  for (int e = threadIdx.x; e < HH; e += kThreads) dst[e] = P[e];
}

// v <- Jt[t] v for t = hi..lo, writing g[t] = v to G[t-1] (or g0 when t == 0).
// LPR lanes cooperate on one row; the wave reduces their partial sums.
__global__ void __launch_bounds__(kThreads)
apply_segments_kernel(int T, int B, int H, int t_min, int S, int seg_begin, int LPR,
                      const float* __restrict__ Jt,
                      const float* __restrict__ vin, int vin_is_seed,
                      float* __restrict__ G, float* __restrict__ g0,
                      float* __restrict__ v_out) {
  extern __shared__ float smem[];
  float* v0 = smem;
  float* v1 = smem + H;
  const int seg = seg_begin + blockIdx.x;
  const int b = blockIdx.y;
  int lo, hi;
  seg_bounds(T, t_min, S, seg, lo, hi);
  const float* vsrc = vin_is_seed ? vin + (size_t)b * H : vin + ((size_t)seg * B + b) * H;
  for (int e = threadIdx.x; e < H; e += kThreads) v0[e] = vsrc[e];
  __syncthreads();
  const int rows_per_pass = kThreads / LPR;
  const int r = threadIdx.x / LPR;
  const int l = threadIdx.x - r * LPR;
  for (int t = hi; t >= lo; --t) {
    const float* Jm = Jt + ((size_t)t * B + b) * H * H;
    float* dst = (t >= 1) ? G + ((size_t)(t - 1) * B + b) * H : g0 + (size_t)b * H;
    for (int i0 = 0; i0 < H; i0 += rows_per_pass) {
      const int i = i0 + r;
      float part = 0.f;
      if (i < H) {
        const float* row = Jm + (size_t)i * H;
        for (int j = l; j < H; j += LPR) part += row[j] * v0[j];
      }
      for (int m = LPR >> 1; m >= 1; m >>= 1) part += __shfl_xor(part, m);
      if (i < H && l == 0) {
        v1[i] = part;
        dst[i] = part;
      }
    }
    __syncthreads();
    float* tmp = v0; v0 = v1; v1 = tmp;
  }
  if (v_out) {
    float* d = v_out + (size_t)b * H;
    for (int e = threadIdx.x; e < H; e += kThreads) d[e] = v0[e];
  }
}

__global__ void copy_rows_kernel(long long n, const float* __restrict__ src, float* __restrict__ dst) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

int lanes_per_row(int H) {
  int cap = kThreads / H;
  if (cap < 1) cap = 1;
  if (cap > 64) cap = 64;
  int lpr = 1;
  while (lpr * 2 <= cap && lpr < H) lpr *= 2;
  return lpr;
}

// gen (H = 128 only): the matrices of this level are generated instead of read from Jt
bppsa_status launch_reduce(int T, int B, int H, int t_min, int S, int seg_begin, int seg_count,
                           const float* Jt, float* tot, hipStream_t s, const bppsa_gru_tiles* gen = nullptr) {
  if (seg_count <= 0) return BPPSA_OK;
  if (H == 128) return bppsa_reduce_h128(T, B, t_min, S, seg_begin, seg_count, Jt, tot, s, gen);
  if (gen) return BPPSA_EUNSUPPORTED;
  const size_t lds = (size_t)2 * H * H * sizeof(float);
  dim3 grid(seg_count, B);
  const int HH = H * H;
#define BPPSA_LAUNCH_REDUCE(E)                                                              \
  do {                                                                                      \
    if (lds > 48 * 1024)                                                                    \
      BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)reduce_segments_kernel<E>,             \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
    reduce_segments_kernel<E><<<grid, kThreads, lds, s>>>(T, B, H, t_min, S, seg_begin, Jt, tot); \
  } while (0)
  if (HH <= 2 * kThreads) BPPSA_LAUNCH_REDUCE(2);
  else if (HH <= 4 * kThreads) BPPSA_LAUNCH_REDUCE(4);
  else if (HH <= 16 * kThreads) BPPSA_LAUNCH_REDUCE(16);
  else BPPSA_LAUNCH_REDUCE(64);
#undef BPPSA_LAUNCH_REDUCE
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status launch_apply(int T, int B, int H, int t_min, int S, int seg_begin, int seg_count,
                          const float* Jt, const float* vin, int vin_is_seed,
                          float* G, float* g0, float* v_out, hipStream_t s, const bppsa_gru_tiles* gen = nullptr) {
  if (seg_count <= 0) return BPPSA_OK;
  if (H == 128)
    return bppsa_apply_h128(T, B, t_min, S, seg_begin, seg_count, Jt, vin, vin_is_seed, G, g0, v_out, s, gen);
  if (gen) return BPPSA_EUNSUPPORTED;
  dim3 grid(seg_count, B);
  apply_segments_kernel<<<grid, kThreads, (size_t)2 * H * sizeof(float), s>>>(
      T, B, H, t_min, S, seg_begin, lanes_per_row(H), Jt, vin, vin_is_seed, G, g0, v_out);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

// A second stream and the events that order it against the caller's stream; one set per
// device, created on first use and kept until the process ends.  `lock` is held while a call
// enqueues work that uses them, so that the records and waits of two host threads do not
// interleave.
constexpr int kMaxSlabs = BPPSA_H128_MAX_SLABS;
struct SideStream {
  hipStream_t stream;
  hipEvent_t fork, join, slab[kMaxSlabs];
  std::mutex lock;
};
SideStream* side_stream() {
  constexpr int kMaxDevices = 64;
  static SideStream table[kMaxDevices];
  static bool made[kMaxDevices];
  static std::mutex table_lock;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(table_lock);
  if (!made[dev]) {
    SideStream& st = table[dev];
    if (hipStreamCreateWithFlags(&st.stream, hipStreamNonBlocking) != hipSuccess) return nullptr;
    if (hipEventCreateWithFlags(&st.fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&st.join, hipEventDisableTiming) != hipSuccess)
      return nullptr;
    for (int i = 0; i < kMaxSlabs; ++i)
      if (hipEventCreateWithFlags(&st.slab[i], hipEventDisableTiming) != hipSuccess) return nullptr;
    made[dev] = true;
  }
  return &table[dev];
}

// H = 128, long chains: the schedule of bppsa_h128_plan.  A second stream walks the serial chain of
// the segments nearest the seed (one 1024-thread workgroup per sample, which has its compute unit
// to itself) while the caller's stream forms the totals of the segments below it on the matrix
// cores, slab by slab, nearest the seed first, a slab filling the other units once.  Behind the
// chain and behind each slab's totals the second stream runs the chain over the slab's totals,
// entered by the vector handed on from above, and then the slab's own matrix-vector pass (bound
// by HBM, or by the vector ALUs on generated Jacobians), which shares the units with the totals
// of the next slab: 242 + 148 registers per lane, 135 KB + 1 KB of LDS.
bppsa_status scan_h128_pipelined(int T, int B, int t_min, int S, int nseg, const float* Jt, const float* seed,
                                 float* G, float* g0, float* tot, float* vin, float* fine_tot, float* fine_vin,
                                 hipStream_t s, SideStream* side, const bppsa_h128_plan& plan,
                                 const bppsa_gru_tiles* gen) {
  constexpr int H = 128;
  const size_t row = (size_t)B * H;
  const int R = nseg - plan.chain_segments;       // segments R-1 .. 0 lie below the serial chain
  std::lock_guard<std::mutex> hold(side->lock);
  hipStream_t s2 = side->stream;
  BPPSA_HIP_TRY(hipEventRecord(side->fork, s));
  BPPSA_HIP_TRY(hipStreamWaitEvent(s2, side->fork, 0));
  // From here on the second stream carries work of this call, so every way out - an error
  // included - goes through the join below: the caller's stream waits for whatever was enqueued
  // on the second stream (and a capturing stream gets its fork joined) before the status returns.
  bppsa_status st = [&]() -> bppsa_status {
    // the serial chain; its last vector enters segment R-1
    bppsa_status e = bppsa_chain_h128(B, t_min + R * S, T - 1, Jt, seed, G, g0, vin + (size_t)(R - 1) * row, s2, gen);
    if (e != BPPSA_OK) return e;
    int j = 0;
    for (int hi = R - 1; hi >= 0; ++j) {
      if (j >= kMaxSlabs) return BPPSA_EINVAL;
      const bppsa_h128_slab sl = bppsa_h128_next_slab(hi, plan.slab);
      // this slab's own view of its stretch of the chain: segments [lo, top] of `steps` steps counted
      // from t_min, totals and incoming vectors in `stot` and `svin` (indexed by segment), the
      // vector entering segment `top` already in svin[top]
      int steps = S, lo = sl.lo, rlo = sl.rlo, top = sl.hi;
      float *stot = tot, *svin = vin;
      if (sl.lo == 0 && plan.last_steps < S) {
        // the slab farthest from the seed, cut into shorter segments with room of their own
        const int f = S / plan.last_steps;
        steps = plan.last_steps;
        top = (sl.hi + 1) * f - 1;
        rlo = 1;
        stot = fine_tot;
        svin = fine_vin;
        if (top + 1 > BPPSA_H128_FINE_SEGMENTS) return BPPSA_EINVAL;
      }
      if (top >= rlo) {
        e = launch_reduce(t_min + (top + 1) * steps, B, H, t_min, steps, rlo, top - rlo + 1, Jt, stot, s, gen);
        if (e != BPPSA_OK) return e;
      }
      BPPSA_HIP_TRY(hipEventRecord(side->slab[j], s));
      BPPSA_HIP_TRY(hipStreamWaitEvent(s2, side->slab[j], 0));
      if (svin != vin) {
        copy_rows_kernel<<<(int)((row + 255) / 256), 256, 0, s2>>>((long long)row, vin + (size_t)sl.hi * row,
                                                                   svin + (size_t)top * row);
        BPPSA_CHECK_LAUNCH();
      }
      if (top >= rlo) {
        // svin[seg-1] = stot[seg] svin[seg] for seg = top .. rlo: the totals as a chain of
        // top-rlo+1 steps, entered by svin[top]; also gives the next slab its entering vector
        // (on the compute units the serial chain has left: beside the matrix-core kernel a
        // 256-thread workgroup would take 6 to 10 us per step)
        e = bppsa_chain_h128(B, rlo, top, stot, svin + (size_t)top * row, svin, nullptr, nullptr, s2, nullptr);
        if (e != BPPSA_OK) return e;
      }
      e = launch_apply(svin == vin ? T : t_min + (top + 1) * steps, B, H, t_min, steps, lo, top - lo + 1, Jt, svin, 0, G,
                       g0, nullptr, s2, gen);
      if (e != BPPSA_OK) return e;
      hi = sl.lo - 1;
    }
    return BPPSA_OK;
  }();
  const bool joined = hipEventRecord(side->join, s2) == hipSuccess &&
                      hipStreamWaitEvent(s, side->join, 0) == hipSuccess;
  if (st != BPPSA_OK) return st;
  return joined ? BPPSA_OK : BPPSA_EHIP;
}

// One level of the recursion; `ws` is the unused tail of the workspace.
bppsa_status scan_level(int T, int B, int H, const float* Jt, const float* seed,
                        float* G, float* g0, char* ws, hipStream_t s, const bppsa_gru_tiles* gen = nullptr,
                        const bppsa_h128_plan* forced = nullptr) {
  const size_t row = (size_t)B * H;
  if (seed != G + (size_t)(T - 1) * row) {
    const long long n = (long long)row;
    copy_rows_kernel<<<(int)((n + 255) / 256), 256, 0, s>>>(n, seed, G + (size_t)(T - 1) * row);
    BPPSA_CHECK_LAUNCH();
  }
  const int t_min = g0 ? 0 : 1;
  const int n = T - t_min;
  if (n <= 0) return BPPSA_OK;
  const int S = bppsa_generic_segment(H);
  if (n <= S) return launch_apply(T, B, H, t_min, n, 0, 1, Jt, seed, 1, G, g0, nullptr, s, gen);

  const int nseg = bppsa_ceil_div(n, S);
  const int T2 = nseg - 1;                               // length of the chain of totals
  float* tot = reinterpret_cast<float*>(ws);
  ws += bppsa_align_up((size_t)T2 * row * H * sizeof(float), 256);
  float* vin = reinterpret_cast<float*>(ws);
  ws += bppsa_align_up((size_t)T2 * row * sizeof(float), 256);

  bppsa_status st;
  if (H == 128) {
    const bppsa_h128_plan plan = forced ? *forced : bppsa_plan_h128(n, B, bppsa_compute_units(), gen != nullptr);
    if (plan.chain_segments >= nseg) return bppsa_chain_h128(B, t_min, T - 1, Jt, seed, G, g0, nullptr, s, gen);
    if (plan.chain_segments >= 1) {
      SideStream* side = side_stream();
      if (side) {
        float* fine_tot = reinterpret_cast<float*>(ws);
        float* fine_vin = reinterpret_cast<float*>(
            ws + bppsa_align_up((size_t)BPPSA_H128_FINE_SEGMENTS * row * H * sizeof(float), 256));
        return scan_h128_pipelined(T, B, t_min, S, nseg, Jt, seed, G, g0, tot, vin, fine_tot, fine_vin, s, side, plan,
                                   gen);
      }
    }
  }
  // interior segments 1..nseg-2: matrix-matrix totals (segment 0's total reaches no output)
  st = launch_reduce(T, B, H, t_min, S, 1, nseg - 2, Jt, tot, s, gen);
  if (st != BPPSA_OK) return st;
  // seed-side segment: matrix-vector only; its last vector seeds the chain of totals
  st = launch_apply(T, B, H, t_min, S, nseg - 1, 1, Jt, seed, 1, G, g0, vin + (size_t)(T2 - 1) * row, s, gen);
  if (st != BPPSA_OK) return st;
  // incoming vectors of segments 0..nseg-2 = scan over the totals
  st = scan_level(T2, B, H, tot, vin + (size_t)(T2 - 1) * row, vin, nullptr, ws, s);
  if (st != BPPSA_OK) return st;
  return launch_apply(T, B, H, t_min, S, 0, nseg - 1, Jt, vin, 0, G, g0, nullptr, s, gen);
}

}  // namespace

bppsa_status bppsa_scan_generic(int T, int B, int H, const float* Jt, const float* seed,
                                float* G, float* g0, void* workspace, hipStream_t stream,
                                const bppsa_gru_tiles* gen, const bppsa_h128_plan* plan) {
  if ((gen || plan) && H != 128) return BPPSA_EUNSUPPORTED;
  return scan_level(T, B, H, Jt, seed, G, g0, static_cast<char*>(workspace), stream, gen, plan);
}
