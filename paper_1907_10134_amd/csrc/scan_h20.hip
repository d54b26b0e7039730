// Single-pass scan for H = 20 (the paper's RNN size, Section 4.1): every
// transposed Jacobian is read from HBM exactly once.
//
// One workgroup owns a segment of S = 32 consecutive chain elements of one
// sample and keeps it in LDS (32 x 1600 B) from load to store:
//   up-sweep   : Algorithm 1's up-sweep on the 32 tiles, in place.  The 31
//                matrix-matrix products run on the matrix cores as 4x4x1 fp32
//                MFMA outer products (20 = 5 x 4, so a 20x20 tile is 25 blocks
//                of 4x4 with no padding);
//   cross-block: instead of one launch per level over the segment totals, the
//                workgroup publishes its total, looks back over its
//                predecessors' published totals / inclusive vectors
//                (matrix-vector products only, since everything to the left
//                ends in the gradient vector, Section 3.1) and publishes its
//                own inclusive vector.  Segment ids are handed out by an atomic
//                ticket, so a workgroup only ever waits for workgroups that are
//                already running;
//   down-sweep : Algorithm 1's down-sweep (reversed operands, matrix-vector
//                only) from the incoming vector, then the 32 gradients are
//                stored.
// The chain runs from the seed end: element c is Jt[T-1-c]; the vector that
// enters element c is g[T-c] = G[T-1-c].
#include <stdlib.h>

#include "bppsa_internal.h"
#include "scan_plan.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int H = 20;
constexpr int HH = 400;
constexpr int PS = 2 * HH + 4;           // LDS stride of a pair of tiles in floats: two tiles back to back
                                        // plus one 16-byte pad.  Level 0 reads the same element of 16
                                        // even (or 16 odd) tiles at once; with this stride the tiles of
                                        // eight consecutive pairs start four banks apart, so those reads
                                        // spread over all 32 banks instead of hitting four of them
constexpr int S = BPPSA_H20_SEGMENT;
// offset of tile p of a segment in LDS
__device__ __forceinline__ constexpr int toff(int p) { return (p >> 1) * PS + (p & 1) * HH; }
constexpr int kThreads = 256;
constexpr int kAggStride = BPPSA_H20_AGG_STRIDE;   // floats per published total (1664 B = 13 lines)
constexpr int kIncStride = BPPSA_H20_INC_STRIDE;   // floats per published vector (128 B)
constexpr unsigned kSpinLimit = 1u << 20;

enum : int { kNone = 0, kTotalReady = 1, kPrefixReady = 2 };

#ifdef BPPSA_TRACE
__device__ long long* g_trace;
#define BPPSA_LB_TRACE(slot, val) do { if (g_trace && (threadIdx.x & 63) == 0) g_trace[((size_t)k * B + b) * 16 + (slot)] = (val); } while (0)
#else
#define BPPSA_LB_TRACE(slot, val) do { } while (0)
#endif

constexpr int kMaxQueues = 8;     // one work queue per compute die (XCD)
constexpr int kHeaderBytes = BPPSA_H20_HEADER_BYTES;

struct Header {          // first kHeaderBytes of the workspace, zeroed before every scan
  int error;             // set when a bounded wait expired: results are invalid
  int pad[31];
  int ticket[kMaxQueues][32];   // next segment of each queue, one cache line apart
  // workgroups that have started, per die (slot kMaxQueues: bystanders of the test hook),
  // one cache line apart
  int started[kMaxQueues + 1][32];
};
static_assert(sizeof(Header) <= kHeaderBytes, "header does not fit");

__device__ __forceinline__ v4f mfma4(float a, float b, v4f c) {
  return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 0);
}

// ---- level 0: 16 products, one per MFMA block (slot); each wave owns a sub-grid of the
// 5 x 5 output blocks of every product.  C = A B with A = tile 2s+1, B = tile 2s.
template <int I0, int NI, int J0, int NJ>
__device__ __forceinline__ void level0_compute(const float* A, const float* Bm, int q, v4f (&acc)[9]) {
#pragma unroll
  for (int e = 0; e < NI * NJ; ++e) acc[e] = v4f{0.f, 0.f, 0.f, 0.f};
  // operands of step k4 + 1 are requested from LDS before the MFMAs of step k4 are issued
  v4f a[2][NI];
  float bv[2][NJ][4];
  auto fetch = [&](int buf, int k4) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
      a[buf][i] = *reinterpret_cast<const v4f*>(A + (4 * (I0 + i) + q) * H + 4 * k4);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) bv[buf][j][kk] = Bm[(4 * k4 + kk) * H + 4 * (J0 + j) + q];
  };
  fetch(0, 0);
#pragma unroll
  for (int k4 = 0; k4 < 5; ++k4) {
    const int cur = k4 & 1;
    if (k4 < 4) fetch(cur ^ 1, k4 + 1);
    __builtin_amdgcn_sched_barrier(0);     // keep the prefetch ahead of this step's MFMAs
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i * NJ + j] = mfma4(a[cur][i][kk], bv[cur][j][kk], acc[i * NJ + j]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int I0, int NI, int J0, int NJ>
__device__ __forceinline__ void level0_store(float* C, int q, const v4f (&acc)[9]) {
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) C[(4 * (I0 + i) + v) * H + 4 * (J0 + j) + q] = acc[i * NJ + j][v];
}

// ---- upper levels: one product per wave; 15 of the 16 MFMA blocks each own a row-block I
// and up to two column-blocks (2jp, 2jp+1).  C overwrites A; only this wave touches A and B.
__device__ __forceinline__ void wave_product(float* A, const float* Bm, int slot, int q) {
  const int s = slot < 15 ? slot : 14;
  const int I = s / 3, jp = s - I * 3;
  const int J0 = 2 * jp, J1 = (jp < 2) ? J0 + 1 : J0;
  v4f c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
  // all 45 operand loads are issued up front (60 registers), then the 40 MFMAs run back to back
  v4f a[5];
  float b0[5][4], b1[5][4];
#pragma unroll
  for (int k4 = 0; k4 < 5; ++k4) {
    a[k4] = *reinterpret_cast<const v4f*>(A + (4 * I + q) * H + 4 * k4);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      b0[k4][kk] = Bm[(4 * k4 + kk) * H + 4 * J0 + q];
      b1[k4][kk] = Bm[(4 * k4 + kk) * H + 4 * J1 + q];
    }
  }
  __builtin_amdgcn_sched_barrier(0);       // do not sink the loads between the MFMAs
#pragma unroll
  for (int k4 = 0; k4 < 5; ++k4) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      c0 = mfma4(a[k4][kk], b0[k4][kk], c0);
      c1 = mfma4(a[k4][kk], b1[k4][kk], c1);
    }
  }
  // every load above has been consumed by an MFMA, and LDS operations of one wave complete
  // in order, so the stores below cannot overtake this wave's reads of A
  if (slot < 15) {
#pragma unroll
    for (int v = 0; v < 4; ++v) A[(4 * I + v) * H + 4 * J0 + q] = c0[v];
    if (jp < 2) {
#pragma unroll
      for (int v = 0; v < 4; ++v) A[(4 * I + v) * H + 4 * J1 + q] = c1[v];
    }
  }
}

// y[row] = sum_k M[row][k] x[k], M a 20x20 tile in LDS, x 20 floats in LDS.
// Four partial sums over k mod 4, combined as (s0 + s1) + (s2 + s3): exactly the arithmetic
// of a look-back hop, so a segment's inclusive vector has the same bits whether its owner
// forms it from LDS or a successor forms it from the published total.  That makes the
// scan's output independent of how far each look-back happened to reach.
__device__ __forceinline__ float row_dot(const float* M, int row, const float* x) {
  const v4f* m4 = reinterpret_cast<const v4f*>(M + row * H);
  const v4f* x4 = reinterpret_cast<const v4f*>(x);
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
  for (int k4 = 0; k4 < 5; ++k4) {
    const v4f m = m4[k4], xv = x4[k4];
    a0 += m[0] * xv[0];
    a1 += m[1] * xv[1];
    a2 += m[2] * xv[2];
    a3 += m[3] * xv[3];
  }
  return (a0 + a1) + (a2 + a3);
}

// Value of `x` in lane `l` (l wave-uniform), as a wave-uniform scalar.
__device__ __forceinline__ float readlane_f(float x, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), l));
}

// Cross-workgroup traffic (status words, published totals and vectors) uses relaxed atomic
// accesses only, so no cache write-back or invalidate is ever issued; ordering comes from
// waiting for the data stores to complete before the status store is issued, and from
// issuing the data loads only after the status value has been observed.
// SCOPE is the level at which those accesses are performed:
//   agent     - the memory side shared by all compute dies (works for any placement);
//   workgroup - the L2 of the compute die the wave runs on.  The vector L1 is
//               write-through and these accesses miss it, so they are coherent between all
//               workgroups of ONE die; the kernel uses this only for chains whose segments
//               all run on the same die (see the queue selection below).
// Status words are always polled with device-scope loads: those bypass the L1 of the compute
// unit (a workgroup-scope load may be served by that L1 and would then never see another
// unit's update) and, for a chain that lives on one die, still hit that die's L2.
template <int SCOPE>
__device__ __forceinline__ int load_status(int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <int SCOPE>
__device__ __forceinline__ void store_status(int* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, SCOPE);
}
template <int SCOPE>
__device__ __forceinline__ void publish1(float* dst, float a) {
  __hip_atomic_store(dst, a, __ATOMIC_RELAXED, SCOPE);
}
template <int SCOPE>
__device__ __forceinline__ float fetch1(const float* src) {
  return __hip_atomic_load(src, __ATOMIC_RELAXED, SCOPE);
}
template <int SCOPE>
__device__ __forceinline__ void publish2(float* dst, float a, float b) {   // dst 8-byte aligned
  unsigned long long bits = (unsigned long long)__builtin_bit_cast(unsigned, a) |
                            ((unsigned long long)__builtin_bit_cast(unsigned, b) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), bits, __ATOMIC_RELAXED, SCOPE);
}
template <int SCOPE>
__device__ __forceinline__ void fetch2(const float* src, float& a, float& b) {
  const unsigned long long bits =
      __hip_atomic_load(reinterpret_cast<const unsigned long long*>(src), __ATOMIC_RELAXED, SCOPE);
  a = __builtin_bit_cast(float, (unsigned)(bits & 0xffffffffull));
  b = __builtin_bit_cast(float, (unsigned)(bits >> 32));
}
__device__ __forceinline__ void wait_all_memory_ops() { __builtin_amdgcn_s_waitcnt(0); }

// Look-back, run by one wave.  Leaves the vector entering this segment in vin[0..20).
// Window: the 64 predecessors k-1 .. k-64 of the same sample; status words are stored
// sample-major so that the window is 256 contiguous bytes (two cache lines per poll).  The nearest one that has
// published its inclusive vector is the base; every nearer one must have published its
// total.  Lower tickets are already running or finished, so the wait ends; a bounded spin
// turns anything unexpected into an error flag instead of a hang.
template <int SCOPE>
__device__ void look_back(int k, int b, int B, int nseg, int* status, const float* agg, const float* incl,
                          float* vin, Header* hdr) {
  const int lane = threadIdx.x & 63;
  const int idx = k - 1 - lane;
  int f = -1;
  for (unsigned spin = 0;; ++spin) {
    int st = kTotalReady;                       // lanes past segment 0 never block the window
    if (idx >= 0) st = load_status<SCOPE>(status + (size_t)b * nseg + idx);
    const unsigned long long pmask = __ballot(idx >= 0 && st == kPrefixReady);
    const unsigned long long amask = __ballot(st >= kTotalReady);
    if (pmask) {
      const int first = __ffsll((long long)pmask) - 1;
      const unsigned long long need = (first == 0) ? 0ull : (~0ull >> (64 - first));
      if ((amask & need) == need) { f = first; break; }
    }
    // give up when the wait is hopeless, or as soon as any other workgroup has given up
    if (spin >= kSpinLimit) break;
    if ((spin & 63) == 63 && __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
    __builtin_amdgcn_s_sleep(2);
  }
  if (f < 0) {                                  // flag it and fall through with zeros
    if (lane == 0) __hip_atomic_store(&hdr->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (lane < H) vin[lane] = 0.f;
    return;
  }
  BPPSA_LB_TRACE(8, wall_clock64());
  BPPSA_LB_TRACE(9, (long long)f);
  // v = inclusive vector of segment k-1-f, then the f totals nearer to us, far to near
  __builtin_amdgcn_s_setprio(3);                // the chain of hops outranks the MFMA waves
  // Three groups of 20 lanes each own one row of a published total (lanes 60..63 mirror
  // group 2).  Totals are fetched six at a time into two register buffers; every load is
  // unconditional (indices past the end are clamped), so the buffers stream while earlier
  // hops are being applied and the whole chain costs about one L2 round trip plus the hops.
  const int grp = lane < 3 * H ? lane / H : 2;
  const int row = lane < 3 * H ? lane - grp * H : lane - 44;
  auto fetch_batch = [&](v4f (&buf)[2][5], int n0) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
      int n = n0 + 3 * sl + grp;
      n = n < f ? n : f - 1;
      n = n < 0 ? 0 : n;
      const float* src = agg + ((size_t)(k - f + n) * B + b) * kAggStride + row * H;
#pragma unroll
      for (int c4 = 0; c4 < 5; ++c4) {
        float e0, e1, e2, e3;
        fetch2<SCOPE>(src + 4 * c4, e0, e1);
        fetch2<SCOPE>(src + 4 * c4 + 2, e2, e3);
        buf[sl][c4] = v4f{e0, e1, e2, e3};
      }
    }
  };
  float v[H];
  auto apply_batch = [&](const v4f (&buf)[2][5], int n0) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        if (n0 + 3 * sl + g < f) {              // wave-uniform
          // four independent partial sums: the hop is on the critical path of every
          // later segment of this sample, so keep its dependency chain short
          float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
          for (int c4 = 0; c4 < 5; ++c4) {
            a0 += buf[sl][c4][0] * v[4 * c4 + 0];
            a1 += buf[sl][c4][1] * v[4 * c4 + 1];
            a2 += buf[sl][c4][2] * v[4 * c4 + 2];
            a3 += buf[sl][c4][3] * v[4 * c4 + 3];
          }
          const float acc = (a0 + a1) + (a2 + a3);
#pragma unroll
          for (int c = 0; c < H; ++c) v[c] = readlane_f(acc, g * H + c);
        }
      }
    }
  };
  const float x = fetch1<SCOPE>(incl + ((size_t)(k - 1 - f) * B + b) * kIncStride + (lane < H ? lane : 0));
  v4f buf0[2][5], buf1[2][5];
  if (f > 0) {                                  // wave-uniform; with f == 0 no total is needed
    fetch_batch(buf0, 0);
    fetch_batch(buf1, 6);
  }
#pragma unroll
  for (int c = 0; c < H; ++c) v[c] = readlane_f(x, c);
  // hop n (0-based, n < f) applies the total of segment k-f+n
  for (int n0 = 0; n0 < f; n0 += 12) {
    apply_batch(buf0, n0);
    if (n0 + 12 < f) fetch_batch(buf0, n0 + 12);
    apply_batch(buf1, n0 + 6);
    if (n0 + 18 < f) fetch_batch(buf1, n0 + 18);
  }
  if (lane == 0) {
#pragma unroll
    for (int c = 0; c < H; ++c) vin[c] = v[c];
  }
  BPPSA_LB_TRACE(10, wall_clock64());
  __builtin_amdgcn_s_setprio(0);
}

#ifdef BPPSA_TRACE
#define BPPSA_STAMP(i) do { if (trace && threadIdx.x == 0) trace[(size_t)me * 16 + (i)] = wall_clock64(); } while (0)
#define BPPSA_TRACE_PARAM , long long* trace
#define BPPSA_TRACE_ARG , nullptr
#define BPPSA_TRACE_FWD , trace
#else
#define BPPSA_STAMP(i) do { } while (0)
#define BPPSA_TRACE_PARAM
#define BPPSA_TRACE_ARG
#define BPPSA_TRACE_FWD
#endif

// Identity of the compute die (XCD) this wave runs on: bits [3:0] of hardware register
// XCC_ID (id 20).
__device__ __forceinline__ int xcc_id() { return __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15; }

// Work distribution.  The samples are dealt round-robin to `nq` queues (sample b belongs to
// queue b % nq); a queue hands out its (segment, sample) pairs in chain order through an
// atomic ticket.  Workgroups are persistent: each drains one queue and leaves when it is
// empty, so a workgroup only ever waits for tickets that were taken before its own.
//   LOCAL  - nq = 8 and the queue is chosen by the die the workgroup runs on: every chain
//            then lives on one die and its look-back traffic stays in that die's L2.  The
//            last workgroup to leave checks that every queue was served by its die; a queue
//            that was not (its die received no workgroup) is untouched, and that workgroup
//            drains it alone with device-scope accesses - slow, but correct for any placement.
//   !LOCAL - the queue is blockIdx % nq and all cross-workgroup traffic is device scope
//            (batch sizes that are not a multiple of 8).
struct Shared {
  float* mat;
  float* vec;
  float* vin;
  int* ticket_s;
};

template <int SCOPE>
__device__ __forceinline__ void drain_queue(int qid, int T, int B, int n, int nseg, int nq,
                                            const float* __restrict__ Jt, const float* __restrict__ seed,
                                            float* __restrict__ G, float* __restrict__ g0, Header* hdr,
                                            int* status, float* agg, float* incl, const Shared sh,
                                            const float* __restrict__ hsrc, const float* __restrict__ wt
                                            BPPSA_TRACE_PARAM) {
  float* const mat = sh.mat;
  float* const vec = sh.vec;
  float* const vin = sh.vin;
  const int bq = (B - qid + nq - 1) / nq;        // samples of this queue: qid, qid + nq, ...
  const int quota = nseg * bq;
  // The ticket of the next segment is requested while the current one is in its down-sweep
  // (below), so that the round trip of the atomic - and of the gradient stores issued before
  // it, which return on the same counter - is off the path between two segments.
  if (threadIdx.x == 0) *sh.ticket_s = __hip_atomic_fetch_add(&hdr->ticket[qid][0], 1, __ATOMIC_RELAXED, SCOPE);
  __syncthreads();
  for (;;) {
    // Re-derive the lane coordinates inside the loop from an opaque copy of the thread id:
    // otherwise every LDS address of the body is hoisted out of the loop and the hoisted
    // values spill.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, slot = lane >> 2, q = lane & 3;
    const int ticket = __builtin_amdgcn_readfirstlane(*sh.ticket_s);
    if (ticket >= quota) break;                  // uniform: the queue is empty
    const int k = ticket / bq;                   // segment, 0 = seed end
    const int b = qid + nq * (ticket - k * bq);
    const size_t me = (size_t)k * B + b;
    // The four waves have different amounts of work (below); which wave takes which part
    // rotates with the ticket, so that the workgroups sharing a compute unit do not all put
    // their heaviest wave on the same SIMD.
    //   role 0: 9 of the 25 level-0 blocks;  role 1: 6 blocks and level 4;
    //   role 2: 6 blocks, a level-3 product and the top of the down-sweep;
    //   role 3: 4 blocks, a level-3 product and the look-back.
    const int role = (wave + ticket) & 3;
    BPPSA_STAMP(0);
    const int c0 = k * S;                        // first chain element of the segment
    const int m = (n - c0 < S) ? (n - c0) : S;   // real elements; the rest are identity tiles

    // ---- load: element p is Jt[T-1-c0-p][b] ------------------------------------------
    {
      constexpr int kChunks = S * HH / 4;        // 16-byte pieces
      v4f tmp[(kChunks + kThreads - 1) / kThreads];
#pragma unroll
      for (int r = 0; r < (kChunks + kThreads - 1) / kThreads; ++r) {
        const int e = tid + r * kThreads;
        const int p = e / (HH / 4), off = e - p * (HH / 4);
        if (e < kChunks && p < m) {
          if (hsrc) {
            // fused tanh-RNN form (Section 4.1): the tile of step t = T-1-c0-p is generated from
            // h[t+1] and the transposed weights, Jt[i][j] = W_hh[j][i] (1 - h[t+1][j]^2), instead
            // of being read
            const int i = off / 5, j4 = (off - i * 5) * 4;
            const v4f wv = *reinterpret_cast<const v4f*>(wt + i * H + j4);
            const v4f hv = *reinterpret_cast<const v4f*>(hsrc + ((size_t)(T - c0 - p) * B + b) * H + j4);
#pragma unroll
            for (int u = 0; u < 4; ++u) tmp[r][u] = wv[u] * __builtin_fmaf(-hv[u], hv[u], 1.0f);   // as the builder
          } else {
            const float* src = Jt + ((size_t)(T - 1 - c0 - p) * B + b) * HH;
            tmp[r] = reinterpret_cast<const v4f*>(src)[off];
          }
        } else {
          const int i0 = (off * 4) / H, j0 = off * 4 - i0 * H;   // identity padding
          tmp[r] = v4f{i0 == j0 ? 1.f : 0.f, i0 == j0 + 1 ? 1.f : 0.f, i0 == j0 + 2 ? 1.f : 0.f,
                       i0 == j0 + 3 ? 1.f : 0.f};
        }
      }
#pragma unroll
      for (int r = 0; r < (kChunks + kThreads - 1) / kThreads; ++r) {
        const int e = tid + r * kThreads;
        const int p = e / (HH / 4), off = e - p * (HH / 4);
        if (e < kChunks) reinterpret_cast<v4f*>(mat + toff(p))[off] = tmp[r];
      }
    }
    __syncthreads();
    BPPSA_STAMP(1);

    // ---- up-sweep level 0: a[2s+1] <- a[2s+1] a[2s] -------------------------------------
    {
      v4f acc[9];
      float* A = mat + toff(2 * slot + 1);
      const float* Bm = mat + toff(2 * slot);
      switch (role) {
        case 0: level0_compute<0, 3, 0, 3>(A, Bm, q, acc); break;
        case 1: level0_compute<0, 3, 3, 2>(A, Bm, q, acc); break;
        case 2: level0_compute<3, 2, 0, 3>(A, Bm, q, acc); break;
        default: level0_compute<3, 2, 3, 2>(A, Bm, q, acc); break;
      }
      __syncthreads();
      switch (role) {
        case 0: level0_store<0, 3, 0, 3>(A, q, acc); break;
        case 1: level0_store<0, 3, 3, 2>(A, q, acc); break;
        case 2: level0_store<3, 2, 0, 3>(A, q, acc); break;
        default: level0_store<3, 2, 3, 2>(A, q, acc); break;
      }
    }
    __syncthreads();
    BPPSA_STAMP(11);
    // ---- up-sweep levels 1..4: pairs (l, r) = (i + 2^d - 1, i + 2^(d+1) - 1) ------------
    // Levels 1 and 2 of the eight tiles 8w .. 8w+7 belong to the wave of role w alone: the LDS operations
    // of one wave complete in order, so no workgroup barrier is needed between the two.
    {
      float* sub = mat + toff(8 * role);
      wave_product(sub + toff(3), sub + toff(1), slot, q);
      wave_product(sub + toff(7), sub + toff(5), slot, q);
      wave_product(sub + toff(7), sub + toff(3), slot, q);
    }
    __syncthreads();
    BPPSA_STAMP(12);
    if (role >= 2) wave_product(mat + toff(16 * (role - 2) + 15), mat + toff(16 * (role - 2) + 7), slot, q);
    __syncthreads();
    if (role == 1) wave_product(mat + toff(31), mat + toff(15), slot, q);
    __syncthreads();
    BPPSA_STAMP(2);
    float* total = mat + toff(S - 1);

    // ---- publish the segment total (interior segments only) -----------------------------
    if (k > 0 && k < nseg - 1) {
      float* dst = agg + me * kAggStride;
      if (tid < HH / 2) publish2<SCOPE>(dst + 2 * tid, total[2 * tid], total[2 * tid + 1]);
      wait_all_memory_ops();
      __syncthreads();
      if (tid == 0) store_status<SCOPE>(status + (size_t)b * nseg + k, kTotalReady);
    }

    BPPSA_STAMP(3);
    // ---- incoming vector, inclusive vector -----------------------------------------------
    if (role == 3) {
      if (k == 0) {
        if (lane < H) vin[lane] = seed[(size_t)b * H + lane];
      } else {
        look_back<SCOPE>(k, b, B, nseg, status, agg, incl, vin, hdr);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      if (lane < H) {
        const float y = row_dot(total, lane, vin);
        if (k < nseg - 1) {
          publish1<SCOPE>(incl + me * kIncStride + lane, y);
        } else {                                  // the chain's last output: g[t_min]
          float* dst = (n == T) ? g0 + (size_t)b * H : G + (size_t)b * H;
          dst[lane] = y;
        }
      }
      if (k < nseg - 1) {
        wait_all_memory_ops();
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) store_status<SCOPE>(status + (size_t)b * nseg + k, kPrefixReady);
      }
    }
    __syncthreads();
    BPPSA_STAMP(4);
    // next ticket: no wait is left in this segment, so holding it delays nobody
    int next_ticket = 0;
    if (tid == 0) next_ticket = __hip_atomic_fetch_add(&hdr->ticket[qid][0], 1, __ATOMIC_RELAXED, SCOPE);

    // ---- down-sweep: T <- a[l]; a[l] <- a[r]; a[r] <- T a[r] ----------------------------
    // Matrix-vector products only.  The wave of role w owns the eight elements 8w .. 8w+7 from
    // here to the store, so no workgroup barrier is needed: it first forms the vector that
    // levels 4 and 3 leave at the top of its sub-tree (up to two products, repeated by every
    // wave that needs them) and then runs levels 2, 1 and 0 of that sub-tree.  LDS operations
    // of one wave complete in order, and every lane's reads of a level are issued before any
    // lane's writes.
    {
      float* const wvec = vec + 8 * role * H;    // vectors entering elements 8w .. 8w+7
      auto wave_sync = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      };
      // level 4 gives element 16 the vector a[15] vin; level 3 gives element 8 a[7] vin and
      // element 24 a[23] (a[15] vin)
      if (lane < H) {
        float u = vin[lane];
        if (role == 1) u = row_dot(mat + toff(7), lane, vin);
        if (role >= 2) u = row_dot(mat + toff(15), lane, vin);
        wvec[7 * H + lane] = u;
      }
      wave_sync();
      if (role == 3) {
        float u = 0.f;
        if (lane < H) u = row_dot(mat + toff(23), lane, wvec + 7 * H);
        wave_sync();
        if (lane < H) wvec[7 * H + lane] = u;
        wave_sync();
      }
#pragma unroll
      for (int d = 2; d >= 0; --d) {
        const int npairs = 8 >> (d + 1);
        float res[2], keep[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          const int e = lane + 64 * r;
          res[r] = 0.f;
          keep[r] = 0.f;
          if (e < npairs * H) {
            const int pr = e / H, row = e - pr * H;
            const int i = pr << (d + 1);
            const int l = i + (1 << d) - 1, rr = i + (2 << d) - 1;
            res[r] = row_dot(mat + toff(8 * role + l), row, wvec + rr * H);
            keep[r] = wvec[rr * H + row];
          }
        }
        wave_sync();
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          const int e = lane + 64 * r;
          if (e < npairs * H) {
            const int pr = e / H, row = e - pr * H;
            const int i = pr << (d + 1);
            const int l = i + (1 << d) - 1, rr = i + (2 << d) - 1;
            wvec[l * H + row] = keep[r];
            wvec[rr * H + row] = res[r];
          }
        }
        wave_sync();
      }

      BPPSA_STAMP(5);
      // ---- store: the vector entering element p is g[T-c0-p] = G[T-1-c0-p] ----------------
      // gradients of a long sequence are streamed past the caches; a short one is left in
      // cache for the parameter-gradient pass that follows
      const bool stream_out = (size_t)T * B * H * sizeof(float) > ((size_t)64 << 20);
      if (tid == 0) *sh.ticket_s = next_ticket;   // every thread read the current one long ago
#pragma unroll
      for (int r = 0; r < 3; ++r) {
        const int e = lane + 64 * r;
        const int p = 8 * role + e / H, row = e - (e / H) * H;
        if (e < 8 * H && p < m) {
          float* dst = G + ((size_t)(T - 1 - c0 - p) * B + b) * H + row;
          if (stream_out) __builtin_nontemporal_store(wvec[e], dst);
          else *dst = wvec[e];
        }
      }
    }
    BPPSA_STAMP(6);
    __syncthreads();                              // LDS and ticket_s are reused by the next segment
  }
}

template <bool LOCAL>
__global__ void __launch_bounds__(kThreads, 3)
scan_h20_kernel(int T, int B, int n, int nseg, int nq, int skip_dies, const float* __restrict__ Jt,
                const float* __restrict__ seed, float* __restrict__ G, float* __restrict__ g0,
                Header* hdr, int* status, float* agg, float* incl, const float* __restrict__ hsrc,
                const float* __restrict__ wt BPPSA_TRACE_PARAM) {
  // 32 tiles, then room so that the 32 down-sweep vectors can start on top of the last tile
  // (the segment total, dead once the inclusive vector has been formed)
  __shared__ __attribute__((aligned(16))) float lds[toff(S - 1) + S * H];
  __shared__ __attribute__((aligned(16))) float vin[H];
  __shared__ int ticket_s;
  const Shared sh = {lds, lds + toff(S - 1), vin, &ticket_s};
  if (!LOCAL) {
    const int qid = (int)(blockIdx.x % (unsigned)nq);
    drain_queue<__HIP_MEMORY_SCOPE_AGENT>(qid, T, B, n, nseg, nq, Jt, seed, G, g0, hdr, status, agg, incl, sh,
                                          hsrc, wt BPPSA_TRACE_FWD);
    return;
  }
  const int qid = xcc_id() & (kMaxQueues - 1);
  // skip_dies is 0 in normal use; a test sets bits to make the workgroups of those dies stand
  // aside, which exercises the fallback below
  const bool aside = ((skip_dies >> qid) & 1) != 0;
  // Count this workgroup in for its die.  The result is not used, so the wave does not wait
  // for the (device-scope, hence slow) atomic; it only has to land before this workgroup ends.
  if (threadIdx.x == 0)
    __hip_atomic_fetch_add(&hdr->started[aside ? kMaxQueues : qid][0], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (!aside)
    drain_queue<__HIP_MEMORY_SCOPE_WORKGROUP>(qid, T, B, n, nseg, nq, Jt, seed, G, g0, hdr, status, agg, incl, sh,
                                              hsrc, wt BPPSA_TRACE_FWD);
  // A queue whose die received no workgroup is untouched.  That is certain only once every
  // workgroup of the grid has started; the workgroups that find this to be the case when they
  // run out of work (the last one to finish always does, because every workgroup waits for its
  // own count to land before it ends) drain such queues together with device-scope accesses.
  __syncthreads();                               // every thread has read the final ticket
  if (threadIdx.x == 0) {
    wait_all_memory_ops();
    int total = 0, unserved = 0;
#pragma unroll
    for (int q = 0; q <= kMaxQueues; ++q) {
      const int c = __hip_atomic_load(&hdr->started[q][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      total += c;
      if (q < kMaxQueues && c == 0) unserved |= 1 << q;
    }
    ticket_s = (total == (int)gridDim.x) ? unserved : 0;
  }
  __syncthreads();
  const int unserved = ticket_s;
  __syncthreads();
  for (int q = 0; q < kMaxQueues; ++q) {
    if ((unserved >> q) & 1)
      drain_queue<__HIP_MEMORY_SCOPE_AGENT>(q, T, B, n, nseg, nq, Jt, seed, G, g0, hdr, status, agg, incl, sh,
                                            hsrc, wt BPPSA_TRACE_FWD);
  }
}

// Zeroes the header and the status words; for the fused form also writes wt[i][j] = W_hh[j][i].
__global__ void clear_kernel(int* p, long long nwords, const float* __restrict__ w_hh, float* __restrict__ wt) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nwords) p[i] = 0;
  if (w_hh && i < HH) {
    const int r = (int)i / H, c = (int)i - r * H;
    wt[c * H + r] = w_hh[i];
  }
}

int resident_workgroups() {
  // 3 workgroups of 52.7 KB fit the 160 KB LDS of each of the 256 compute units
  static int cached = 0;
  if (!cached) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    cached = 3 * cus;
  }
  return cached;
}

}  // namespace

// Jt given: the scan proper.  Jt == nullptr: the fused tanh-RNN form, tiles generated from
// (h, w_hh) inside the kernel.
bppsa_status bppsa_scan_h20(int T, int B, const float* Jt, const float* seed, float* G, float* g0,
                            void* workspace, hipStream_t stream, const float* h, const float* w_hh) {
  const int n = g0 ? T : T - 1;                 // chain elements Jt[T-1] .. Jt[T-n]
  if (n <= 0) {                                 // T == 1 without g0: only G[0] = seed (no Jacobian is read)
    clear_kernel<<<1, 64, 0, stream>>>(static_cast<int*>(workspace), 1, nullptr, nullptr);   // the error word
    BPPSA_CHECK_LAUNCH();
    return bppsa_scan_generic(T, B, H, Jt, seed, G, g0, workspace, stream);
  }
  const int nseg = bppsa_ceil_div(n, S);
  const long long nblk = (long long)nseg * B;
  if (nblk > 0x7fffffffLL) return BPPSA_EOVERFLOW;
  char* ws = static_cast<char*>(workspace);
  Header* hdr = reinterpret_cast<Header*>(ws);
  int* status = reinterpret_cast<int*>(ws + kHeaderBytes);
  const size_t status_bytes = bppsa_align_up((size_t)nblk * sizeof(int), 256);
  float* agg = reinterpret_cast<float*>(ws + kHeaderBytes + status_bytes);
  float* incl = agg + (size_t)nblk * kAggStride;
  float* wt = incl + (size_t)nblk * kIncStride;  // [H][H], fused form only
  const long long nwords = (kHeaderBytes + (long long)status_bytes) / 4;
  clear_kernel<<<(int)((nwords + 255) / 256), 256, 0, stream>>>(reinterpret_cast<int*>(ws), nwords, Jt ? nullptr : w_hh,
                                                                wt);
  BPPSA_CHECK_LAUNCH();
  // Persistent grid: as many workgroups as the device holds at once (3 per compute unit).
  // BPPSA_H20_SKIP_DIES (a bit mask, tests only) makes the workgroups of the named dies stand
  // aside so that the last workgroup's device-scope fallback runs.
  const char* skip_env = getenv("BPPSA_H20_SKIP_DIES");
  const int skip_dies = skip_env ? atoi(skip_env) & 0xff : 0;
  const int resident = resident_workgroups();
  long long want = resident;
  if (want > nblk) want = nblk;
  const int grid = (int)want;
  if (B % kMaxQueues == 0) {
    scan_h20_kernel<true><<<grid, kThreads, 0, stream>>>(T, B, n, nseg, kMaxQueues, skip_dies, Jt, seed, G, g0, hdr,
                                                         status, agg, incl, Jt ? nullptr : h, wt BPPSA_TRACE_ARG);
  } else {
    // device-scope form: as many queues as the largest divisor of B up to 8, so that the ticket
    // counters are spread and every queue carries the same number of samples
    int nq = 1;
    for (int d = 2; d <= kMaxQueues; ++d)
      if (B % d == 0) nq = d;
    scan_h20_kernel<false><<<grid, kThreads, 0, stream>>>(T, B, n, nseg, nq, 0, Jt, seed, G, g0, hdr, status,
                                                          agg, incl, Jt ? nullptr : h, wt BPPSA_TRACE_ARG);
  }
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
