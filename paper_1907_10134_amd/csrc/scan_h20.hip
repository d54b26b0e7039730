// Single-pass scan for H = 20 (the paper's RNN size, Section 4.1): every
// transposed Jacobian is read from HBM exactly once.
//
// A workgroup owns a unit of consecutive chain elements of one sample: one half of S = 32
// elements for short chains, two halves (64 elements) for long ones.  A half lives in LDS
// (32 x 1600 B) while Algorithm 1's up-sweep runs on it:
//   up-sweep   : in place on the 32 tiles.  The 31 matrix-matrix products run on the matrix
//                cores as 4x4x1 fp32 MFMA outer products (20 = 5 x 4, so a 20x20 tile is 25
//                blocks of 4x4 with no padding);
//   two halves : the first half's tree is then parked in registers (50 per lane) and its total
//                kept in LDS, the second half (requested into registers while the first was
//                being reduced) takes its place, and the unit total is the product of the two
//                totals - one more level of the same up-sweep.  A unit twice as long halves
//                the number of links of the cross-unit chain, and the tiles of the next unit
//                are already on their way while this one waits for its incoming vector;
//   cross-unit : instead of one launch per level over the unit totals, the workgroup
//                publishes its total, looks back over its predecessors' published totals /
//                inclusive vectors (matrix-vector products only, since everything to the
//                left ends in the gradient vector, Section 3.1) and publishes its own
//                inclusive vector.  Unit ids are handed out by an atomic ticket, so a
//                workgroup only ever waits for workgroups that are already running;
//   down-sweep : Algorithm 1's down-sweep (reversed operands, matrix-vector only) from the
//                incoming vector, on the parked half out of registers and on the resident
//                half out of LDS; the gradients are stored as they are formed.
// The chain runs from the seed end: element c is Jt[T-1-c]; the vector that enters element c
// is g[T-c] = G[T-1-c].
#include "bppsa_internal.h"
#include "scan_plan.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int H = 20;
constexpr int HH = 400;
constexpr int PS = 2 * HH + 4;           // LDS stride of a pair of tiles in floats: two tiles back to back
                                        // plus one 16-byte pad.  Level 0 reads the same element of 16
                                        // even (or 16 odd) tiles at once; with this stride the tiles of
                                        // eight consecutive pairs start four banks apart, so those reads
                                        // spread over all 32 banks instead of hitting four of them
constexpr int S = BPPSA_H20_SEGMENT;
// offset of tile p of a half in LDS
__device__ __forceinline__ constexpr int toff(int p) { return (p >> 1) * PS + (p & 1) * HH; }
constexpr int kThreads = 256;
constexpr int kAggStride = BPPSA_H20_AGG_STRIDE;   // floats per published total (1664 B = 13 lines)
constexpr int kIncStride = BPPSA_H20_INC_STRIDE;   // floats per published vector (128 B)
constexpr unsigned kSpinLimit = 1u << 20;
// Tiles travel global memory -> registers -> LDS in 16-byte pieces.  200 of the 256 threads
// take part: thread t owns piece t % 100 of the tiles t / 100, t / 100 + 2, ..., so that all its
// addresses are one base plus a multiple of a fixed stride.
constexpr int kLoaders = 2 * (HH / 4);
constexpr int kPref = S / 2;                       // pieces per loader thread

enum : int { kNone = 0, kTotalReady = 1, kPrefixReady = 2 };

constexpr int kMaxQueues = 8;     // one work queue per compute die (XCD)
constexpr int kHeaderBytes = BPPSA_H20_HEADER_BYTES;

struct Header {          // first kHeaderBytes of the workspace, zeroed before every scan
  int error;             // set when a bounded wait expired: results are invalid
  int pad[31];
  int ticket[kMaxQueues][32];   // next unit of each queue, one cache line apart
  // workgroups that have started, per die (slot kMaxQueues: bystanders of the diagnostic call),
  // one cache line apart
  int started[kMaxQueues + 1][32];
};
static_assert(sizeof(Header) <= kHeaderBytes, "header does not fit");

__device__ __forceinline__ v4f mfma4(float a, float b, v4f c) {
  return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 0);
}

// ---- level 0: 16 products, one per MFMA block (slot); each wave owns one or two rectangles of
// the 5 x 5 output blocks of every product.  C = A B with A = tile 2s+1, B = tile 2s.  The
// accumulators of rectangle (I0, NI, J0, NJ) are acc[E0 .. E0 + NI * NJ).
template <int I0, int NI, int J0, int NJ, int E0>
__device__ __forceinline__ void level0_compute(const float* A, const float* Bm, int q, v4f (&acc)[7]) {
#pragma unroll
  for (int e = 0; e < NI * NJ; ++e) acc[E0 + e] = v4f{0.f, 0.f, 0.f, 0.f};
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
          acc[E0 + i * NJ + j] = mfma4(a[cur][i][kk], bv[cur][j][kk], acc[E0 + i * NJ + j]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int I0, int NI, int J0, int NJ, int E0>
__device__ __forceinline__ void level0_store(float* C, int q, const v4f (&acc)[7]) {
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) C[(4 * (I0 + i) + v) * H + 4 * (J0 + j) + q] = acc[E0 + i * NJ + j][v];
}

// ---- upper levels: one product per wave; 15 of the 16 MFMA blocks each own a row-block I
// and up to two column-blocks (2jp, 2jp+1).  C overwrites A; only this wave touches A and B.
__device__ __forceinline__ void wave_product(float* A, const float* Bm, int slot, int q) {
  // the few address registers of a product are formed here, per call, rather than once for all
  // the products of a level and kept
  asm volatile("" : "+v"(slot), "+v"(q));
  const int s = slot < 15 ? slot : 14;
  const int I = s / 3, jp = s - I * 3;
  const int J0 = 2 * jp, J1 = (jp < 2) ? J0 + 1 : J0;
  v4f c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
  // Operands travel LDS -> registers three k-steps ahead of the MFMAs that use them (a ring of
  // three stages, 36 registers): the loads of step k4 + 3 are issued when the MFMAs of step k4
  // have been issued and its stage is free again.
  v4f a[3];
  float b0[3][4], b1[3][4];
  auto fetch = [&](int st, int k4) {
    a[st] = *reinterpret_cast<const v4f*>(A + (4 * I + q) * H + 4 * k4);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      b0[st][kk] = Bm[(4 * k4 + kk) * H + 4 * J0 + q];
      b1[st][kk] = Bm[(4 * k4 + kk) * H + 4 * J1 + q];
    }
  };
  fetch(0, 0);
  fetch(1, 1);
  fetch(2, 2);
  __builtin_amdgcn_sched_barrier(0);       // do not sink the loads between the MFMAs
#pragma unroll
  for (int k4 = 0; k4 < 5; ++k4) {
    const int st = k4 % 3;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      c0 = mfma4(a[st][kk], b0[st][kk], c0);
      c1 = mfma4(a[st][kk], b1[st][kk], c1);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (k4 + 3 < 5) {
      fetch(st, k4 + 3);
      __builtin_amdgcn_sched_barrier(0);
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

// Look-back, run by one wave.  Leaves the vector entering this unit in vin[0..20).
// Window: the 64 predecessors k-1 .. k-64 of the same sample; status words are stored
// sample-major so that the window is 256 contiguous bytes (two cache lines per poll).  The nearest one that has
// published its inclusive vector is the base; every nearer one must have published its
// total.  Lower tickets are already running or finished, so the wait ends; a bounded spin
// turns anything unexpected into an error flag instead of a hang.
template <int SCOPE>
__device__ __forceinline__ void look_back(int k, int b, int B, int nunit, int* status, const float* agg, const float* incl,
                          float* vin, Header* hdr, int* hops) {
  const int lane = threadIdx.x & 63;
  const int idx = k - 1 - lane;
  int f = -1;
  for (unsigned spin = 0;; ++spin) {
    int st = kTotalReady;                       // lanes past unit 0 never block the window
    if (idx >= 0) st = load_status<SCOPE>(status + (size_t)b * nunit + idx);
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
  // v = inclusive vector of unit k-1-f, then the f totals nearer to us, far to near
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
          // later unit of this sample, so keep its dependency chain short
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
  // hop n (0-based, n < f) applies the total of unit k-f+n
  for (int n0 = 0; n0 < f; n0 += 12) {
    apply_batch(buf0, n0);
    if (n0 + 12 < f) fetch_batch(buf0, n0 + 12);
    apply_batch(buf1, n0 + 6);
    if (n0 + 18 < f) fetch_batch(buf1, n0 + 18);
  }
  if (lane == 0) {
#pragma unroll
    for (int c = 0; c < H; ++c) vin[c] = v[c];
    hops[(size_t)k * B + b] = f;                // diagnostic: totals this look-back applied
  }
  __builtin_amdgcn_s_setprio(0);
}

// Identity of the compute die (XCD) this wave runs on: bits [3:0] of hardware register
// XCC_ID (id 20).
__device__ __forceinline__ int xcc_id() { return __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15; }

// Orders the LDS accesses of the lanes of one wave (no other wave is involved).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Algorithm 1's up-sweep on the 32 tiles of a half, in place: after it tile 31 holds the
// half's total, the odd tiles the partial products of their levels, the even tiles are
// unchanged.  `lo` (second half of a two-half unit) is the total of the first half: the wave
// that forms this half's total multiplies it in, which is the next level of the same sweep.
// Two parts, each called by all four waves and each ending with a workgroup barrier: level 0
// (16 products, one per MFMA block) needs the most registers of the whole kernel, so the
// request for the next half is issued between the two.
//   role 0: 7 of the 25 level-0 blocks;  role 1: 6 blocks, level 4 (and the unit total);
//   role 2: 6 blocks and a level-3 product;  role 3: 6 blocks, a level-3 product (and, later,
//   the look-back).
__device__ __forceinline__ void up_sweep_level0(float* mat, int role, int slot, int q) {
  // ---- level 0: a[2s+1] <- a[2s+1] a[2s] ----------------------------------------------------
  // The 25 output blocks are cut into rectangles of 6, 6, 6, 4 and 3 blocks; the wave of role 0,
  // which has the least to do in the levels above, takes the last two.  No rectangle needs more
  // than six accumulators and five operand vectors at a time.
  v4f acc[7];
  float* A = mat + toff(2 * slot + 1);
  const float* Bm = mat + toff(2 * slot);
  switch (role) {
    case 0:
      level0_compute<3, 2, 3, 2, 0>(A, Bm, q, acc);
      level0_compute<0, 3, 4, 1, 4>(A, Bm, q, acc);
      break;
    case 1: level0_compute<0, 3, 0, 2, 0>(A, Bm, q, acc); break;
    case 2: level0_compute<0, 3, 2, 2, 0>(A, Bm, q, acc); break;
    default: level0_compute<3, 2, 0, 3, 0>(A, Bm, q, acc); break;
  }
  __syncthreads();
  switch (role) {
    case 0:
      level0_store<3, 2, 3, 2, 0>(A, q, acc);
      level0_store<0, 3, 4, 1, 4>(A, q, acc);
      break;
    case 1: level0_store<0, 3, 0, 2, 0>(A, q, acc); break;
    case 2: level0_store<0, 3, 2, 2, 0>(A, q, acc); break;
    default: level0_store<3, 2, 0, 3, 0>(A, q, acc); break;
  }
  __syncthreads();
}

__device__ __forceinline__ void up_sweep_upper(float* mat, int role, int slot, int q, const float* lo) {
  // ---- levels 1..4: pairs (l, r) = (i + 2^d - 1, i + 2^(d+1) - 1) ------------------------------
  // Levels 1 and 2 of the eight tiles 8w .. 8w+7 belong to the wave of role w alone: the LDS
  // operations of one wave complete in order, so no workgroup barrier is needed between the two.
  {
    float* sub = mat + toff(8 * role);
    wave_product(sub + toff(3), sub + toff(1), slot, q);
    wave_product(sub + toff(7), sub + toff(5), slot, q);
    wave_product(sub + toff(7), sub + toff(3), slot, q);
  }
  __syncthreads();
  // levels 3 and 4 (and the unit total) keep one or two waves busy while the others wait for
  // them: those waves run at a raised priority
  if (role >= 2) {
    __builtin_amdgcn_s_setprio(2);
    wave_product(mat + toff(16 * (role - 2) + 15), mat + toff(16 * (role - 2) + 7), slot, q);
    __builtin_amdgcn_s_setprio(1);
  }
  __syncthreads();
  if (role == 1) {
    __builtin_amdgcn_s_setprio(2);
    wave_product(mat + toff(31), mat + toff(15), slot, q);
    if (lo) wave_product(mat + toff(31), lo, slot, q);
    __builtin_amdgcn_s_setprio(1);
  }
  __syncthreads();
}

// ---- down-sweep of eight elements by one wave ------------------------------------------------
// Written for the vectors E[e] that ENTER element e: Algorithm 1's down-sweep gives the right
// child of a node the node's vector multiplied by the left child's product, i.e.
//     E[s + 1] = a[s] E[s + 1 - 2^d],   d = number of trailing one bits of s,
// where a[s] is what the up-sweep left in tile s.  Within the eight elements of a wave that
// is one product with tile 3 (level 2), two with tiles 1 and 5 (level 1) and four with the
// even tiles (level 0); tile 7 - the product of all eight - belongs to the levels above.
// A product is split over 40 lanes: lane pairs own the two halves of a row.  The 320 half
// rows of the eight tiles are laid out in the order they are needed, [tile 7 | 3 | 1 5 |
// 0 2 4 6], and lane l holds positions l, l + 64, ..., l + 256 - in registers for the parked
// half (`park`), in LDS for the resident one.
__device__ __forceinline__ void halfrow_of(int pos, int& grp, int& tile, int& row, int& half) {
  grp = pos / 40;
  const int within = pos - grp * 40;
  row = within >> 1;
  half = within & 1;
  tile = (int)((0x64205137u >> (4 * grp)) & 7u);   // groups 0..7 hold tiles 7, 3, 1, 5, 0, 2, 4, 6
}

// sum of x over the two lanes of a pair (lanes 2m and 2m+1)
__device__ __forceinline__ float pair_sum(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
  return x + __builtin_bit_cast(float, y);
}

// Copies the tree of the wave's eight tiles from LDS into registers.  Group 0 holds the tile
// the wave needs for the level above its own eight: the product of all eight elements for the
// waves of roles 0 and 1 (tiles 7 and 15), and tile 23 for both role 2 and role 3, so that the
// wave of role 3 can form its own entering vector E[24] = a[23] E[16].
__device__ __forceinline__ void park_octet(const float* mat, int role, int lane, float (&park)[5][10]) {
  asm volatile("" : "+v"(lane));                 // index arithmetic is redone where it is used, not kept in registers
  const int top = role == 0 ? 7 : (role == 1 ? 15 : 23);
#pragma unroll
  for (int j = 0; j < 5; ++j) {
    int grp, tile, row, half;
    halfrow_of(lane + 64 * j, grp, tile, row, half);
    const int t = grp == 0 ? top : 8 * role + tile;
    const v2f* src = reinterpret_cast<const v2f*>(mat + toff(t) + row * H + half * 10);
#pragma unroll
    for (int c = 0; c < 5; ++c) {
      const v2f w = src[c];
      park[j][2 * c] = w[0];
      park[j][2 * c + 1] = w[1];
    }
  }
}

// Where the gradients of a unit go: the vector entering element e of the unit is
// top[-e * estride + row] for e < m (elements past m are identity padding).
struct GradOut {
  float* top;
  int estride;
  int m;
  bool stream_out;
  __device__ __forceinline__ void put(int e, int row, float v) const {
    if (e < m) {
      float* dst = top - (long long)e * estride + row;
      if (stream_out) __builtin_nontemporal_store(v, dst);
      else *dst = v;
    }
  }
};

// Per lane and per position j of the half-row layout, worked out once per unit and used by the
// down-sweeps of both halves:
//   moff : offset (floats) of the half row inside the wave's eight tiles in LDS (resident half);
//   soff : offset (floats) inside Eloc of the half of the source vector E[tile + 1 - 2^d];
//   info : row | (tile + 1) << 8 | half << 16.
struct LaneLayout {
  int moff[5], soff[5], info[5];
};

__device__ __forceinline__ void make_lane_layout(int lane, LaneLayout& L) {
#pragma unroll
  for (int j = 0; j < 5; ++j) {
    int grp, tile, row, half;
    halfrow_of(lane + 64 * j, grp, tile, row, half);
    const int dstl = tile + 1;
    const int srcl = dstl - (dstl & -dstl);      // 4 -> 0, 2 -> 0, 6 -> 4, odd d -> d - 1
    L.moff[j] = toff(tile) + row * H + half * 10;
    L.soff[j] = (srcl >> 1) * H + half * 10;
    L.info[j] = row | (dstl << 8) | (half << 16);
  }
}

// One group of half rows: the lanes LO <= lane < HI of position J form E[tile + 1] from their half
// row (registers for the parked half, LDS for the resident one), keep even results in Eloc
// (vectors entering local elements 0, 2, 4, 6) and store every result that is a real element.
// glow points at the gradient row of local element 8 (the lowest address of the eight); lim is
// the number of real elements from the wave's first one on.
template <bool PARKED, int J, int LO, int HI>
__device__ __forceinline__ void down_group(const float (&park)[5][10], const float* oct, const LaneLayout& L, int lane,
                                           float* Eloc, float* glow, int estride, int lim, bool stream_out) {
  float hr[10];
  if (PARKED) {
#pragma unroll
    for (int c = 0; c < 10; ++c) hr[c] = park[J][c];
  } else {
    const v2f* src = reinterpret_cast<const v2f*>(oct + L.moff[J]);
#pragma unroll
    for (int c = 0; c < 5; ++c) {
      const v2f w = src[c];
      hr[2 * c] = w[0];
      hr[2 * c + 1] = w[1];
    }
  }
  const v2f* sv = reinterpret_cast<const v2f*>(Eloc + L.soff[J]);
  float a0 = 0.f, a1 = 0.f;
#pragma unroll
  for (int c = 0; c < 5; ++c) {
    const v2f x = sv[c];
    a0 += hr[2 * c] * x[0];
    a1 += hr[2 * c + 1] * x[1];
  }
  const float sum = pair_sum(a0 + a1);
  const int info = L.info[J];
  const int row = info & 0xff, dstl = (info >> 8) & 0xff;
  const bool mine = (LO == 0 || lane >= LO) && (HI == 64 || lane < HI) && (info >> 16) == 0;
  if (mine) {
    if (!(dstl & 1)) Eloc[(dstl >> 1) * H + row] = sum;
    if (dstl < lim) {
      float* dst = glow + (unsigned)((8 - dstl) * estride + row);
      if (stream_out) __builtin_nontemporal_store(sum, dst);
      else *dst = sum;
    }
  }
}

// Levels 2, 1 and 0 of the wave's eight elements; Eloc[0..20) holds the vector entering the
// first of them.  Only this wave touches Eloc, so wave-level ordering suffices.
template <bool PARKED>
__device__ __forceinline__ void octet_levels(const float (&park)[5][10], const float* oct, const LaneLayout& L, int lane,
                                             float* Eloc, float* glow, int estride, int lim, bool stream_out) {
  // one group at a time (no interleaving by the scheduler): the registers are needed for the
  // parked half and for the tiles already requested for the next unit
  down_group<PARKED, 0, 40, 64>(park, oct, L, lane, Eloc, glow, estride, lim, stream_out);   // tile 3: positions 40..79
  __builtin_amdgcn_sched_barrier(0);
  down_group<PARKED, 1, 0, 16>(park, oct, L, lane, Eloc, glow, estride, lim, stream_out);
  wave_sync();
  down_group<PARKED, 1, 16, 64>(park, oct, L, lane, Eloc, glow, estride, lim, stream_out);  // tiles 1, 5: positions 80..159
  __builtin_amdgcn_sched_barrier(0);
  down_group<PARKED, 2, 0, 32>(park, oct, L, lane, Eloc, glow, estride, lim, stream_out);
  wave_sync();
  down_group<PARKED, 2, 32, 64>(park, oct, L, lane, Eloc, glow, estride, lim, stream_out);  // tiles 0, 2, 4, 6: positions 160..319
  __builtin_amdgcn_sched_barrier(0);
  down_group<PARKED, 3, 0, 64>(park, oct, L, lane, Eloc, glow, estride, lim, stream_out);
  __builtin_amdgcn_sched_barrier(0);
  down_group<PARKED, 4, 0, 64>(park, oct, L, lane, Eloc, glow, estride, lim, stream_out);
}

// dst[0..20) = (parked group 0 of this wave) src[0..20): the product with the tile of the
// level above the wave's eight elements.  Result also stored as the vector entering element e.
__device__ __forceinline__ void parked_top(const float (&park)[5][10], int lane, const float* src, float* dst, int e,
                                           const GradOut& out) {
  const int row = (lane >> 1) < H ? (lane >> 1) : 0, half = lane & 1;
  const v2f* sv = reinterpret_cast<const v2f*>(src + half * 10);
  float a0 = 0.f, a1 = 0.f;
#pragma unroll
  for (int c = 0; c < 5; ++c) {
    const v2f x = sv[c];
    a0 += park[0][2 * c] * x[0];
    a1 += park[0][2 * c + 1] * x[1];
  }
  const float sum = pair_sum(a0 + a1);
  if (lane < 40 && half == 0) {
    dst[row] = sum;
    out.put(e, row, sum);
  }
}

// Work distribution.  The samples are dealt round-robin to `nq` queues (sample b belongs to
// queue b % nq); a queue hands out its (unit, sample) pairs in chain order through an
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
  float* mat;            // the 32 tiles of the resident half
  float* lo;             // total of the first half; then the even vectors of the parked half
  float* vin;            // vector entering the unit
  float* vmid;           // vector entering the second half
  int* ticket_s;
};

struct Problem {
  int T, B, n, nunit, halves;
  const float* __restrict__ Jt;
  const float* __restrict__ seed;
  float* __restrict__ G;
  float* __restrict__ g0;
  Header* hdr;
  int* status;
  float* agg;
  float* incl;
  int* hops;
  const float* __restrict__ hsrc;    // fused tanh-RNN form: hidden states, else null
  const float* __restrict__ wt;      // fused form: W_hh transposed
};

template <int SCOPE, bool TWO, bool FUSED>
__device__ __forceinline__ void drain_queue(int qid, int nq, const Problem& pr, const Shared sh) {
  const int T = pr.T, B = pr.B, n = pr.n, nunit = pr.nunit;
  constexpr bool two = TWO;                       // units of two halves
  constexpr int U = TWO ? 2 * S : S;              // elements of a unit
  float* const mat = sh.mat;
  float* const vin = sh.vin;
  const int bq = (B - qid + nq - 1) / nq;         // samples of this queue: qid, qid + nq, ...
  const int quota = nunit * bq;
  const bool stream_out = (size_t)T * B * H * sizeof(float) > ((size_t)64 << 20);

  // Tiles of a half travel global memory -> registers -> LDS.  They are requested one half
  // ahead: the second half while the first is being reduced, the first half of the next unit
  // while this unit waits for its incoming vector and runs its down-sweep.
  v4f pref[kPref];
  // requests half `hf` of the unit of ticket `tk`
  auto request_half = [&](int tk, int hf) {
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int k = tk / bq, b = qid + nq * (tk - k * bq);
    const int c0 = k * U + S * hf;               // first chain element of the half
    const int mh = n - c0;                       // real elements (may be <= 0 or > S)
    // every element of pref is assigned on every path: a conditional assignment would keep the
    // previous contents alive, and with them 64 registers, all the way round the loop
    const v4f zero = {0.f, 0.f, 0.f, 0.f};
    const int p0 = tid >= HH / 4 ? 1 : 0, off = tid - p0 * (HH / 4);
    // what a thread fetches of one tile, and the distance (floats) between consecutive tiles
    const int piece = FUSED ? ((off - (off / 5) * 5) * 4) : 4 * off;
    const unsigned tstride = FUSED ? (unsigned)B * H : (unsigned)B * HH;
    const float* arr = FUSED ? pr.hsrc + (size_t)B * H : pr.Jt;   // fused form (Section 4.1): h[t+1] stands for tile t
    if (mh >= S) {
      // a full half (all but the last unit of a sample): one uniform base - the tile of the
      // half's last element, which has the lowest address - plus a 32-bit offset per thread
      if (tid < kLoaders) {
        const char* base = reinterpret_cast<const char*>(arr + ((size_t)(T - 1 - c0 - (S - 1)) * B + b) * (FUSED ? H : HH));
        const unsigned voff = ((unsigned)(S - 1 - p0) * tstride + (unsigned)piece) * 4u;
#pragma unroll
        for (int r = 0; r < kPref; ++r)
          pref[r] = *reinterpret_cast<const v4f*>(base + (size_t)(voff - (unsigned)(2 * r) * tstride * 4u));
      } else {
#pragma unroll
        for (int r = 0; r < kPref; ++r) pref[r] = zero;
      }
    } else {
#pragma unroll
      for (int r = 0; r < kPref; ++r) {
        v4f x = zero;
        if (tid < kLoaders && p0 + 2 * r < mh)
          x = *reinterpret_cast<const v4f*>(arr + ((size_t)(T - 1 - c0 - p0 - 2 * r) * B + b) * (FUSED ? H : HH) + piece);
        pref[r] = x;
      }
    }
  };
  // moves the requested half into LDS; elements past the end of the chain become identity tiles
  auto land_half = [&](int tk, int hf) {
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int k = tk / bq;
    const int mh = n - (k * U + S * hf);
    if (tid < kLoaders) {
      const int p0 = tid >= HH / 4 ? 1 : 0, off = tid - p0 * (HH / 4);
      v4f wv = {0.f, 0.f, 0.f, 0.f};
      if (FUSED) {
        const int i = off / 5, j4 = (off - i * 5) * 4;
        wv = *reinterpret_cast<const v4f*>(pr.wt + i * H + j4);
      }
      float* dst = mat + p0 * HH + 4 * off;      // tile p0 + 2r sits r pair strides further
      if (mh >= S) {
#pragma unroll
        for (int r = 0; r < kPref; ++r) {
          v4f val = pref[r];
          if (FUSED) {
            // Jt[i][j] = W_hh[j][i] (1 - h[t+1][j]^2), the arithmetic of the builder
#pragma unroll
            for (int u = 0; u < 4; ++u) val[u] = wv[u] * __builtin_fmaf(-val[u], val[u], 1.0f);
          }
          *reinterpret_cast<v4f*>(dst + r * PS) = val;
        }
      } else {
        const int i0 = (off * 4) / H, j0 = off * 4 - i0 * H;
        const v4f ident = {i0 == j0 ? 1.f : 0.f, i0 == j0 + 1 ? 1.f : 0.f, i0 == j0 + 2 ? 1.f : 0.f,
                           i0 == j0 + 3 ? 1.f : 0.f};
#pragma unroll
        for (int r = 0; r < kPref; ++r) {
          v4f val = ident;
          if (p0 + 2 * r < mh) {
            val = pref[r];
            if (FUSED) {
#pragma unroll
              for (int u = 0; u < 4; ++u) val[u] = wv[u] * __builtin_fmaf(-val[u], val[u], 1.0f);
            }
          }
          *reinterpret_cast<v4f*>(dst + r * PS) = val;
        }
      }
    }
  };

  if (threadIdx.x == 0) *sh.ticket_s = __hip_atomic_fetch_add(&pr.hdr->ticket[qid][0], 1, __ATOMIC_RELAXED, SCOPE);
  __syncthreads();
  int ticket = __builtin_amdgcn_readfirstlane(*sh.ticket_s);
  request_half(ticket, 0);                       // past the end of the queue: fetches nothing
  for (;;) {
    // Re-derive the lane coordinates inside the loop from an opaque copy of the thread id:
    // otherwise every LDS address of the body is hoisted out of the loop and the hoisted
    // values spill.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, slot = lane >> 2, q = lane & 3;
    if (ticket >= quota) break;                  // uniform: the queue is empty
    const int k = ticket / bq;                   // unit, 0 = seed end
    const int b = qid + nq * (ticket - k * bq);
    const size_t me = (size_t)k * B + b;
    // The four waves have different amounts of work; which wave takes which part rotates with
    // the ticket, so that the workgroups sharing a compute unit do not all put their heaviest
    // wave on the same SIMD.
    const int role = (wave + ticket) & 3;
    const int c0 = k * U;                        // first chain element of the unit
    const int m = (n - c0 < U) ? (n - c0) : U;   // real elements; the rest are identity tiles
    const GradOut out = {pr.G + ((size_t)(T - 1 - c0) * B + b) * H, B * H, m, stream_out};

    // Everything up to the published total is what later units of this sample wait for; it runs
    // at a higher wave priority than the down-sweeps of the other workgroups of the compute unit.
    __builtin_amdgcn_s_setprio(1);
    float park[5][10];
    if (two) {
      // ---- first half: reduce, park the tree in registers, keep the total in LDS ---------------
      land_half(ticket, 0);
      __syncthreads();
      up_sweep_level0(mat, role, slot, q);
      request_half(ticket, 1);
      up_sweep_upper(mat, role, slot, q, nullptr);
      park_octet(mat, role, lane, park);
      if (tid < HH / 4) reinterpret_cast<v4f*>(sh.lo)[tid] = reinterpret_cast<const v4f*>(mat + toff(S - 1))[tid];
      __syncthreads();
    }
    // ---- last half: reduce; with two halves the unit total is (this total) (first total) -------
    land_half(ticket, two ? 1 : 0);
    // The ticket of the next unit is requested now, so that the round trip of the atomic is off
    // the path between two units.
    int next_ticket = 0;
    if (tid == 0) next_ticket = __hip_atomic_fetch_add(&pr.hdr->ticket[qid][0], 1, __ATOMIC_RELAXED, SCOPE);
    __syncthreads();
    up_sweep_level0(mat, role, slot, q);
    up_sweep_upper(mat, role, slot, q, two ? sh.lo : nullptr);
    float* total = mat + toff(S - 1);

    // ---- publish the unit total (interior units only) -------------------------------------------
    const bool interior = k > 0 && k < nunit - 1;
    if (interior && tid < HH / 2) publish2<SCOPE>(pr.agg + me * kAggStride + 2 * tid, total[2 * tid], total[2 * tid + 1]);
    wait_all_memory_ops();                        // the total is out (and thread 0 has its next ticket)
    if (tid == 0) *sh.ticket_s = next_ticket;     // every thread read the current one long ago
    __syncthreads();
    if (interior && tid == 0) store_status<SCOPE>(pr.status + (size_t)b * nunit + k, kTotalReady);
    const int next = __builtin_amdgcn_readfirstlane(*sh.ticket_s);
    __builtin_amdgcn_s_setprio(0);

    // ---- incoming vector, inclusive vector; the next unit's first half is requested ------------
    if (role == 3) {
      if (k == 0) {
        if (lane < H) vin[lane] = pr.seed[(size_t)b * H + lane];
      } else {
        look_back<SCOPE>(k, b, B, nunit, pr.status, pr.agg, pr.incl, vin, pr.hdr, pr.hops);
      }
      wave_sync();
      if (lane < H) {
        const float y = row_dot(total, lane, vin);
        if (k < nunit - 1) {
          publish1<SCOPE>(pr.incl + me * kIncStride + lane, y);
        } else {                                  // the chain's last output: g[t_min]
          float* dst = (n == T) ? pr.g0 + (size_t)b * H : pr.G + (size_t)b * H;
          dst[lane] = y;
        }
      } else if (two && lane >= 32 && lane < 32 + H) {
        sh.vmid[lane - 32] = row_dot(sh.lo, lane - 32, vin);
      }
      if (k < nunit - 1) {
        wait_all_memory_ops();
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) store_status<SCOPE>(pr.status + (size_t)b * nunit + k, kPrefixReady);
      }
      // this wave's loads return in order, so its share of the next half is requested only now
      // (unconditionally: past the end of the queue there is nothing to fetch and the registers
      // are simply cleared, which ends the life of their previous contents)
      request_half(next, 0);
    } else {
      request_half(next, 0);
    }
    __syncthreads();

    // ---- down-sweep -----------------------------------------------------------------------------
    // Matrix-vector products only.  The wave of role w owns elements 8w .. 8w+7 of each half and
    // runs levels 2, 1, 0 of that sub-tree alone; the vector entering its first element comes
    // from the levels above: E[8] = a[7] E[0], E[16] = a[15] E[0], E[24] = a[23] E[16].
    {
      float* const EA = sh.lo;                   // [4 waves][4 vectors][20], parked half
      float* const EB = total;                   // same for the resident half (the total is dead now)
      LaneLayout L;
      make_lane_layout(lane, L);
      const int estride = B * H;
      if (two) {
        // parked half, levels above the waves: role 0 forms E[8], role 1 E[16]
        if (role == 0 && lane < H) {
          const float u = vin[lane];
          EA[lane] = u;
          out.put(0, lane, u);
        }
        if (role <= 1) parked_top(park, lane, vin, EA + (role + 1) * 4 * H, 8 * (role + 1), out);
      }
      // resident half: every wave forms the vector entering its own eight elements itself (up
      // to two products, repeated by the waves that need them), so no workgroup barrier is needed
      {
        const float* vB = two ? sh.vmid : vin;
        const int ebase = (two ? S : 0) + 8 * role;
        float* Eloc = EB + role * 4 * H;
        if (lane < H) {
          float u = vB[lane];
          if (role == 1) u = row_dot(mat + toff(7), lane, vB);
          if (role >= 2) u = row_dot(mat + toff(15), lane, vB);
          Eloc[lane] = u;
        }
        wave_sync();
        if (role == 3) {
          float u = 0.f;
          if (lane < H) u = row_dot(mat + toff(23), lane, Eloc);
          wave_sync();
          if (lane < H) Eloc[lane] = u;
          wave_sync();
        }
        if (lane < H) out.put(ebase, lane, Eloc[lane]);
        octet_levels<false>(park, mat + toff(8 * role), L, lane, Eloc, out.top - (long long)(ebase + 8) * estride,
                            estride, m - ebase, stream_out);
      }
      if (two) {
        __syncthreads();                          // E[8] and E[16] of the parked half are in LDS
        float* Eloc = EA + role * 4 * H;
        if (role == 3) {
          parked_top(park, lane, EA + 2 * 4 * H, Eloc, 24, out);
          wave_sync();
        }
        octet_levels<true>(park, mat, L, lane, Eloc, out.top - (long long)(8 * role + 8) * estride, estride,
                           m - 8 * role, stream_out);
      }
    }
    ticket = next;
    __syncthreads();                              // LDS and ticket_s are reused by the next unit
  }
}

template <bool LOCAL, bool TWO, bool FUSED>
__global__ void __launch_bounds__(kThreads, 3)
scan_h20_kernel(int nq, int skip_dies, const Problem pr) {
  // 32 tiles (the last one is the unit total and, once that is dead, the even vectors of the
  // resident half's down-sweep), the first half's total, two vectors
  __shared__ __attribute__((aligned(16))) float lds[toff(S - 1) + HH + HH + 2 * H];
  __shared__ int ticket_s;
  const Shared sh = {lds, lds + toff(S - 1) + HH, lds + toff(S - 1) + 2 * HH, lds + toff(S - 1) + 2 * HH + H, &ticket_s};
  if (!LOCAL) {
    const int qid = (int)(blockIdx.x % (unsigned)nq);
    drain_queue<__HIP_MEMORY_SCOPE_AGENT, TWO, FUSED>(qid, nq, pr, sh);
    return;
  }
  const int qid = xcc_id() & (kMaxQueues - 1);
  // skip_dies is 0 in normal use; the diagnostic call sets bits to make the workgroups of those
  // dies stand aside, which exercises the fallback below
  const bool aside = ((skip_dies >> qid) & 1) != 0;
  // Count this workgroup in for its die.  The result is not used, so the wave does not wait
  // for the (device-scope, hence slow) atomic; it only has to land before this workgroup ends.
  if (threadIdx.x == 0)
    __hip_atomic_fetch_add(&pr.hdr->started[aside ? kMaxQueues : qid][0], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (!aside) drain_queue<__HIP_MEMORY_SCOPE_WORKGROUP, TWO, FUSED>(qid, nq, pr, sh);
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
      const int c = __hip_atomic_load(&pr.hdr->started[q][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      total += c;
      if (q < kMaxQueues && c == 0) unserved |= 1 << q;
    }
    ticket_s = (total == (int)gridDim.x) ? unserved : 0;
  }
  __syncthreads();
  const int unserved = ticket_s;
  __syncthreads();
  for (int q = 0; q < kMaxQueues; ++q) {
    if ((unserved >> q) & 1) drain_queue<__HIP_MEMORY_SCOPE_AGENT, TWO, FUSED>(q, nq, pr, sh);
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

// Sum, count and maximum of the hop counts the look-backs of the last scan recorded.
__global__ void hops_stats_kernel(const int* __restrict__ hops, int nunit, int B, long long* __restrict__ out) {
  __shared__ long long ssum[256];
  __shared__ int smax[256];
  long long sum = 0;
  int mx = 0;
  const long long total = (long long)nunit * B;
  for (long long i = (long long)B + threadIdx.x; i < total; i += blockDim.x) {   // unit 0 has no look-back
    const int f = hops[i];
    sum += f;
    mx = f > mx ? f : mx;
  }
  ssum[threadIdx.x] = sum;
  smax[threadIdx.x] = mx;
  __syncthreads();
  for (int w = 128; w >= 1; w >>= 1) {
    if ((int)threadIdx.x < w) {
      ssum[threadIdx.x] += ssum[threadIdx.x + w];
      smax[threadIdx.x] = smax[threadIdx.x] > smax[threadIdx.x + w] ? smax[threadIdx.x] : smax[threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    out[0] = ssum[0];
    out[1] = total - B;
    out[2] = smax[0];
  }
}

// How a call is cut into units and where its pieces sit in the workspace.
struct Layout {
  int n, halves, nunit;
  long long nblk;
  size_t status_bytes;
};

bool make_layout(int T, int B, bool want_g0, int unit_halves, Layout& L) {
  L.n = want_g0 ? T : T - 1;                    // chain elements Jt[T-1] .. Jt[T-n]
  // Persistent grid: as many workgroups as the device holds at once (3 of 53 KB of LDS per
  // compute unit).  Chains that give every resident workgroup at most one half are cut into
  // units of one half; longer ones into units of two halves.
  const int resident = 3 * bppsa_compute_units();
  const int nhalf = bppsa_ceil_div(L.n > 0 ? L.n : 1, S);
  L.halves = unit_halves;
  if (L.halves != 1 && L.halves != 2) L.halves = ((long long)nhalf * B > resident) ? 2 : 1;
  L.nunit = bppsa_ceil_div(L.n > 0 ? L.n : 1, S * L.halves);
  L.nblk = (long long)L.nunit * B;
  L.status_bytes = bppsa_align_up((size_t)L.nblk * sizeof(int), 256);
  return L.nblk <= 0x7fffffffLL;
}

}  // namespace

// Jt given: the scan proper.  Jt == nullptr: the fused tanh-RNN form, tiles generated from
// (h, w_hh) inside the kernel.  skip_dies and unit_halves are 0 except in the diagnostic call.
bppsa_status bppsa_scan_h20(int T, int B, const float* Jt, const float* seed, float* G, float* g0,
                            void* workspace, hipStream_t stream, const float* h, const float* w_hh,
                            int skip_dies, int unit_halves) {
  Layout L;
  if (!make_layout(T, B, g0 != nullptr, unit_halves, L)) return BPPSA_EOVERFLOW;
  const int n = L.n;
  if (n <= 0) {                                 // T == 1 without g0: only G[0] = seed (no Jacobian is read)
    clear_kernel<<<1, 64, 0, stream>>>(static_cast<int*>(workspace), 1, nullptr, nullptr);   // the error word
    BPPSA_CHECK_LAUNCH();
    return bppsa_scan_generic(T, B, H, Jt, seed, G, g0, workspace, stream);
  }
  const int halves = L.halves;
  const long long nblk = L.nblk;
  char* ws = static_cast<char*>(workspace);
  Problem pr;
  pr.T = T; pr.B = B; pr.n = n; pr.nunit = L.nunit; pr.halves = halves;
  pr.Jt = Jt; pr.seed = seed; pr.G = G; pr.g0 = g0;
  pr.hdr = reinterpret_cast<Header*>(ws);
  pr.status = reinterpret_cast<int*>(ws + kHeaderBytes);
  const size_t status_bytes = L.status_bytes;
  pr.hops = reinterpret_cast<int*>(ws + kHeaderBytes + status_bytes);
  pr.agg = reinterpret_cast<float*>(ws + kHeaderBytes + 2 * status_bytes);
  pr.incl = pr.agg + (size_t)nblk * kAggStride;
  float* wt = pr.incl + (size_t)nblk * kIncStride;   // [H][H], fused form only
  pr.hsrc = Jt ? nullptr : h;
  pr.wt = wt;
  // header, status words and hop counts
  const long long nwords = (kHeaderBytes + 2 * (long long)status_bytes) / 4;
  clear_kernel<<<(int)((nwords + 255) / 256), 256, 0, stream>>>(reinterpret_cast<int*>(ws), nwords, Jt ? nullptr : w_hh,
                                                                wt);
  BPPSA_CHECK_LAUNCH();
  long long want = 3 * bppsa_compute_units();
  if (want > nblk) want = nblk;
  const int grid = (int)want;
  const bool local = B % kMaxQueues == 0;
  // device-scope form (batch sizes that are not a multiple of 8): as many queues as the largest
  // divisor of B up to 8, so that the ticket counters are spread and every queue carries the same
  // number of samples
  int nq = kMaxQueues;
  if (!local) {
    nq = 1;
    for (int d = 2; d <= kMaxQueues; ++d)
      if (B % d == 0) nq = d;
  }
  const int skip = local ? (skip_dies & 0xff) : 0;
#define BPPSA_H20_LAUNCH(L, W, F) scan_h20_kernel<L, W, F><<<grid, kThreads, 0, stream>>>(nq, skip, pr)
  const int variant = (local ? 4 : 0) | (halves == 2 ? 2 : 0) | (Jt ? 0 : 1);
  switch (variant) {
    case 0: BPPSA_H20_LAUNCH(false, false, false); break;
    case 1: BPPSA_H20_LAUNCH(false, false, true); break;
    case 2: BPPSA_H20_LAUNCH(false, true, false); break;
    case 3: BPPSA_H20_LAUNCH(false, true, true); break;
    case 4: BPPSA_H20_LAUNCH(true, false, false); break;
    case 5: BPPSA_H20_LAUNCH(true, false, true); break;
    case 6: BPPSA_H20_LAUNCH(true, true, false); break;
    default: BPPSA_H20_LAUNCH(true, true, true); break;
  }
#undef BPPSA_H20_LAUNCH
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

// Diagnostic: statistics of the look-backs of the last H = 20 scan that used `workspace` with
// these sizes: out[0] = totals applied by all look-backs, out[1] = number of look-backs,
// out[2] = the most one look-back applied.  out is device memory (3 x int64).
bppsa_status bppsa_scan_h20_hops(int T, int B, int want_g0, int unit_halves, const void* workspace,
                                 long long* out, hipStream_t stream) {
  Layout L;
  if (!make_layout(T, B, want_g0 != 0, unit_halves, L)) return BPPSA_EOVERFLOW;
  const int* hops = reinterpret_cast<const int*>(static_cast<const char*>(workspace) + kHeaderBytes + L.status_bytes);
  hops_stats_kernel<<<1, 256, 0, stream>>>(hops, L.n > 0 ? L.nunit : 1, B, out);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
