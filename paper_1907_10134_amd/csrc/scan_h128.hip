// H = 128 kernels of the segmented scan (the GRU size of the long-sequence workload).
//
// At this size a matrix-matrix node of the up-sweep (Algorithm 1, a[r] <- a[r] a[l]) is
// 4.2 MFLOP against 64 KB of operand traffic: it belongs on the matrix cores.  The reduce
// kernel keeps the running product of a segment in registers, as MFMA results that are the next
// step's B operands, and streams one transposed Jacobian per step through LDS; the apply kernel
// walks a segment with matrix-vector products (the down-sweep side), streaming each Jacobian
// once with the next one already in flight; the chain kernels walk the stretch of a long chain
// nearest the seed, which needs no matrix-matrix product at all, one workgroup per sample.
//
// This file is compiled with MFMA results in ordinary vector registers (see the build script):
// an accumulation register cannot be a B operand.
#include "scan_h128_common.h"

namespace {

// The value another lane of the same row of 16 lanes holds, without going through LDS: lane i
// reads lane i ^ 1, i ^ 2 (exact), 7 - i % 8 within its half row, or 15 - i within its row.  The
// last two flip lane bit 2, resp. 3, together with the bits below it, which is all an exchange
// between the two halves of a group of lanes needs when only the sum over the group matters.
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;
template <int CTRL>
__device__ __forceinline__ float dpp_from(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// P <- J P for J = Jt[hi-1], ..., Jt[lo], starting from P = Jt[hi]; tot[seg][b] = P.
//
// v_mfma_f32_32x32x2_f32 contracts two k values per issue: lane l supplies A[i = l % 32][k(l / 32)]
// and B[k(l / 32)][j = l % 32], and holds D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32] in
// accumulator register v.  Any assignment of the 128 k values to (issue, lane half) is valid as
// long as A and B agree.  Here issue (kb, q, s) of lane half h takes k = 32 kb + 8 q + 4 h + s,
// which is exactly the row that accumulator register 4 q + s of row-block kb holds in that lane
// half: the running product never leaves the registers.  Each of the four waves owns a strip of
// 32 columns of P (four 32 x 32 accumulator blocks) and therefore holds every k of its columns;
// the accumulators of one step are the B operands of the next, and two sets alternate.  Only the
// Jacobian goes through LDS, [i][k] with one 16-byte read per row-block feeding four issues, in
// two buffers: while a step reads one, the Jacobian of the next step is written to the other
// piece by piece between the issues (from registers filled one step earlier), and the registers
// are refilled from memory for the step after.  A step therefore has one barrier
// and nothing but its 256 issues on the critical path.
//
// One step: nw = A old, A read from As; piece g of the next Jacobian goes to An during k group g.
// The scheduling barriers pin the order written here.  Left alone, the scheduler puts the LDS
// reads of the next group behind the last issue that uses the registers they could share, and
// the memory requests in one burst ahead of the first issue, which leaves the matrix pipe idle
// for a fifth of the step.
__device__ __forceinline__ void reduce_h128_step(const float* __restrict__ As, float* __restrict__ An,
                                                 const v4f* __restrict__ refill, v4f (&pre)[kChunks], int tid,
                                                 int l32, int hsel, const v16f (&old)[4], v16f (&nw)[4]) {
  const float* arow = As + l32 * LS + 4 * hsel;
  float* stage = An + (tid >> 5) * LS + (tid & 31) * 4;      // piece g lies 8 g rows further down
  const v16f zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  v4f a4[2][4];
#pragma unroll
  for (int bi = 0; bi < 4; ++bi) a4[0][bi] = *reinterpret_cast<const v4f*>(arow + 32 * bi * LS);
#pragma unroll
  for (int g = 0; g < 16; ++g) {                 // g = 4 kb + q
    const int cur = g & 1;
    if (g < 15) {                                // operands of the next k group
#pragma unroll
      for (int bi = 0; bi < 4; ++bi)
        a4[cur ^ 1][bi] = *reinterpret_cast<const v4f*>(arow + 32 * bi * LS + 8 * (g + 1));
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if (s == 1) {
        *reinterpret_cast<v4f*>(stage + 8 * g * LS) = pre[g];
      } else if (s == 2) {
        pre[g] = refill[tid + g * kThreads];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int bi = 0; bi < 4; ++bi)
        nw[bi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[cur][bi][s], old[g >> 2][4 * (g & 3) + s],
                                                      (g == 0 && s == 0) ? zero : nw[bi], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

__global__ void __launch_bounds__(kThreads, 1)
reduce_h128_kernel(int T, int B, int t_min, int S, int seg_begin, const float* __restrict__ Jt,
                   float* __restrict__ tot) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* As0 = smem;                // [128][LS]  A[i][k], two buffers
  float* As1 = smem + H * LS;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, hsel = lane >> 5;
  const int seg = seg_begin + blockIdx.x;
  const int b = blockIdx.y;
  int lo, hi;
  seg_bounds(T, t_min, S, seg, lo, hi);

  v4f pre[kChunks];
  // tile t into the registers of its pieces; t is clamped to the segment, so the steps near the
  // end refill and stage a tile nobody reads instead of branching
  auto tile = [&](int t) { return reinterpret_cast<const v4f*>(Jt + ((size_t)max(t, lo) * B + b) * HH); };
  auto fetch = [&](int t) {
    const v4f* src = tile(t);
#pragma unroll
    for (int r = 0; r < kChunks; ++r) pre[r] = src[tid + r * kThreads];
  };
  auto stage_all = [&](float* As) {
#pragma unroll
    for (int r = 0; r < kChunks; ++r) {
      const int e = tid + r * kThreads;
      *reinterpret_cast<v4f*>(As + (e >> 5) * LS + (e & 31) * 4) = pre[r];
    }
  };
  // P = Jt[hi] through LDS into the accumulator layout: register v of row-block kb holds row
  // 32 kb + 8 (v / 4) + 4 hsel + v % 4 of column 32 wave + l32
  v16f P[4], Q[4];
  fetch(hi);
  stage_all(As1);
  fetch(hi - 1);
  __syncthreads();
#pragma unroll
  for (int kb = 0; kb < 4; ++kb)
#pragma unroll
    for (int v = 0; v < 16; ++v)
      P[kb][v] = As1[(32 * kb + 8 * (v >> 2) + 4 * hsel + (v & 3)) * LS + 32 * wave + l32];
  stage_all(As0);
  fetch(hi - 2);
  __syncthreads();
  // Step i multiplies by Jt[hi-1-i], read from buffer i % 2.  Buffer (i + 1) % 2 was last read in
  // step i - 1 (or above, for P), which every wave has left, so the tile of step i + 1 may be
  // written to it during step i; the registers then take the tile of step i + 2.
  const int steps = hi - lo;
  for (int i = 0; i < steps; i += 2) {
    reduce_h128_step(As0, As1, tile(hi - 3 - i), pre, tid, l32, hsel, P, Q);
    __syncthreads();
    if (i + 1 < steps) {
      reduce_h128_step(As1, As0, tile(hi - 4 - i), pre, tid, l32, hsel, Q, P);
      __syncthreads();
    }
  }
  // an odd number of steps leaves the product in Q
  float* dst = tot + ((size_t)seg * B + b) * HH + 32 * wave + l32;
  const bool inQ = (steps & 1) != 0;              // uniform
#pragma unroll
  for (int kb = 0; kb < 4; ++kb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 32 * kb + 8 * (v >> 2) + 4 * hsel + (v & 3);
      dst[row * H] = inQ ? Q[kb][v] : P[kb][v];
    }
}

// v <- Jt[t] v for t = hi..lo, writing g[t] = v to G[t-1] (g0 when t == 0).
// Thread (r, c) = (tid / 32, tid % 32) holds columns 4c..4c+3 of rows r, r+8, ..., r+120; the 32
// threads of a row group keep their slice of v in registers and reduce their partial sums with
// a halving exchange (16 + 8 + 4 + 2 + 1 shuffles instead of 5 per row).
template <bool GEN>
__global__ void __launch_bounds__(kThreads)
apply_h128_kernel(int T, int B, int t_min, int S, int seg_begin, const float* __restrict__ Jt,
                  const float* __restrict__ vin, int vin_is_seed, float* __restrict__ G,
                  float* __restrict__ g0, float* __restrict__ v_out, const float* __restrict__ coef,
                  const float* __restrict__ wT) {
  __shared__ __attribute__((aligned(16))) float vs[2][H];
  // this kernel may share a compute unit with the matrix-core kernel of the pipelined form
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x;
  const int c = tid & 31, r = tid >> 5;
  const int seg = seg_begin + blockIdx.x;
  const int b = blockIdx.y;
  int lo, hi;
  seg_bounds(T, t_min, S, seg, lo, hi);
  const float* vsrc = vin_is_seed ? vin + (size_t)b * H : vin + ((size_t)seg * B + b) * H;
  if (tid < H) vs[0][tid] = vsrc[tid];
  v4f pre[GEN ? 1 : kChunks];
  // Generated form (GRU, Appendix E): Jt v = W_hr^T (a . v) + W_hn^T (c . v) + W_hz^T (e . v) + z . v,
  // three products with matrices that do not change; no tile is formed.  The thread keeps the
  // 3 x 16 weight pieces of its places, scales its four entries of v by a, c and e, and the lane
  // that ends up with a row's sum adds that row's z v.
  GruWeights gw;
  GruCoef cf;
  // the row whose sum this lane writes if it is a writer (c even): bit 4 of c chose q bit 3,
  // bit 3 -> q bit 2, bit 2 -> q bit 1, bit 1 -> q bit 0
  const int row = r + 8 * (((c >> 4) & 1) * 8 + ((c >> 3) & 1) * 4 + ((c >> 2) & 1) * 2 + ((c >> 1) & 1));
  float zrow = 0.f;
  if (GEN) {
    load_gru_weights(wT, tid, gw);
    cf = load_gru_coef(coef, (size_t)hi * B + b, tid);
    zrow = coef[((size_t)hi * B + b) * 4 * H + 3 * H + row];
  } else {
    const float* src = Jt + ((size_t)hi * B + b) * HH;
#pragma unroll
    for (int q = 0; q < kChunks; ++q) pre[q] = reinterpret_cast<const v4f*>(src)[tid + q * kThreads];
  }
  __syncthreads();
  int cur = 0;
  for (int t = hi; t >= lo; --t) {
    const v4f x = *reinterpret_cast<const v4f*>(&vs[cur][4 * c]);
    float part[kChunks];
    float diag = 0.f;
    if (GEN) {
      const v4f xa = x * cf.a, xc = x * cf.c, xe = x * cf.e;
      diag = zrow * vs[cur][row];
#pragma unroll
      for (int q = 0; q < kChunks; ++q) {       // row r + 8 q
        float acc = gw.r[q][0] * xa[0];
#pragma unroll
        for (int u = 1; u < 4; ++u) acc += gw.r[q][u] * xa[u];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc += gw.n[q][u] * xc[u];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc += gw.z[q][u] * xe[u];
        part[q] = acc;
      }
    } else {
#pragma unroll
      for (int q = 0; q < kChunks; ++q) {       // row r + 8 q
        const v4f m = pre[q];
        part[q] = (m[0] * x[0] + m[1] * x[1]) + (m[2] * x[2] + m[3] * x[3]);
      }
    }
    if (t - 1 >= lo) {
      if (GEN) {
        cf = load_gru_coef(coef, (size_t)(t - 1) * B + b, tid);
        zrow = coef[((size_t)(t - 1) * B + b) * 4 * H + 3 * H + row];
      } else {
        const float* src = Jt + ((size_t)(t - 1) * B + b) * HH;
#pragma unroll
        for (int q = 0; q < kChunks; ++q) pre[q] = reinterpret_cast<const v4f*>(src)[tid + q * kThreads];
      }
    }
    // halving exchange over the 32 lanes of the row group: after the step on lane bit k a lane
    // keeps the rows whose index bit matches its own bit k and has added what its partner (a
    // lane with the other bit k) held for them.  Bit 4 crosses the rows of 16 lanes and goes
    // through LDS; the others stay in the vector pipe.
#define BPPSA_HALVE(n, m, GET)                                      \
    {                                                               \
      const bool upper = (c & (m)) != 0;                            \
      _Pragma("unroll") for (int q = 0; q < (n); ++q) {             \
        const float mine = upper ? part[q + (n)] : part[q];         \
        const float send = upper ? part[q] : part[q + (n)];         \
        part[q] = mine + GET(send);                                 \
      }                                                             \
    }
#define BPPSA_GET16(x) __shfl_xor((x), 16)
    BPPSA_HALVE(8, 16, BPPSA_GET16)
    BPPSA_HALVE(4, 8, dpp_from<kDppMirror>)
    BPPSA_HALVE(2, 4, dpp_from<kDppHalfMirror>)
    BPPSA_HALVE(1, 2, dpp_from<kDppXor2>)
#undef BPPSA_GET16
#undef BPPSA_HALVE
    // lanes c and c ^ 1 now hold the two halves of the sum of row `row`
    const float sum = part[0] + dpp_from<kDppXor1>(part[0]) + diag;
    float* dst = (t >= 1) ? G + ((size_t)(t - 1) * B + b) * H : g0 + (size_t)b * H;
    if ((c & 1) == 0) {
      vs[cur ^ 1][row] = sum;
      dst[row] = sum;
    }
    __syncthreads();
    cur ^= 1;
  }
  if (v_out && tid < H) v_out[(size_t)b * H + tid] = vs[cur][tid];
}

// The seed-side stretch of a long chain: v <- Jt[t] v for t = hi..lo with one workgroup of 1024
// threads per sample, writing g[t] = v to G[t-1] (g0 when t == 0) and the last vector to v_out.
// Nothing here is parallel over t, so a step must be short: thread (r, c) = (tid / 32, tid % 32)
// holds columns 4c..4c+3 of rows r, r+32, r+64, r+96 (four 16-byte pieces per tile) and the 32
// partial sums of a row meet in six exchanges.  Sixteen waves fill a compute unit's registers:
// the workgroup has the unit to itself.
constexpr int kChainThreads = 1024;
constexpr int kChainPieces = HH / 4 / kChainThreads;   // 4

// partial sums part[q] of rows r + 32 q over the thread's four columns -> the row sum, held by
// the eight lanes c with the same c / 8; returns the row and leaves the sum in `sum`
__device__ __forceinline__ int chain_row_sum(float (&part)[kChainPieces], int r, int c, float& sum) {
  // halving exchange: lane bit 4 keeps the rows with q bit 1 equal to it (through LDS: the partner
  // is in the other row of 16 lanes), lane bit 3 those with q bit 0; the eight lanes of a half
  // row then add up
  {
    const bool upper = (c & 16) != 0;
    const float m0 = upper ? part[2] : part[0], s0 = upper ? part[0] : part[2];
    const float m1 = upper ? part[3] : part[1], s1 = upper ? part[1] : part[3];
    part[0] = m0 + __shfl_xor(s0, 16);
    part[1] = m1 + __shfl_xor(s1, 16);
  }
  {
    const bool upper = (c & 8) != 0;
    const float m0 = upper ? part[1] : part[0], s0 = upper ? part[0] : part[1];
    part[0] = m0 + dpp_from<kDppMirror>(s0);
  }
  sum = part[0];
  sum += dpp_from<kDppXor1>(sum);
  sum += dpp_from<kDppXor2>(sum);
  sum += dpp_from<kDppHalfMirror>(sum);
  return r + 32 * (((c >> 4) & 1) * 2 + ((c >> 3) & 1));
}

// Stored Jacobians: kChainDepth tiles are in flight in registers.  (A compute unit draws about
// 50 GB/s from memory however many requests it has outstanding, so a step of this form takes
// 1.3 us: six tiles in flight are more than that needs.)
constexpr int kChainDepth = 6;

__global__ void __launch_bounds__(kChainThreads)
chain_h128_kernel(int B, int lo, int hi, const float* __restrict__ Jt, const float* __restrict__ seed,
                  float* __restrict__ G, float* __restrict__ g0, float* __restrict__ v_out) {
  __shared__ __attribute__((aligned(16))) float vs[2][H];
  const int tid = threadIdx.x;
  const int c = tid & 31, r = tid >> 5;
  const int b = blockIdx.x;
  if (tid < H) vs[0][tid] = seed[(size_t)b * H + tid];
  v4f pre[kChainDepth][kChainPieces];
  auto request = [&](int slot, int t) {          // t below lo: a tile nobody uses, no branch
    const v4f* src = reinterpret_cast<const v4f*>(Jt + ((size_t)max(t, lo) * B + b) * HH);
#pragma unroll
    for (int q = 0; q < kChainPieces; ++q) pre[slot][q] = src[tid + q * kChainThreads];
  };
#pragma unroll
  for (int k = 0; k < kChainDepth; ++k) request(k, hi - k);
  __syncthreads();
  int cur = 0;
  for (int t0 = hi; t0 >= lo; t0 -= kChainDepth) {
#pragma unroll
    for (int k = 0; k < kChainDepth; ++k) {
      const int t = t0 - k;
      if (t < lo) break;                          // uniform
      const v4f x = *reinterpret_cast<const v4f*>(&vs[cur][4 * c]);
      float part[kChainPieces];
#pragma unroll
      for (int q = 0; q < kChainPieces; ++q) {    // row r + 32 q
        const v4f m = pre[k][q];
        part[q] = (m[0] * x[0] + m[1] * x[1]) + (m[2] * x[2] + m[3] * x[3]);
      }
      request(k, t - kChainDepth);
      float sum;
      const int row = chain_row_sum(part, r, c, sum);
      float* dst = (t >= 1) ? G + ((size_t)(t - 1) * B + b) * H : g0 + (size_t)b * H;
      if ((c & 7) == 0) {
        vs[cur ^ 1][row] = sum;
        dst[row] = sum;
      }
      __syncthreads();
      cur ^= 1;
    }
  }
  if (v_out && tid < H) v_out[(size_t)b * H + tid] = vs[cur][tid];
}

// Generated Jacobians (GRU, Appendix E).  With Jt = W_hr^T diag(a) + W_hn^T diag(c) + W_hz^T diag(e)
// + diag(z), a step is Jt v = W_hr^T (a . v) + W_hn^T (c . v) + W_hz^T (e . v) + z . v: three products
// with matrices that do not change, so no tile is formed at all.  The thread keeps the 3 x 4 weight
// pieces of its places in registers, scales its four entries of v by a, c and e, and spends three
// multiply-adds per entry of a tile.  The coefficient vectors of kChainBlock steps at a time (2 KB
// per step) go through LDS, the next block already in flight in registers while one is in use.
constexpr int kChainBlock = 8;

__global__ void __launch_bounds__(kChainThreads)
chain_h128_gen_kernel(int B, int lo, int hi, const float* __restrict__ seed, float* __restrict__ G,
                      float* __restrict__ g0, float* __restrict__ v_out, const float* __restrict__ coef,
                      const float* __restrict__ wT) {
  __shared__ __attribute__((aligned(16))) float vs[2][H];
  __shared__ __attribute__((aligned(16))) float cfs[2][kChainBlock][4 * H];
  const int tid = threadIdx.x;
  const int c = tid & 31, r = tid >> 5;
  const int b = blockIdx.x;
  if (tid < H) vs[0][tid] = seed[(size_t)b * H + tid];
  v4f wr[kChainPieces], wn[kChainPieces], wz[kChainPieces];
#pragma unroll
  for (int q = 0; q < kChainPieces; ++q) {
    const int e = tid + q * kChainThreads;
    wr[q] = reinterpret_cast<const v4f*>(wT)[e];
    wn[q] = reinterpret_cast<const v4f*>(wT + HH)[e];
    wz[q] = reinterpret_cast<const v4f*>(wT + 2 * HH)[e];
  }
  // the block of steps t0 .. t0 - 7: thread (j, p) = (tid / 128, tid % 128) moves piece p of step
  // t0 - j (clamped to lo: rows nobody uses)
  const int bj = tid >> 7, bp = tid & 127;
  v4f in;
  auto request = [&](int t0) {
    in = reinterpret_cast<const v4f*>(coef + ((size_t)max(t0 - bj, lo) * B + b) * 4 * H)[bp];
  };
  auto deposit = [&](int buf) { reinterpret_cast<v4f*>(&cfs[buf][bj][0])[bp] = in; };
  request(hi);
  deposit(0);
  request(hi - kChainBlock);
  __syncthreads();
  // the row this lane writes if it is one of the writers (c % 8 == 0)
  const int row = r + 32 * (((c >> 4) & 1) * 2 + ((c >> 3) & 1));
  int cur = 0, buf = 0;
  for (int t0 = hi; t0 >= lo; t0 -= kChainBlock) {
    for (int j = 0; j < kChainBlock; ++j) {
      const int t = t0 - j;
      if (t < lo) break;                          // uniform
      const v4f x = *reinterpret_cast<const v4f*>(&vs[cur][4 * c]);
      const v4f* f = reinterpret_cast<const v4f*>(&cfs[buf][j][0]) + c;
      const v4f xa = x * f[0], xc = x * f[H / 4], xe = x * f[2 * (H / 4)];
      const float diag = cfs[buf][j][3 * H + row] * vs[cur][row];
      float part[kChainPieces];
#pragma unroll
      for (int q = 0; q < kChainPieces; ++q) {    // row r + 32 q
        float acc = wr[q][0] * xa[0];
#pragma unroll
        for (int u = 1; u < 4; ++u) acc += wr[q][u] * xa[u];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc += wn[q][u] * xc[u];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc += wz[q][u] * xe[u];
        part[q] = acc;
      }
      float sum;
      chain_row_sum(part, r, c, sum);
      sum += diag;
      float* dst = (t >= 1) ? G + ((size_t)(t - 1) * B + b) * H : g0 + (size_t)b * H;
      if ((c & 7) == 0) {
        vs[cur ^ 1][row] = sum;
        dst[row] = sum;
      }
      __syncthreads();
      cur ^= 1;
    }
    // the other buffer was last read in the block before this one, behind many barriers; the
    // barrier below puts its new contents in front of the next block's reads
    deposit(buf ^ 1);
    request(t0 - 2 * kChainBlock);
    __syncthreads();
    buf ^= 1;
  }
  if (v_out && tid < H) v_out[(size_t)b * H + tid] = vs[cur][tid];
}

}  // namespace

bppsa_status bppsa_reduce_h128(int T, int B, int t_min, int S, int seg_begin, int seg_count,
                               const float* Jt, float* tot, hipStream_t s, const bppsa_gru_tiles* gen) {
  if (seg_count <= 0) return BPPSA_OK;
  if (gen) return bppsa_reduce_h128_gen(T, B, t_min, S, seg_begin, seg_count, tot, s, gen);
  const size_t lds = (size_t)2 * H * LS * sizeof(float);
  // set on every call: the attribute belongs to the current device's copy of the kernel, and the
  // library keeps no per-process record of which devices it has run on
  BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)reduce_h128_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
  reduce_h128_kernel<<<dim3(seg_count, B), kThreads, lds, s>>>(T, B, t_min, S, seg_begin, Jt, tot);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_apply_h128(int T, int B, int t_min, int S, int seg_begin, int seg_count,
                              const float* Jt, const float* vin, int vin_is_seed, float* G, float* g0,
                              float* v_out, hipStream_t s, const bppsa_gru_tiles* gen) {
  if (seg_count <= 0) return BPPSA_OK;
  if (gen)
    apply_h128_kernel<true><<<dim3(seg_count, B), kThreads, 0, s>>>(T, B, t_min, S, seg_begin, nullptr, vin,
                                                                    vin_is_seed, G, g0, v_out, gen->coef, gen->wT);
  else
    apply_h128_kernel<false><<<dim3(seg_count, B), kThreads, 0, s>>>(T, B, t_min, S, seg_begin, Jt, vin,
                                                                     vin_is_seed, G, g0, v_out, nullptr, nullptr);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_chain_h128(int B, int lo, int hi, const float* Jt, const float* seed, float* G, float* g0,
                              float* v_out, hipStream_t s, const bppsa_gru_tiles* gen) {
  if (hi < lo) return BPPSA_OK;
  if (gen)
    chain_h128_gen_kernel<<<B, kChainThreads, 0, s>>>(B, lo, hi, seed, G, g0, v_out, gen->coef, gen->wT);
  else
    chain_h128_kernel<<<B, kChainThreads, 0, s>>>(B, lo, hi, Jt, seed, G, g0, v_out);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
