// H = 128 kernels of the segmented scan (the GRU size of the long-sequence workload).
//
// At this size a matrix-matrix node of the up-sweep (Algorithm 1, a[r] <- a[r] a[l]) is
// 4.2 MFLOP against 64 KB of operand traffic: it belongs on the matrix cores.  The reduce
// kernel keeps the running product of a segment in registers, as MFMA results that are the next
// step's B operands, and streams one transposed Jacobian per step through LDS; the apply kernel
// walks a segment with matrix-vector products (the down-sweep side), streaming each Jacobian
// once with the next one already in flight.
//
// This file is compiled with MFMA results in ordinary vector registers (see the build script):
// an accumulation register cannot be a B operand.
#include "scan_h128_common.h"

namespace {

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
  GruWeights gw;
  GruCoef cf;
  if (GEN) {
    load_gru_weights(wT, tid, gw);
    cf = load_gru_coef(coef, (size_t)hi * B + b, tid);
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
#pragma unroll
    for (int q = 0; q < kChunks; ++q) {         // row r + 8 q
      const v4f m = GEN ? gru_piece(gw, cf, tid, q) : pre[q];
      part[q] = (m[0] * x[0] + m[1] * x[1]) + (m[2] * x[2] + m[3] * x[3]);
    }
    if (t - 1 >= lo) {
      if (GEN) {
        cf = load_gru_coef(coef, (size_t)(t - 1) * B + b, tid);
      } else {
        const float* src = Jt + ((size_t)(t - 1) * B + b) * HH;
#pragma unroll
        for (int q = 0; q < kChunks; ++q) pre[q] = reinterpret_cast<const v4f*>(src)[tid + q * kThreads];
      }
    }
    // halving exchange over the 32 lanes of the row group: after the step with mask m a lane
    // keeps the rows whose index bit matches its own lane bit
#define BPPSA_HALVE(n, m)                                           \
    {                                                               \
      const bool upper = (c & (m)) != 0;                            \
      _Pragma("unroll") for (int q = 0; q < (n); ++q) {             \
        const float mine = upper ? part[q + (n)] : part[q];         \
        const float send = upper ? part[q] : part[q + (n)];         \
        part[q] = mine + __shfl_xor(send, (m));                     \
      }                                                             \
    }
    BPPSA_HALVE(8, 16)
    BPPSA_HALVE(4, 8)
    BPPSA_HALVE(2, 4)
    BPPSA_HALVE(1, 2)
#undef BPPSA_HALVE
    // lanes c and c ^ 1 now hold the two halves of row r + 8 * rowsel
    const float sum = part[0] + __shfl_xor(part[0], 1);
    // row index: bit 4 of c chose q bit 3, bit 3 -> q bit 2, bit 2 -> q bit 1, bit 1 -> q bit 0
    const int qsel = ((c >> 4) & 1) * 8 + ((c >> 3) & 1) * 4 + ((c >> 2) & 1) * 2 + ((c >> 1) & 1);
    const int row = r + 8 * qsel;
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
