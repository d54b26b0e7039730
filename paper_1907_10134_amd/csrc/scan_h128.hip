// H = 128 kernels of the segmented scan (the GRU size of the long-sequence workload).
//
// At this size a matrix-matrix node of the up-sweep (Algorithm 1, a[r] <- a[r] a[l]) is
// 4.2 MFLOP against 64 KB of operand traffic: it belongs on the matrix cores.  The reduce
// kernel keeps the running product of a segment in MFMA accumulators and streams one
// transposed Jacobian per step through LDS; the apply kernel walks a segment with
// matrix-vector products (the down-sweep side), streaming each Jacobian once with the next
// one already in flight.
#include "bppsa_internal.h"
#include "scan_plan.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int H = 128;
constexpr int HH = H * H;
constexpr int LS = H + 4;            // LDS row stride in floats: rows 8 apart share a bank, so the
                                     // 16-byte reads of 8 consecutive rows tile all 32 banks
constexpr int kThreads = 256;
constexpr int kChunks = HH / 4 / kThreads;   // 16-byte pieces of a tile per thread (16)

__device__ __forceinline__ void seg_bounds(int T, int t_min, int S, int seg, int& lo, int& hi) {
  lo = t_min + seg * S;
  hi = min(lo + S, T) - 1;
}

// GRU transposed Jacobians generated in place of being read (Appendix E):
//   Jt[i][j] = W_hr[j][i] a_j + W_hn[j][i] c_j + W_hz[j][i] e_j + [i == j] z_j
// with the per-step coefficient vectors (a, c, e, z) of bppsa_gru_coefs_h128 and the three
// recurrent matrices transposed, wT[g][i][j] (g = r, n, z).  Both kernels below give thread tid
// the 16-byte pieces e = tid + 256 q of a tile, i.e. rows tid / 32 + 8 q and columns
// 4 (tid % 32) .. + 3: the same places in every tile, so the thread keeps its 3 x 16 pieces of
// the weights in registers for the whole segment and a tile costs it four coefficient reads and
// 192 multiply-adds instead of 256 bytes from HBM.
struct GruWeights {
  v4f r[kChunks], n[kChunks], z[kChunks];
};
struct GruCoef {
  v4f a, c, e, z;
};

__device__ __forceinline__ void load_gru_weights(const float* __restrict__ wT, int tid, GruWeights& w) {
#pragma unroll
  for (int q = 0; q < kChunks; ++q) {
    const int e = tid + q * kThreads;
    w.r[q] = reinterpret_cast<const v4f*>(wT)[e];
    w.n[q] = reinterpret_cast<const v4f*>(wT + HH)[e];
    w.z[q] = reinterpret_cast<const v4f*>(wT + 2 * HH)[e];
  }
}
__device__ __forceinline__ GruCoef load_gru_coef(const float* __restrict__ coef, size_t row, int tid) {
  const v4f* c = reinterpret_cast<const v4f*>(coef + row * 4 * H) + (tid & 31);
  return GruCoef{c[0], c[H / 4], c[2 * (H / 4)], c[3 * (H / 4)]};
}
__device__ __forceinline__ v4f gru_piece(const GruWeights& w, const GruCoef& cf, int tid, int q) {
  v4f o = w.r[q] * cf.a + w.n[q] * cf.c + w.z[q] * cf.e;
  const int d = (tid >> 5) + 8 * q - 4 * (tid & 31);      // row minus first column of the piece
#pragma unroll
  for (int u = 0; u < 4; ++u) o[u] += (d == u) ? cf.z[u] : 0.f;
  return o;
}

// P <- J P for J = Jt[hi-1], ..., Jt[lo], starting from P = Jt[hi]; tot[seg][b] = P.
//
// v_mfma_f32_32x32x2_f32 contracts two k values per issue: lane l supplies A[i = l % 32][k(l / 32)]
// and B[k(l / 32)][j = l % 32], and holds D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32] in
// accumulator register v.  Any assignment of the 128 k values to (issue, lane half) is valid as
// long as A and B agree; here issue 4 g + s of lane half h takes k = 8 g + 4 h + s, so that one
// 16-byte LDS read per operand feeds four issues.  A is stored [i][k] and the running product
// is stored transposed, [j][k], which is also the order in which the accumulators come out.
// Each of the four waves owns a 64 x 64 quadrant of the product (2 x 2 MFMA blocks).
// GEN: the Jacobians are generated from (coef, wT) instead of read from Jt.
template <bool GEN>
__global__ void __launch_bounds__(kThreads, 1)
reduce_h128_kernel(int T, int B, int t_min, int S, int seg_begin, const float* __restrict__ Jt,
                   float* __restrict__ tot, const float* __restrict__ coef, const float* __restrict__ wT) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* As = smem;                 // [128][LS]  A[i][k]
  float* Bt = smem + H * LS;        // [128][LS]  P^T: Bt[j][k] = P[k][j]
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wr = wave >> 1, wc = wave & 1;
  const int l32 = lane & 31, hsel = lane >> 5;
  const int seg = seg_begin + blockIdx.x;
  const int b = blockIdx.y;
  int lo, hi;
  seg_bounds(T, t_min, S, seg, lo, hi);

  GruWeights gw;
  GruCoef cf;
  if (GEN) {
    load_gru_weights(wT, tid, gw);
    cf = load_gru_coef(coef, (size_t)hi * B + b, tid);
  }
  // P = Jt[hi], written transposed (once per segment)
  {
    const float* src = GEN ? nullptr : Jt + ((size_t)hi * B + b) * HH;
#pragma unroll
    for (int r = 0; r < kChunks; ++r) {
      const int e = tid + r * kThreads;
      const int k = e >> 5, j4 = (e & 31) * 4;
      const v4f x = GEN ? gru_piece(gw, cf, tid, r) : reinterpret_cast<const v4f*>(src)[e];
      Bt[(j4 + 0) * LS + k] = x[0];
      Bt[(j4 + 1) * LS + k] = x[1];
      Bt[(j4 + 2) * LS + k] = x[2];
      Bt[(j4 + 3) * LS + k] = x[3];
    }
  }
  v16f acc[2][2];
  v4f pre[GEN ? 1 : kChunks];
  if (hi - 1 >= lo) {
    if (GEN) {
      cf = load_gru_coef(coef, (size_t)(hi - 1) * B + b, tid);
    } else {
      const float* src = Jt + ((size_t)(hi - 1) * B + b) * HH;
#pragma unroll
      for (int r = 0; r < kChunks; ++r) pre[r] = reinterpret_cast<const v4f*>(src)[tid + r * kThreads];
    }
  }
  for (int t = hi - 1; t >= lo; --t) {
    // the prefetched (or generated) Jacobian becomes the A operand
#pragma unroll
    for (int r = 0; r < kChunks; ++r) {
      const int e = tid + r * kThreads;
      *reinterpret_cast<v4f*>(As + (e >> 5) * LS + (e & 31) * 4) = GEN ? gru_piece(gw, cf, tid, r) : pre[r];
    }
    __syncthreads();
    if (t - 1 >= lo) {
      if (GEN) {
        cf = load_gru_coef(coef, (size_t)(t - 1) * B + b, tid);
      } else {
        const float* src = Jt + ((size_t)(t - 1) * B + b) * HH;
#pragma unroll
        for (int r = 0; r < kChunks; ++r) pre[r] = reinterpret_cast<const v4f*>(src)[tid + r * kThreads];
      }
    }
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
      for (int bj = 0; bj < 2; ++bj)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0.f;
    const float* arow = As + (64 * wr + l32) * LS + 4 * hsel;
    const float* brow = Bt + (64 * wc + l32) * LS + 4 * hsel;
    v4f a4[2][2], b4[2][2];
    a4[0][0] = *reinterpret_cast<const v4f*>(arow);
    a4[0][1] = *reinterpret_cast<const v4f*>(arow + 32 * LS);
    b4[0][0] = *reinterpret_cast<const v4f*>(brow);
    b4[0][1] = *reinterpret_cast<const v4f*>(brow + 32 * LS);
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      const int cur = g & 1;
      if (g < 15) {                               // operands of the next k group
        a4[cur ^ 1][0] = *reinterpret_cast<const v4f*>(arow + 8 * (g + 1));
        a4[cur ^ 1][1] = *reinterpret_cast<const v4f*>(arow + 32 * LS + 8 * (g + 1));
        b4[cur ^ 1][0] = *reinterpret_cast<const v4f*>(brow + 8 * (g + 1));
        b4[cur ^ 1][1] = *reinterpret_cast<const v4f*>(brow + 32 * LS + 8 * (g + 1));
      }
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
          for (int bj = 0; bj < 2; ++bj)
            acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[cur][bi][s], b4[cur][bj][s], acc[bi][bj], 0, 0, 0);
    }
    __syncthreads();                              // every wave has finished reading As and Bt
    if (t > lo) {
      // the product becomes the next B operand: accumulator registers 4 q .. 4 q + 3 are four
      // consecutive k of one column
#pragma unroll
      for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const v4f x = {acc[bi][bj][4 * q], acc[bi][bj][4 * q + 1], acc[bi][bj][4 * q + 2], acc[bi][bj][4 * q + 3]};
            *reinterpret_cast<v4f*>(Bt + (64 * wc + 32 * bj + l32) * LS + 64 * wr + 32 * bi + 8 * q + 4 * hsel) = x;
          }
    }
  }
  float* dst = tot + ((size_t)seg * B + b) * HH;
  if (hi > lo) {
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
      for (int bj = 0; bj < 2; ++bj)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = 64 * wr + 32 * bi + 8 * (v >> 2) + 4 * hsel + (v & 3);
          dst[row * H + 64 * wc + 32 * bj + l32] = acc[bi][bj][v];
        }
  } else {                                        // one-step segment: the total is Jt[hi] itself
    __syncthreads();
    for (int e = tid; e < HH; e += kThreads) dst[e] = Bt[(e & (H - 1)) * LS + (e >> 7)];
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
  const size_t lds = (size_t)2 * H * LS * sizeof(float);
  // set on every call: the attribute belongs to the current device's copy of the kernel, and the
  // library keeps no per-process record of which devices it has run on
  if (gen) {
    BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)reduce_h128_kernel<true>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    reduce_h128_kernel<true><<<dim3(seg_count, B), kThreads, lds, s>>>(T, B, t_min, S, seg_begin, nullptr, tot,
                                                                       gen->coef, gen->wT);
  } else {
    BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)reduce_h128_kernel<false>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    reduce_h128_kernel<false><<<dim3(seg_count, B), kThreads, lds, s>>>(T, B, t_min, S, seg_begin, Jt, tot,
                                                                        nullptr, nullptr);
  }
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
