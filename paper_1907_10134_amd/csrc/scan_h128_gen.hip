// H = 128 segment totals with the GRU Jacobians generated instead of read (the reduce step of
// bppsa_gru_scan_fused).
//
// A thread owns the same sixteen 16-byte pieces of every tile and keeps the matching 3 x 16
// pieces of the transposed recurrent weights in registers for the whole segment, so a tile costs
// it four coefficient reads and 192 multiply-adds.  With 192 registers gone to the weights the
// running product cannot stay in registers as it does in the kernel that reads its tiles: it
// goes through LDS, transposed, next to the generated tile.  (Streaming the weights from the
// cache instead, so that this kernel could share the other one's layout, was measured: 12 %
// slower per launch.)
#include "scan_h128_common.h"

namespace {

// P <- J P for J = Jt[hi-1], ..., Jt[lo], starting from P = Jt[hi]; tot[seg][b] = P.
//
// v_mfma_f32_32x32x2_f32 contracts two k values per issue: lane l supplies A[i = l % 32][k(l / 32)]
// and B[k(l / 32)][j = l % 32], and holds D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32] in
// accumulator register v.  Any assignment of the 128 k values to (issue, lane half) is valid as
// long as A and B agree; here issue 4 g + s of lane half h takes k = 8 g + 4 h + s, so that one
// 16-byte LDS read per operand feeds four issues.  A is stored [i][k] and the running product
// is stored transposed, [j][k], which is also the order in which the accumulators come out.
// Each of the four waves owns a 64 x 64 quadrant of the product (2 x 2 MFMA blocks).
__global__ void __launch_bounds__(kThreads, 1)
reduce_h128_gen_kernel(int T, int B, int t_min, int S, int seg_begin, float* __restrict__ tot,
                       const float* __restrict__ coef, const float* __restrict__ wT) {
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
  load_gru_weights(wT, tid, gw);
  GruCoef cf = load_gru_coef(coef, (size_t)hi * B + b, tid);
  // P = Jt[hi], written transposed (once per segment)
#pragma unroll
  for (int r = 0; r < kChunks; ++r) {
    const int e = tid + r * kThreads;
    const int k = e >> 5, j4 = (e & 31) * 4;
    const v4f x = gru_piece(gw, cf, tid, r);
    Bt[(j4 + 0) * LS + k] = x[0];
    Bt[(j4 + 1) * LS + k] = x[1];
    Bt[(j4 + 2) * LS + k] = x[2];
    Bt[(j4 + 3) * LS + k] = x[3];
  }
  v16f acc[2][2];
  if (hi - 1 >= lo) cf = load_gru_coef(coef, (size_t)(hi - 1) * B + b, tid);
  for (int t = hi - 1; t >= lo; --t) {
    // the generated Jacobian becomes the A operand
#pragma unroll
    for (int r = 0; r < kChunks; ++r) {
      const int e = tid + r * kThreads;
      *reinterpret_cast<v4f*>(As + (e >> 5) * LS + (e & 31) * 4) = gru_piece(gw, cf, tid, r);
    }
    __syncthreads();
    if (t - 1 >= lo) cf = load_gru_coef(coef, (size_t)(t - 1) * B + b, tid);
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

}  // namespace

bppsa_status bppsa_reduce_h128_gen(int T, int B, int t_min, int S, int seg_begin, int seg_count, float* tot,
                                   hipStream_t s, const bppsa_gru_tiles* gen) {
  if (seg_count <= 0) return BPPSA_OK;
  const size_t lds = (size_t)2 * H * LS * sizeof(float);
  // set on every call: the attribute belongs to the current device's copy of the kernel, and the
  // library keeps no per-process record of which devices it has run on
  BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)reduce_h128_gen_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
  reduce_h128_gen_kernel<<<dim3(seg_count, B), kThreads, lds, s>>>(T, B, t_min, S, seg_begin, tot, gen->coef, gen->wT);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
