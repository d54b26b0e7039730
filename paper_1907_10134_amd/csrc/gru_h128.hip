// H = 128 GRU kernels: the gate pre-activations are a [rows x 128] x [128 x 384] product and
// run on the matrix cores; the Jacobians (Appendix E) are then streamed out with the three
// recurrent weight matrices held in registers.
#include "bppsa_internal.h"
#include "scan_plan.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int H = 128;
constexpr int LS = H + 4;          // LDS row stride of the staged hidden states (bank spread)
constexpr int kBatch = 32;         // (t, b) rows per gate tile = one MFMA block of rows

__device__ __forceinline__ float sigmoidf_(float a) { return 1.0f / (1.0f + expf(-a)); }

// Gates of kBatch rows for the 32 hidden units j = 32 w + (lane % 32), computed by one wave.
//   R = W_hr h' + b_hr, Z = W_hz h' + b_hz, M = W_hn h' + b_hn   (32x32x2 fp32 MFMA, K = 128)
//   r = sigmoid(W_ir x + b_ir + R), z = sigmoid(W_iz x + b_iz + Z), n = tanh(W_in x + b_in + r M)
// hp: LDS [kBatch][LS], rows past the end zero-filled.  The weights are read straight from
// global memory (196 KB, cache resident): lane l needs W[gate row 32 w + l % 32][4 consecutive k].
// emit(row, j, r, z, n, M, h'[row][j]) is called for every valid row of the tile.
template <class F>
__device__ __forceinline__ void gru_gates_h128(int w, int lane, long long row0, long long rows, int I,
                                               const float* hp, const float* __restrict__ x,
                                               const float* __restrict__ w_ih, const float* __restrict__ w_hh,
                                               const float* __restrict__ b_ih, const float* __restrict__ b_hh,
                                               F&& emit) {
  const int l32 = lane & 31, hs = lane >> 5;
  const int j = 32 * w + l32;
  v16f acc[3];
#pragma unroll
  for (int g = 0; g < 3; ++g)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[g][v] = 0.f;
  const float* arow = hp + l32 * LS + 4 * hs;
  const float* wrow = w_hh + (size_t)j * H + 4 * hs;
#pragma unroll 4
  for (int g8 = 0; g8 < 16; ++g8) {
    const v4f a4 = *reinterpret_cast<const v4f*>(arow + 8 * g8);
    v4f b4[3];
#pragma unroll
    for (int g = 0; g < 3; ++g) b4[g] = *reinterpret_cast<const v4f*>(wrow + (size_t)g * H * H + 8 * g8);
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int g = 0; g < 3; ++g)
        acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[s], b4[g][s], acc[g], 0, 0, 0);
  }
  const float bhr = b_hh ? b_hh[j] : 0.f, bhz = b_hh ? b_hh[H + j] : 0.f, bhn = b_hh ? b_hh[2 * H + j] : 0.f;
  const float bir = b_ih ? b_ih[j] : 0.f, biz = b_ih ? b_ih[H + j] : 0.f, bin = b_ih ? b_ih[2 * H + j] : 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = 8 * (v >> 2) + 4 * hs + (v & 3);
    if (row0 + row < rows) {
      float ir = bir, iz = biz, in = bin;
      const float* xr = x + (size_t)(row0 + row) * I;
      for (int i = 0; i < I; ++i) {
        const float xv = xr[i];
        ir += w_ih[(size_t)j * I + i] * xv;
        iz += w_ih[(size_t)(H + j) * I + i] * xv;
        in += w_ih[(size_t)(2 * H + j) * I + i] * xv;
      }
      const float r = sigmoidf_(ir + (acc[0][v] + bhr));
      const float z = sigmoidf_(iz + (acc[1][v] + bhz));
      const float M = acc[2][v] + bhn;
      const float n = tanhf(in + r * M);
      emit(row, j, r, z, n, M, hp[row * LS + j]);
    }
  }
}

// Stage h'[row0 .. row0 + kBatch) into LDS, zero-filling rows past the end.
template <int THREADS>
__device__ __forceinline__ void stage_hidden(int tid, long long row0, long long rows,
                                             const float* __restrict__ h, float* hp) {
#pragma unroll
  for (int q = 0; q < kBatch * (H / 4) / THREADS; ++q) {
    const int e = tid + q * THREADS;
    const int row = e >> 5, c4 = (e & 31) * 4;
    v4f v = {0.f, 0.f, 0.f, 0.f};
    if (row0 + row < rows) v = *reinterpret_cast<const v4f*>(h + (size_t)(row0 + row) * H + c4);
    *reinterpret_cast<v4f*>(hp + row * LS + c4) = v;
  }
}

// Jt[i][j] = W_hr[j][i] a_j + W_hn[j][i] c_j + W_hz[j][i] e_j + [i == j] z_j   (Appendix E)
// Persistent workgroups of 512 threads.  Thread (i0 = tid / 32, j4 = 4 (tid % 32)) owns the
// elements (i0 + 16 q, j4 .. j4 + 3), q < 8, of every tile and keeps the matching 3 x 32 weights
// in registers, so a tile costs 16 coefficient reads from LDS, 96 multiply-adds and eight
// 16-byte streaming stores per thread.
constexpr int kJacThreads = 512;

__global__ void __launch_bounds__(kJacThreads, 2)
gru_jacobians_h128_kernel(long long rows, int I, long long nbatch, const float* __restrict__ h,
                          const float* __restrict__ x, const float* __restrict__ w_ih,
                          const float* __restrict__ w_hh, const float* __restrict__ b_ih,
                          const float* __restrict__ b_hh, float* __restrict__ Jt) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* hp = smem;                    // [kBatch][LS]
  float* coef = smem + kBatch * LS;    // [kBatch][4][H]: a, c, e, z
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int j4 = (tid & 31) * 4, i0 = tid >> 5;
  v4f wr[8], wn[8], wz[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int i = i0 + 16 * q;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      wr[q][u] = w_hh[(size_t)(j4 + u) * H + i];
      wz[q][u] = w_hh[(size_t)(H + j4 + u) * H + i];
      wn[q][u] = w_hh[(size_t)(2 * H + j4 + u) * H + i];
    }
  }
  for (long long batch = blockIdx.x; batch < nbatch; batch += gridDim.x) {
    const long long row0 = batch * kBatch;
    const int nrows = (int)((rows - row0 < kBatch) ? (rows - row0) : kBatch);
    stage_hidden<kJacThreads>(tid, row0, rows, h, hp);
    __syncthreads();
    if (wave < 4) {
      gru_gates_h128(wave, lane, row0, rows, I, hp, x, w_ih, w_hh, b_ih, b_hh,
                     [&](int row, int j, float r, float z, float n, float M, float hprev) {
                       const float dn = (1.f - z) * (1.f - n * n);
                       float* c = coef + row * 4 * H;
                       c[j] = dn * M * r * (1.f - r);
                       c[H + j] = dn * r;
                       c[2 * H + j] = (hprev - n) * z * (1.f - z);
                       c[3 * H + j] = z;
                     });
    }
    __syncthreads();
    for (int r = 0; r < nrows; ++r) {
      const float* c = coef + r * 4 * H + j4;
      const v4f ca = *reinterpret_cast<const v4f*>(c);
      const v4f cc = *reinterpret_cast<const v4f*>(c + H);
      const v4f ce = *reinterpret_cast<const v4f*>(c + 2 * H);
      const v4f cz = *reinterpret_cast<const v4f*>(c + 3 * H);
      float* dst = Jt + (size_t)(row0 + r) * H * H + j4;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int i = i0 + 16 * q;
        v4f o = wr[q] * ca + wn[q] * cc + wz[q] * ce;
#pragma unroll
        for (int u = 0; u < 4; ++u) o[u] += (i == j4 + u) ? cz[u] : 0.f;
        __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(dst + (size_t)i * H));
      }
    }
    __syncthreads();                   // hp and coef are rewritten by the next batch
  }
}

// The coefficient vectors of the closed form above for every (t, b) row, coef[row][4][H] =
// (a, c, e, z), for a scan that generates the Jacobians itself instead of reading them.
__global__ void __launch_bounds__(256)
gru_coefs_h128_kernel(long long rows, int I, const float* __restrict__ h, const float* __restrict__ x,
                      const float* __restrict__ w_ih, const float* __restrict__ w_hh,
                      const float* __restrict__ b_ih, const float* __restrict__ b_hh, float* __restrict__ coef) {
  __shared__ __attribute__((aligned(16))) float hp[kBatch * LS];
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * kBatch;
  stage_hidden<256>(tid, row0, rows, h, hp);
  __syncthreads();
  gru_gates_h128(tid >> 6, tid & 63, row0, rows, I, hp, x, w_ih, w_hh, b_ih, b_hh,
                 [&](int row, int j, float r, float z, float n, float M, float hprev) {
                   const float dn = (1.f - z) * (1.f - n * n);
                   float* c = coef + (size_t)(row0 + row) * 4 * H;
                   c[j] = dn * M * r * (1.f - r);
                   c[H + j] = dn * r;
                   c[2 * H + j] = (hprev - n) * z * (1.f - z);
                   c[3 * H + j] = z;
                 });
}

// wT[g][i][j] = W_hg[j][i] for g = r, n, z (the order of the coefficients a, c, e)
__global__ void __launch_bounds__(256)
gru_transpose_weights_h128_kernel(const float* __restrict__ w_hh, float* __restrict__ wT) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;      // over 3 * H * H
  if (e >= 3 * H * H) return;
  const int g = e / (H * H), rem = e - g * H * H;
  const int i = rem / H, j = rem - i * H;
  const int src_gate = g == 0 ? 0 : (g == 1 ? 2 : 1);       // w_hh rows are ordered r, z, n
  wT[e] = w_hh[((size_t)src_gate * H + j) * H + i];
}

// delta[row][0..4H) = (dR, dZ, dN, dM) for every (t, b) row, given g = dL/dh[t+1]: the chain
// rule through the cell of Section 4.2 with the gates recomputed as above.
constexpr int kDeltaThreads = 256;

__global__ void __launch_bounds__(kDeltaThreads)
gru_deltas_h128_kernel(long long rows, int I, const float* __restrict__ h, const float* __restrict__ x,
                       const float* __restrict__ G, const float* __restrict__ w_ih,
                       const float* __restrict__ w_hh, const float* __restrict__ b_ih,
                       const float* __restrict__ b_hh, float* __restrict__ delta) {
  __shared__ __attribute__((aligned(16))) float hp[kBatch * LS];
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * kBatch;
  stage_hidden<kDeltaThreads>(tid, row0, rows, h, hp);
  __syncthreads();
  gru_gates_h128(tid >> 6, tid & 63, row0, rows, I, hp, x, w_ih, w_hh, b_ih, b_hh,
                 [&](int row, int j, float r, float z, float n, float M, float hprev) {
                   const float gv = G[(size_t)(row0 + row) * H + j];
                   const float dN = gv * (1.f - z) * (1.f - n * n);
                   const float dZ = gv * (hprev - n) * z * (1.f - z);
                   float* d = delta + (size_t)(row0 + row) * 4 * H;
                   d[j] = dN * M * r * (1.f - r);
                   d[H + j] = dZ;
                   d[2 * H + j] = dN;
                   d[3 * H + j] = dN * r;
                 });
}

// Partial sums of the GRU parameter gradients (Eq. 2, summed over steps and samples):
//   dW_hh[g][c] = sum_rows Dh[row][g] h'[row][c],  db_hh[g] = sum_rows Dh[row][g],
//   dW_ih[g][i] = sum_rows Di[row][g] x[row][i],   db_ih[g] = sum_rows Di[row][g],
// with Dh = (dR, dZ, dM) and Di = (dR, dZ, dN).  The first is a [384 x rows] x [rows x 128]
// product: every wave owns a strip of 32 gates and a range of rows and accumulates the four
// 32 x 32 blocks of its strip with 32x32x2 fp32 MFMA, both operands coming straight from
// global memory (lane l supplies Dh[row][g0 + l % 32] and h'[row][32 cb + l % 32], the lane
// half choosing which of the two rows of the issue).  The bias and input columns are running
// sums of the A operand in the same lanes.  Each wave writes its own partial, laid out
// [3H][H + 1 + I + 1] like the generic kernel's, for the shared finishing kernel.
constexpr int kPartMaxI = 4;

__global__ void __launch_bounds__(256)
gru_param_partials_h128_kernel(long long rows, int I, int nsplit, long long rows_per_split,
                               const float* __restrict__ h, const float* __restrict__ x,
                               const float* __restrict__ delta, float* __restrict__ part) {
  const int lane = threadIdx.x & 63, l32 = lane & 31, hs = lane >> 5;
  const int split = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (split >= nsplit) return;                 // whole wave
  const int g0 = blockIdx.x * 32;
  const int W = H + 1 + I + 1;
  const int colh = (g0 < 2 * H) ? g0 + l32 : g0 + H + l32;   // dM sits after dN
  const int coli = g0 + l32;
  const long long r_begin = (long long)split * rows_per_split;
  long long r_end = r_begin + rows_per_split;
  if (r_end > rows) r_end = rows;
  v16f acc[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[cb][v] = 0.f;
  float sum_h = 0.f, sum_i = 0.f, sum_x[kPartMaxI];
#pragma unroll
  for (int i = 0; i < kPartMaxI; ++i) sum_x[i] = 0.f;
  for (long long r = r_begin; r < r_end; r += 16) {
    float a[8], ai[8], b[8][4], xv[8][kPartMaxI];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const long long row = r + 2 * u + hs;
      const bool ok = row < r_end;
      const float* d = delta + (size_t)row * 4 * H;
      a[u] = ok ? d[colh] : 0.f;
      ai[u] = ok ? d[coli] : 0.f;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) b[u][cb] = ok ? h[(size_t)row * H + 32 * cb + l32] : 0.f;
#pragma unroll
      for (int i = 0; i < kPartMaxI; ++i) xv[u][i] = (ok && i < I) ? x[(size_t)row * I + i] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u][cb], acc[cb], 0, 0, 0);
      sum_h += a[u];
      sum_i += ai[u];
#pragma unroll
      for (int i = 0; i < kPartMaxI; ++i) sum_x[i] += ai[u] * xv[u][i];
    }
  }
  float* dst = part + ((size_t)split * 3 * H + g0) * W;
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int g = 8 * (v >> 2) + 4 * hs + (v & 3);
      dst[(size_t)g * W + 32 * cb + l32] = acc[cb][v];
    }
  sum_h += __shfl_xor(sum_h, 32);
  sum_i += __shfl_xor(sum_i, 32);
#pragma unroll
  for (int i = 0; i < kPartMaxI; ++i) sum_x[i] += __shfl_xor(sum_x[i], 32);
  if (hs == 0) {
    float* drow = dst + (size_t)l32 * W;
    drow[H] = sum_h;
#pragma unroll
    for (int i = 0; i < kPartMaxI; ++i)
      if (i < I) drow[H + 1 + i] = sum_x[i];
    drow[H + 1 + I] = sum_i;
  }
}

// ---- the recurrence itself (bppsa_forward, GRU, H = 128) -------------------------------------------
// One workgroup of 1024 threads per sample walks the sequence.  Thread (r, c) = (tid / 32, tid % 32)
// keeps columns 4c..4c+3 of rows r, r+32, r+64, r+96 of W_hr, W_hz and W_hn in registers (48 values),
// multiplies them with its four entries of the state, and the 32 partial sums of a row meet in one
// LDS exchange (across rows of 16 lanes) and four DPP exchanges; the 128 threads that own a hidden
// unit then add the input part and the biases and apply the gates (Section 4.2).  A step costs two
// workgroup barriers and reads no weight from memory.
constexpr int kFwdThreads = 1024;
constexpr int kFwdMaxI = 8;

template <int CTRL>
__device__ __forceinline__ float fwd_dpp(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// part[q] = partial sum of row r + 32 q over the thread's four columns -> the sum of one row over all
// 128 columns, in each of the eight lanes c with the same c / 8; that row is
// r + 32 (2 (c / 16) + (c / 8) % 2).  (DPP controls: 0x140 row mirror, 0xB1 / 0x4E quad permutations
// [1,0,3,2] / [2,3,0,1], 0x141 half-row mirror; a partner with other low lane bits serves as well as
// the exact one, since only the sum over the group is wanted.)
__device__ __forceinline__ float fwd_row_sum(float (&part)[4], int c) {
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
    part[0] = m0 + fwd_dpp<0x140>(s0);
  }
  float sum = part[0];
  sum += fwd_dpp<0xB1>(sum);
  sum += fwd_dpp<0x4E>(sum);
  sum += fwd_dpp<0x141>(sum);
  return sum;
}

__global__ void __launch_bounds__(kFwdThreads)
gru_forward_h128_kernel(int T, int B, int I, const float* __restrict__ x, const float* __restrict__ w_ih,
                        const float* __restrict__ w_hh, const float* __restrict__ b_ih,
                        const float* __restrict__ b_hh, float* __restrict__ h) {
  __shared__ __attribute__((aligned(16))) float hs[2][H];
  __shared__ float gh[3][H];
  const int tid = threadIdx.x;
  const int c = tid & 31, r = tid >> 5;
  const int b = blockIdx.x;
  v4f w[3][4];
#pragma unroll
  for (int g = 0; g < 3; ++g)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      w[g][q] = *reinterpret_cast<const v4f*>(w_hh + (size_t)(g * H + r + 32 * q) * H + 4 * c);
  const int row = r + 32 * (((c >> 4) & 1) * 2 + ((c >> 3) & 1));
  // the threads that own a hidden unit: biases, input weights, and the inputs of the next step
  const int j = tid < H ? tid : 0;
  float bi[3], bh[3], wi[3][kFwdMaxI], xs[kFwdMaxI];
#pragma unroll
  for (int g = 0; g < 3; ++g) {
    bi[g] = b_ih ? b_ih[g * H + j] : 0.f;
    bh[g] = b_hh ? b_hh[g * H + j] : 0.f;
#pragma unroll
    for (int i = 0; i < kFwdMaxI; ++i) wi[g][i] = i < I ? w_ih[(size_t)(g * H + j) * I + i] : 0.f;
  }
#pragma unroll
  for (int i = 0; i < kFwdMaxI; ++i) xs[i] = i < I ? x[(size_t)b * I + i] : 0.f;     // x[0][b]
  if (tid < H) hs[0][tid] = h[(size_t)b * H + tid];
  __syncthreads();
  int cur = 0;
  for (int t = 1; t <= T; ++t) {
    const v4f hv = *reinterpret_cast<const v4f*>(&hs[cur][4 * c]);
#pragma unroll
    for (int g = 0; g < 3; ++g) {
      float part[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        part[q] = (w[g][q][0] * hv[0] + w[g][q][1] * hv[1]) + (w[g][q][2] * hv[2] + w[g][q][3] * hv[3]);
      const float sum = fwd_row_sum(part, c);
      if ((c & 7) == 0) gh[g][row] = sum;
    }
    float xn[kFwdMaxI];
#pragma unroll
    for (int i = 0; i < kFwdMaxI; ++i) xn[i] = (i < I && t < T) ? x[((size_t)t * B + b) * I + i] : 0.f;
    __syncthreads();
    if (tid < H) {
      float ai[3];
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        ai[g] = bi[g];
#pragma unroll
        for (int i = 0; i < kFwdMaxI; ++i) ai[g] += wi[g][i] * xs[i];
      }
      const float rr = sigmoidf_(ai[0] + (gh[0][tid] + bh[0]));
      const float zz = sigmoidf_(ai[1] + (gh[1][tid] + bh[1]));
      const float nn = tanhf(ai[2] + rr * (gh[2][tid] + bh[2]));
      const float hn = (1.f - zz) * nn + zz * hs[cur][tid];
      hs[cur ^ 1][tid] = hn;
      h[((size_t)t * B + b) * H + tid] = hn;
    }
#pragma unroll
    for (int i = 0; i < kFwdMaxI; ++i) xs[i] = xn[i];
    __syncthreads();
    cur ^= 1;
  }
}

}  // namespace

bppsa_status bppsa_build_jacobians_gru_h128(int T, int B, int I, const float* h, const float* x,
                                            const float* w_ih, const float* w_hh, const float* b_ih,
                                            const float* b_hh, float* Jt, hipStream_t stream) {
  const long long rows = (long long)T * B;
  const long long nbatch = (rows + kBatch - 1) / kBatch;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  const long long grid = nbatch < cus ? nbatch : cus;     // one 81 KB workgroup per compute unit
  const size_t lds = (size_t)(kBatch * LS + kBatch * 4 * H) * sizeof(float);
  BPPSA_HIP_TRY(hipFuncSetAttribute((const void*)gru_jacobians_h128_kernel,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  gru_jacobians_h128_kernel<<<(int)grid, kJacThreads, lds, stream>>>(rows, I, nbatch, h, x, w_ih, w_hh, b_ih,
                                                                    b_hh, Jt);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_gru_coefs_h128(long long rows, int I, const float* h, const float* x, const float* w_ih,
                                  const float* w_hh, const float* b_ih, const float* b_hh, float* coef,
                                  float* wT, hipStream_t stream) {
  const long long nbatch = (rows + kBatch - 1) / kBatch;
  if (nbatch > 0x7fffffffLL) return BPPSA_EOVERFLOW;
  gru_transpose_weights_h128_kernel<<<3 * H * H / 256, 256, 0, stream>>>(w_hh, wT);
  BPPSA_CHECK_LAUNCH();
  gru_coefs_h128_kernel<<<(int)nbatch, 256, 0, stream>>>(rows, I, h, x, w_ih, w_hh, b_ih, b_hh, coef);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_gru_deltas_h128(long long rows, int I, const float* h, const float* x, const float* G,
                                   const float* w_ih, const float* w_hh, const float* b_ih,
                                   const float* b_hh, float* delta, hipStream_t stream) {
  const long long nbatch = (rows + kBatch - 1) / kBatch;
  if (nbatch > 0x7fffffffLL) return BPPSA_EOVERFLOW;
  gru_deltas_h128_kernel<<<(int)nbatch, kDeltaThreads, 0, stream>>>(rows, I, h, x, G, w_ih, w_hh, b_ih, b_hh,
                                                                   delta);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

// `part` receives nsplit partials of [3H][H + 1 + I + 1]; returns BPPSA_EUNSUPPORTED for I > 4.
bppsa_status bppsa_gru_param_partials_h128(long long rows, int I, int nsplit, const float* h, const float* x,
                                           const float* delta, float* part, hipStream_t stream) {
  if (I > kPartMaxI) return BPPSA_EUNSUPPORTED;
  long long rps = (rows + nsplit - 1) / nsplit;
  rps = (rps + 1) / 2 * 2;
  gru_param_partials_h128_kernel<<<dim3(3 * H / 32, (nsplit + 3) / 4), 256, 0, stream>>>(rows, I, nsplit, rps, h, x,
                                                                                         delta, part);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

bppsa_status bppsa_gru_forward_h128(int T, int B, int I, const float* x, const float* w_ih, const float* w_hh,
                                    const float* b_ih, const float* b_hh, float* h, hipStream_t stream) {
  if (I > kFwdMaxI) return BPPSA_EUNSUPPORTED;
  gru_forward_h128_kernel<<<B, kFwdThreads, 0, stream>>>(T, B, I, x, w_ih, w_hh, b_ih, b_hh, h);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
