// Analytic generation of transposed Jacobians directly in CSR (Appendix D):
// 3x3 convolution (and the convolution of any kernel size, stride, padding and dilation), ReLU,
// 2x2 max-pooling and the fully connected layer.
// Row pointers come from a count pass plus an exclusive prefix sum; column
// indices within a row ascend because candidates are enumerated in column order
// and compacted with wave-level prefix counts.
#include "bppsa_internal.h"
#include "sparse_common.h"

namespace {

// Candidate q of row (c, y, x) of a convolution Jacobian: q = co * 9 + tap, tap = (dy+1)*3 + (dx+1).
struct ConvCand {
  bool valid;
  int col;
  int widx;
};

__device__ __forceinline__ ConvCand conv_candidate(int q, int c, int y, int x, int ci, int h, int w,
                                                   const uint8_t* __restrict__ mask) {
  ConvCand r;
  const int co = q / 9, tap = q - co * 9;
  const int dy = tap / 3 - 1, dx = tap - (tap / 3) * 3 - 1;
  const int yy = y + dy, xx = x + dx;
  r.widx = ((co * ci + c) * 3 + (1 - dy)) * 3 + (1 - dx);
  r.col = co * h * w + yy * w + xx;
  r.valid = (yy >= 0) && (yy < h) && (xx >= 0) && (xx < w) && (mask == nullptr || mask[r.widx] != 0);
  return r;
}

// One wave per row.  fill == 0: write the row length into indptr[row].
template <int FILL>
__global__ void __launch_bounds__(256)
conv_rows_kernel(int ci, int co, int h, int w, const float* __restrict__ weight,
                 const uint8_t* __restrict__ mask, int32_t* __restrict__ indptr,
                 int32_t* __restrict__ indices, float* __restrict__ data) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int rows = ci * h * w;
  if (row >= rows) return;
  const int c = row / (h * w);
  const int rem = row - c * h * w;
  const int y = rem / w, x = rem - y * w;
  const int ncand = co * 9;
  int count = 0;
  const int base = FILL ? indptr[row] : 0;
  for (int q0 = 0; q0 < ncand; q0 += 64) {
    const int q = q0 + lane;
    ConvCand cd;
    cd.valid = false;
    if (q < ncand) cd = conv_candidate(q, c, y, x, ci, h, w, mask);
    const unsigned long long bal = __ballot(cd.valid);
    if (FILL && cd.valid) {
      const int off = count + __popcll(bal & ((1ull << lane) - 1ull));
      indices[base + off] = cd.col;
      data[base + off] = weight[cd.widx];
    }
    count += __popcll(bal);
  }
  if (!FILL && lane == 0) indptr[row] = count;
}

// Any kernel size, stride, zero padding and dilation (the generic routine the footnote of Appendix
// D.1 leaves open).  Input (c, y, x) feeds output (o, oy, ox) through tap (ky, kx) when
// y = oy sh - ph + ky dh and x = ox sw - pw + kx dw; for a given output the tap is unique, so
// no entry is a sum.  Candidate q = o * kh * kw + tap with the taps taken from the last to the
// first, which makes (oy, ox) and with it the column ascend along a row.
struct ConvGeom {
  int kh, kw, sh, sw, ph, pw, dh, dw, oh, ow;
};

__device__ __forceinline__ ConvCand conv2d_candidate(int q, int c, int y, int x, int ci, const ConvGeom& g,
                                                     const uint8_t* __restrict__ mask) {
  ConvCand r;
  const int taps = g.kh * g.kw;
  const int o = q / taps, tap = q - o * taps;
  const int ky = g.kh - 1 - tap / g.kw, kx = g.kw - 1 - (tap - (tap / g.kw) * g.kw);
  const int ny = y + g.ph - ky * g.dh, nx = x + g.pw - kx * g.dw;      // oy sh and ox sw
  const int oy = ny / g.sh, ox = nx / g.sw;
  r.widx = ((o * ci + c) * g.kh + ky) * g.kw + kx;
  r.col = (o * g.oh + oy) * g.ow + ox;
  r.valid = ny >= 0 && nx >= 0 && oy * g.sh == ny && ox * g.sw == nx && oy < g.oh && ox < g.ow &&
            (mask == nullptr || mask[r.widx] != 0);
  return r;
}

template <int FILL>
__global__ void __launch_bounds__(256)
conv2d_rows_kernel(int ci, int co, int h, int w, ConvGeom g, const float* __restrict__ weight,
                   const uint8_t* __restrict__ mask, int32_t* __restrict__ indptr,
                   int32_t* __restrict__ indices, float* __restrict__ data) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int rows = ci * h * w;
  if (row >= rows) return;
  const int c = row / (h * w);
  const int rem = row - c * h * w;
  const int y = rem / w, x = rem - y * w;
  const int ncand = co * g.kh * g.kw;
  int count = 0;
  const int base = FILL ? indptr[row] : 0;
  for (int q0 = 0; q0 < ncand; q0 += 64) {
    const int q = q0 + lane;
    ConvCand cd;
    cd.valid = false;
    if (q < ncand) cd = conv2d_candidate(q, c, y, x, ci, g, mask);
    const unsigned long long bal = __ballot(cd.valid);
    if (FILL && cd.valid) {
      const int off = count + __popcll(bal & ((1ull << lane) - 1ull));
      indices[base + off] = cd.col;
      data[base + off] = weight[cd.widx];
    }
    count += __popcll(bal);
  }
  if (!FILL && lane == 0) indptr[row] = count;
}

// host: checks the geometry, fills in the output size; false if a size does not fit 32 bits
bppsa_status conv2d_geometry(int ci, int co, int h, int w, const bppsa_conv2d_geometry* in, ConvGeom* g) {
  if (!in || ci < 1 || co < 1 || h < 1 || w < 1) return BPPSA_EINVAL;
  if (in->kh < 1 || in->kw < 1 || in->stride_h < 1 || in->stride_w < 1 || in->pad_h < 0 || in->pad_w < 0 ||
      in->dil_h < 1 || in->dil_w < 1)
    return BPPSA_EINVAL;
  const int64_t span_h = (int64_t)h + 2LL * in->pad_h - (int64_t)in->dil_h * (in->kh - 1) - 1;
  const int64_t span_w = (int64_t)w + 2LL * in->pad_w - (int64_t)in->dil_w * (in->kw - 1) - 1;
  if (span_h < 0 || span_w < 0) return BPPSA_ESHAPE;               // the kernel does not fit: no output
  const int64_t oh = span_h / in->stride_h + 1, ow = span_w / in->stride_w + 1;
  const int64_t rows = (int64_t)ci * h * w, cols = (int64_t)co * oh * ow;
  const int64_t taps = (int64_t)in->kh * in->kw;
  if (rows >= INT32_MAX || cols >= INT32_MAX || taps >= INT32_MAX || (int64_t)co * taps >= INT32_MAX ||
      (int64_t)co * ci * taps >= INT32_MAX)
    return BPPSA_EOVERFLOW;
  // every stored entry is one (output element, input channel, tap) triple
  if ((double)cols * (double)ci * (double)taps >= (double)INT32_MAX) return BPPSA_EOVERFLOW;
  // intermediate coordinates: y + pad and ky * dil
  if ((int64_t)h + in->pad_h >= INT32_MAX || (int64_t)w + in->pad_w >= INT32_MAX ||
      (int64_t)in->dil_h * in->kh >= INT32_MAX || (int64_t)in->dil_w * in->kw >= INT32_MAX)
    return BPPSA_EOVERFLOW;
  *g = ConvGeom{in->kh, in->kw, in->stride_h, in->stride_w, in->pad_h, in->pad_w, in->dil_h, in->dil_w, (int)oh, (int)ow};
  return BPPSA_OK;
}

template <int FILL>
__global__ void __launch_bounds__(256)
linear_rows_kernel(int out, int in, const float* __restrict__ weight,
                   const uint8_t* __restrict__ mask, int32_t* __restrict__ indptr,
                   int32_t* __restrict__ indices, float* __restrict__ data) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);   // input feature
  if (row >= in) return;
  int count = 0;
  const int base = FILL ? indptr[row] : 0;
  for (int j0 = 0; j0 < out; j0 += 64) {
    const int j = j0 + lane;
    const bool valid = (j < out) && (mask == nullptr || mask[(size_t)j * in + row] != 0);
    const unsigned long long bal = __ballot(valid);
    if (FILL && valid) {
      const int off = count + __popcll(bal & ((1ull << lane) - 1ull));
      indices[base + off] = j;
      data[base + off] = weight[(size_t)j * in + row];
    }
    count += __popcll(bal);
  }
  if (!FILL && lane == 0) indptr[row] = count;
}

__global__ void relu_kernel(int d, const float* __restrict__ x, int32_t* __restrict__ indptr,
                            int32_t* __restrict__ indices, float* __restrict__ data) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < d) {
    indptr[i] = i;
    indices[i] = i;
    data[i] = x[i] > 0.f ? 1.f : 0.f;
  }
  if (i == d) indptr[d] = d;
}

// Is input element (c, y, x) the first maximum of its 2x2 window (row-major window order)?
__device__ __forceinline__ bool pool_is_argmax(const float* __restrict__ plane, int w, int y, int x) {
  const int y0 = y & ~1, x0 = x & ~1;
  float best = plane[y0 * w + x0];
  int by = y0, bx = x0;
  float v = plane[y0 * w + x0 + 1];
  if (v > best) { best = v; by = y0; bx = x0 + 1; }
  v = plane[(y0 + 1) * w + x0];
  if (v > best) { best = v; by = y0 + 1; bx = x0; }
  v = plane[(y0 + 1) * w + x0 + 1];
  if (v > best) { best = v; by = y0 + 1; bx = x0 + 1; }
  return by == y && bx == x;
}

template <int FILL>
__global__ void pool_kernel(int c, int h, int w, const float* __restrict__ x,
                            int32_t* __restrict__ indptr, int32_t* __restrict__ indices,
                            float* __restrict__ data) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= c * h * w) return;
  const int ch = i / (h * w);
  const int rem = i - ch * h * w;
  const int y = rem / w, xx = rem - y * w;
  const bool hit = pool_is_argmax(x + (size_t)ch * h * w, w, y, xx);
  if (!FILL) {
    indptr[i] = hit ? 1 : 0;
  } else if (hit) {
    const int p = indptr[i];
    indices[p] = (ch * (h / 2) + (y >> 1)) * (w / 2) + (xx >> 1);
    data[p] = 1.f;
  }
}

}  // namespace

extern "C" bppsa_status bppsa_csr_conv3x3_indptr(int ci, int co, int h, int w, const uint8_t* mask,
                                                 int32_t* indptr, void* stream) {
  if (ci < 1 || co < 1 || h < 1 || w < 1 || !indptr) return BPPSA_EINVAL;
  const int64_t rows = (int64_t)ci * h * w, cols = (int64_t)co * h * w;
  const int64_t nnz_max = (int64_t)ci * co * (3LL * h - 2) * (3LL * w - 2);
  if (rows >= INT32_MAX || cols >= INT32_MAX || nnz_max >= INT32_MAX || (int64_t)co * ci * 9 >= INT32_MAX)
    return BPPSA_EOVERFLOW;
  hipStream_t s = (hipStream_t)stream;
  conv_rows_kernel<0><<<bppsa_ceil_div((int)rows, 4), 256, 0, s>>>(ci, co, h, w, nullptr, mask, indptr, nullptr, nullptr);
  BPPSA_CHECK_LAUNCH();
  return bppsa_lengths_to_indptr(indptr, (int)rows, s);
}

extern "C" bppsa_status bppsa_csr_conv3x3_fill(int ci, int co, int h, int w, const float* weight,
                                               const uint8_t* mask, const int32_t* indptr,
                                               int32_t* indices, float* data, void* stream) {
  if (ci < 1 || co < 1 || h < 1 || w < 1 || !weight || !indptr || !indices || !data) return BPPSA_EINVAL;
  const int64_t rows = (int64_t)ci * h * w;
  const int64_t nnz_max = (int64_t)ci * co * (3LL * h - 2) * (3LL * w - 2);
  if (rows >= INT32_MAX || (int64_t)co * h * w >= INT32_MAX || nnz_max >= INT32_MAX) return BPPSA_EOVERFLOW;
  conv_rows_kernel<1><<<bppsa_ceil_div((int)rows, 4), 256, 0, (hipStream_t)stream>>>(
      ci, co, h, w, weight, mask, const_cast<int32_t*>(indptr), indices, data);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_csr_conv2d_indptr(int ci, int co, int h, int w, const bppsa_conv2d_geometry* geometry,
                                                const uint8_t* mask, int32_t* indptr, void* stream) {
  if (!indptr) return BPPSA_EINVAL;
  ConvGeom g;
  BPPSA_TRY(conv2d_geometry(ci, co, h, w, geometry, &g));
  const int rows = ci * h * w;
  hipStream_t s = (hipStream_t)stream;
  conv2d_rows_kernel<0><<<bppsa_ceil_div(rows, 4), 256, 0, s>>>(ci, co, h, w, g, nullptr, mask, indptr, nullptr, nullptr);
  BPPSA_CHECK_LAUNCH();
  return bppsa_lengths_to_indptr(indptr, rows, s);
}

extern "C" bppsa_status bppsa_csr_conv2d_fill(int ci, int co, int h, int w, const bppsa_conv2d_geometry* geometry,
                                              const float* weight, const uint8_t* mask, const int32_t* indptr,
                                              int32_t* indices, float* data, void* stream) {
  if (!weight || !indptr || !indices || !data) return BPPSA_EINVAL;
  ConvGeom g;
  BPPSA_TRY(conv2d_geometry(ci, co, h, w, geometry, &g));
  conv2d_rows_kernel<1><<<bppsa_ceil_div(ci * h * w, 4), 256, 0, (hipStream_t)stream>>>(
      ci, co, h, w, g, weight, mask, const_cast<int32_t*>(indptr), indices, data);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_csr_relu(int d, const float* x, int32_t* indptr, int32_t* indices,
                                       float* data, void* stream) {
  if (d < 1 || !x || !indptr || !indices || !data) return BPPSA_EINVAL;
  if (d == INT32_MAX) return BPPSA_EOVERFLOW;
  relu_kernel<<<bppsa_ceil_div(d + 1, 256), 256, 0, (hipStream_t)stream>>>(d, x, indptr, indices, data);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_csr_maxpool2x2(int c, int h, int w, const float* x, int32_t* indptr,
                                             int32_t* indices, float* data, void* stream) {
  if (c < 1 || h < 2 || w < 2 || !x || !indptr || !indices || !data) return BPPSA_EINVAL;
  if ((h & 1) || (w & 1)) return BPPSA_ESHAPE;
  const int64_t rows = (int64_t)c * h * w;
  if (rows >= INT32_MAX) return BPPSA_EOVERFLOW;
  hipStream_t s = (hipStream_t)stream;
  const int nb = bppsa_ceil_div((int)rows, 256);
  pool_kernel<0><<<nb, 256, 0, s>>>(c, h, w, x, indptr, nullptr, nullptr);
  BPPSA_CHECK_LAUNCH();
  bppsa_status st = bppsa_lengths_to_indptr(indptr, (int)rows, s);
  if (st != BPPSA_OK) return st;
  pool_kernel<1><<<nb, 256, 0, s>>>(c, h, w, x, indptr, indices, data);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}

extern "C" bppsa_status bppsa_csr_linear_indptr(int out, int in, const uint8_t* mask, int32_t* indptr,
                                                void* stream) {
  if (out < 1 || in < 1 || !indptr) return BPPSA_EINVAL;
  if ((int64_t)out * in >= INT32_MAX) return BPPSA_EOVERFLOW;
  hipStream_t s = (hipStream_t)stream;
  linear_rows_kernel<0><<<bppsa_ceil_div(in, 4), 256, 0, s>>>(out, in, nullptr, mask, indptr, nullptr, nullptr);
  BPPSA_CHECK_LAUNCH();
  return bppsa_lengths_to_indptr(indptr, in, s);
}

extern "C" bppsa_status bppsa_csr_linear_fill(int out, int in, const float* weight, const uint8_t* mask,
                                              const int32_t* indptr, int32_t* indices, float* data,
                                              void* stream) {
  if (out < 1 || in < 1 || !weight || !indptr || !indices || !data) return BPPSA_EINVAL;
  if ((int64_t)out * in >= INT32_MAX) return BPPSA_EOVERFLOW;
  linear_rows_kernel<1><<<bppsa_ceil_div(in, 4), 256, 0, (hipStream_t)stream>>>(
      out, in, weight, mask, const_cast<int32_t*>(indptr), indices, data);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
