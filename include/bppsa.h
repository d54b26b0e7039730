/*
 * bppsa.h - C ABI of the MI355X (gfx950) BPPSA library.
 *
 * BPPSA recasts back-propagation as an exclusive scan, under the operator
 * A <> B = B A, over the array [ g_n, Jt_n, ..., Jt_1 ] of the loss gradient
 * and the transposed per-step Jacobians (paper Section 3.1, Eq. 4 and Eq. 5),
 * evaluated by a modified Blelloch up-sweep / down-sweep (Section 3.2,
 * Algorithm 1).  This header declares the calls of that hot path.
 *
 * Conventions shared by every call
 *   - Every array pointer is a DEVICE pointer to memory owned by the caller
 *     (fp32 values, int32 indices), C-contiguous in the stated shape.  The
 *     library neither frees nor retains caller memory and never modifies an
 *     input array.
 *   - Scratch space comes only from the caller's `workspace` (device memory,
 *     256-byte aligned) whose size the matching *_workspace_bytes query returns.
 *     A workspace that is too small yields BPPSA_EWORKSPACE and nothing is
 *     launched.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; they do not synchronise.  Launch failures
 *     are reported as BPPSA_EHIP.
 *   - Shapes are validated on the host before anything is launched:
 *     BPPSA_EINVAL for null pointers / non-positive sizes, BPPSA_ESHAPE for
 *     sizes a kernel cannot take, BPPSA_EOVERFLOW when an index would not fit
 *     its integer type, BPPSA_EUNSUPPORTED for a cell / size with no kernel.
 *   - Time indexing: hidden states h[0..T] with h[0] the initial state;
 *     x[t-1] is the input that produces h[t]; Jt[t] = (d h[t+1] / d h[t])^T for
 *     t = 0..T-1, so that g[t] = Jt[t] g[t+1] with g[t] = dL/dh[t] (Eq. 3).
 *     In the paper's array a[0] = g[T] and a[k] = Jt[T-k].
 */
#ifndef BPPSA_H
#define BPPSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BPPSA_OK = 0,
  BPPSA_EINVAL = 1,
  BPPSA_ESHAPE = 2,
  BPPSA_EWORKSPACE = 3,
  BPPSA_EOVERFLOW = 4,
  BPPSA_EHIP = 5,
  BPPSA_EUNSUPPORTED = 6
} bppsa_status;

typedef enum { BPPSA_RNN_TANH = 0, BPPSA_GRU = 1 } bppsa_cell;

/* Human-readable name of a status code (static storage, never NULL). */
const char* bppsa_strerror(int status);

/* ------------------------------------------------------------------------
 * Workload preparation (outside the timed hot path).
 * ---------------------------------------------------------------------- */

/*
 * Forward recurrence that produces the hidden states the hot path consumes.
 *   RNN (Section 4.1):  h[t] = tanh(W_ih x[t-1] + b_ih + W_hh h[t-1] + b_hh)
 *   GRU (Section 4.2):  gates r, z, n in that row order of w_ih [3H,I],
 *                       w_hh [3H,H], b_ih [3H], b_hh [3H].
 * h is [T+1,B,H]; h[0] is read as the initial state, h[1..T] are written.
 * x is [T,B,I].  RNN: w_ih [H,I], w_hh [H,H], b_ih [H], b_hh [H]; either bias
 * may be NULL (treated as zero).
 */
bppsa_status bppsa_forward(int cell, int T, int B, int H, int I,
                           const float* x, const float* w_ih, const float* w_hh,
                           const float* b_ih, const float* b_hh,
                           float* h, void* stream);

/*
 * Softmax cross-entropy head on the last hidden state, mean over the batch
 * (Section 4.1): z = W_out h_T + b_out, L = mean_b( logsumexp(z_b) - z_b[y_b] ).
 * Writes seed[B,H] = dL/dh_T (the a[0] of Eq. 5) and, if loss != NULL, L.
 * h_last [B,H], w_out [C,H], b_out [C], labels [B] int32 in [0,C).  C <= 64.
 */
bppsa_status bppsa_head_seed(int B, int H, int C,
                             const float* h_last, const float* w_out,
                             const float* b_out, const int32_t* labels,
                             float* seed, float* loss, void* stream);

/* ------------------------------------------------------------------------
 * Hot path.
 * ---------------------------------------------------------------------- */

/*
 * Materialise the transposed step Jacobians, the matrix entries of Eq. 5.
 *   RNN: Jt[t][b][i][j] = W_hh[j][i] * (1 - h[t+1][b][j]^2)   (from the RNN
 *        equation of Section 4.1); only h and w_hh are read, x / w_ih / b_* may
 *        be NULL.
 *   GRU: the gates are recomputed from (h[t], x[t]) for all t in parallel and
 *        combined as in Appendix E's closed form.
 * Jt is [T,B,H,H], row-major per matrix, written in full.
 */
bppsa_status bppsa_build_jacobians(int cell, int T, int B, int H, int I,
                                   const float* h, const float* x,
                                   const float* w_ih, const float* w_hh,
                                   const float* b_ih, const float* b_hh,
                                   float* Jt, void* stream);

/* Bytes of workspace bppsa_scan needs for these sizes (host-only, pure). */
size_t bppsa_scan_workspace_bytes(int T, int B, int H);

/*
 * The scan of Eq. 4 / Algorithm 1:  G[t-1][b] = dL/dh[t] for t = 1..T given
 * seed[b] = dL/dh[T], i.e. G[T-1] = seed and G[t-1] = Jt[t] G[t].
 * If g0 != NULL it receives dL/dh[0] = Jt[0] G[0] (the inclusive tail); with
 * g0 == NULL Jt[0] is never read (Algorithm 1's last input reaches no output).
 * Jt [T,B,H,H], seed [B,H], G [T,B,H], g0 [B,H] or NULL.  T = 1 is legal.
 * Values follow any bracketing of the products (Section 3.5): results agree
 * with sequential back-propagation up to fp32 rounding order; repeated calls
 * on the same inputs return the same bits.
 * Kernels: H = 20 runs as one pass over Jt (units of 32 or 64 steps held in LDS
 * and registers, Algorithm 1 inside a unit, look-back across units); H = 128 and
 * every other H <= 128 run the hybrid of Section 5.3 (segment totals, scan of
 * the totals, matrix-vector down-sweep); H > 128 yields BPPSA_EUNSUPPORTED.
 * At H = 128, chains longer than one segment are scheduled by a cost model
 * (bppsa_scan_h128_schedule shows its choice): the steps nearest the seed are
 * walked by a serial matrix-vector chain per sample while the totals of the
 * other segments are formed on the matrix cores.  The chain and the
 * matrix-vector kernels are enqueued on a second stream owned by the library
 * (one per device, created on first use) and tied to `stream` with events on
 * both sides: work enqueued on `stream` after the call still sees every
 * result, and the call can be captured into a HIP graph.
 * The workspace is scratch only; its contents before the call do not matter.
 * For H = 20 its first 4-byte word is an error flag: it is 0 after a normal
 * call and 1 if a bounded wait inside the kernel expired, in which case G is
 * invalid (this cannot happen while the device makes progress; the caller may
 * read the word after synchronising).  Calls that share a workspace must be
 * ordered on one stream.
 */
bppsa_status bppsa_scan(int T, int B, int H,
                        const float* Jt, const float* seed,
                        float* G, float* g0,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * bppsa_scan for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and kernels as bppsa_scan, but the scratch
 * is a fixed array of BPPSA_SCAN_STATIC_SCRATCH_BYTES inside the library (one copy
 * per GPU, held until the process ends); the call allocates nothing and frees
 * nothing.  Sizes whose bppsa_scan_workspace_bytes exceeds that maximum are
 * rejected with BPPSA_EWORKSPACE and nothing is launched (T = 1000, B = 16, H = 20
 * needs 0.9 MiB; T * B up to about 70 000 fits at H = 20).  Every call on a GPU
 * shares that GPU's array: calls must be ordered on one stream; calls that overlap
 * on one GPU race.  What has to start at zero is cleared by the call itself.
 */
#define BPPSA_SCAN_STATIC_SCRATCH_BYTES (4u << 20)
bppsa_status bppsa_scan_static(int T, int B, int H,
                               const float* Jt, const float* seed,
                               float* G, float* g0, void* stream);

/*
 * bppsa_build_jacobians + bppsa_scan in one pass for the tanh RNN: the transposed
 * Jacobians of Section 4.1, Jt[t][i][j] = W_hh[j][i] (1 - h[t+1][j]^2), are generated
 * inside the scan kernel from h [T+1,B,H] and w_hh [H,H] and never stored, so neither
 * the [T,B,H,H] array nor its HBM round trip exists.  Outputs, g0 and the workspace
 * (bppsa_scan_workspace_bytes) are those of bppsa_scan, and the values are bit-identical
 * to bppsa_build_jacobians followed by bppsa_scan.  H = 20 only (the paper's RNN size):
 * other sizes return BPPSA_EUNSUPPORTED and should use the two calls.
 */
bppsa_status bppsa_rnn_scan_fused(int T, int B, int H, const float* h, const float* w_hh,
                                  const float* seed, float* G, float* g0,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * The GRU counterpart for H = 128 (the size of Section 4.2's workload): the scan with the
 * transposed Jacobians of Appendix E's closed form generated inside its kernels from the
 * hidden states, the inputs and the weights, so no [T,B,H,H] array exists.  A first kernel
 * recomputes the gates of every step and keeps four H-vectors per step; where the scan needs a
 * Jacobian as a matrix (the A operand of a matrix-matrix step) its kernel forms it from those
 * and the three recurrent matrices held in registers, and where it needs a Jacobian times a
 * vector it applies the three matrices to the vector scaled by those vectors instead.
 * Arguments as for bppsa_build_jacobians (cell GRU) followed by bppsa_scan; the result equals
 * those two calls up to rounding.  workspace: at least bppsa_gru_scan_fused_workspace_bytes
 * bytes (0 for sizes it does not serve), 256-byte aligned.  Other H: BPPSA_EUNSUPPORTED.
 */
size_t bppsa_gru_scan_fused_workspace_bytes(int T, int B, int H);
bppsa_status bppsa_gru_scan_fused(int T, int B, int H, int I,
                                  const float* h, const float* x,
                                  const float* w_ih, const float* w_hh,
                                  const float* b_ih, const float* b_hh,
                                  const float* seed, float* G, float* g0,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace bppsa_param_grads needs (host-only, pure). */
size_t bppsa_param_grads_workspace_bytes(int cell, int T, int B, int H, int I);

/*
 * Parameter gradients, Eq. 2 summed over the steps that share the parameters.
 *   RNN: delta[t] = (1 - h[t]^2) o G[t-1];  dW_hh = sum delta[t] h[t-1]^T,
 *        dW_ih = sum delta[t] x[t-1]^T, db = sum delta[t]  (t = 1..T, all b).
 *        Outputs dW_ih [H,I], dW_hh [H,H], db_ih [H]; db_hh [H] (same values)
 *        is written when non-NULL.  w_* and b_* inputs are not read.
 *   GRU: dW_ih [3H,I], dW_hh [3H,H], db_ih [3H], db_hh [3H]; the gates are
 *        recomputed from (h, x, weights); db_ih and db_hh differ only in the
 *        n-gate rows.
 * Outputs are overwritten, not accumulated.  Sums use blocked fp32 partials
 * reduced in a fixed order (deterministic).
 */
bppsa_status bppsa_param_grads(int cell, int T, int B, int H, int I,
                               const float* h, const float* x, const float* G,
                               const float* w_ih, const float* w_hh,
                               const float* b_ih, const float* b_hh,
                               float* dW_ih, float* dW_hh,
                               float* db_ih, float* db_hh,
                               void* workspace, size_t workspace_bytes,
                               void* stream);


/* ------------------------------------------------------------------------
 * One training iteration (Section 4.1): forward, head, backward as a scan,
 * optimiser step.
 * ---------------------------------------------------------------------- */

/*
 * bppsa_head_seed plus the head's own parameter gradients: dW_out [C,H] = dz^T h_T and
 * db_out [C] = sum_b dz, with dz = (softmax(z) - onehot(y)) / B.  loss, dW_out and db_out may be
 * NULL.  Sums over the batch run in index order (deterministic).  C <= 64 and B (C + 1) <= 12288.
 */
bppsa_status bppsa_head_backward(int B, int H, int C,
                                 const float* h_last, const float* w_out, const float* b_out,
                                 const int32_t* labels, float* seed, float* loss,
                                 float* dW_out, float* db_out, void* stream);

/*
 * One Adam update of n parameters in place (Kingma & Ba, Algorithm 1; the optimiser Section 4.1
 * trains with):  m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 * theta <- theta - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps).
 * step = 1 for the first update; m and v start at zero.  All arrays are device memory.  The
 * constants come as doubles so that 1 - beta and the two bias corrections are rounded to fp32 once.
 */
bppsa_status bppsa_adam_step(int64_t n, float* theta, const float* grad, float* m, float* v,
                             int step, double lr, double beta1, double beta2, double eps, void* stream);

/*
 * The whole iteration for the tanh RNN, enqueued on `stream` without synchronising:
 * bppsa_forward, bppsa_head_backward on h[T], the backward pass over the T steps as a scan
 * (bppsa_build_jacobians + bppsa_scan when st->Jt is given, else bppsa_rnn_scan_fused, which
 * exists for H = 20), bppsa_param_grads, bppsa_adam_step over all parameters.
 * Parameters, gradients and both Adam moments are flat device arrays of
 * bppsa_rnn_param_count(H, I, C) floats laid out as
 *     W_ih [H,I] | W_hh [H,H] | b_ih [H] | b_hh [H] | W_out [C,H] | b_out [C].
 * x is [T,B,I], labels [B] int32.  st->h is [T+1,B,H] with h[0] the initial state (the caller
 * zeroes it once; rows 1..T are overwritten), st->G [T,B,H], st->seed [B,H], st->loss [1] (may be
 * NULL), st->Jt [T,B,H,H] or NULL, st->workspace of at least
 * bppsa_rnn_train_workspace_bytes(T, B, H, I) bytes, 256-byte aligned (the scan's part comes
 * first, so for H = 20 its first word is the scan's error flag after the iteration, as described
 * at bppsa_scan).  The struct is host memory, its pointers device memory; nothing is allocated.
 * st->loss receives the loss before the update.
 */
typedef struct bppsa_rnn_train_state {
  float* params;
  float* grads;
  float* adam_m;
  float* adam_v;
  float* h;
  float* G;
  float* seed;
  float* loss;
  float* Jt;
  void* workspace;
  size_t workspace_bytes;
} bppsa_rnn_train_state;
size_t bppsa_rnn_param_count(int H, int I, int C);
size_t bppsa_rnn_train_workspace_bytes(int T, int B, int H, int I);
bppsa_status bppsa_rnn_train_step(int T, int B, int H, int I, int C,
                                  const float* x, const int32_t* labels,
                                  const bppsa_rnn_train_state* st, int step,
                                  double lr, double beta1, double beta2, double eps, void* stream);

/* ------------------------------------------------------------------------
 * Sparse path: CSR transposed Jacobians of a (pruned) CNN and their scan.
 * ---------------------------------------------------------------------- */

/*
 * A CSR matrix in the SciPy convention used by Appendix D: row i owns
 * indices[indptr[i] .. indptr[i+1]) (ascending) and the matching data.  A
 * transposed Jacobian (d out / d in)^T has rows = input elements and
 * cols = output elements.  The struct itself lives in HOST memory; the three
 * arrays are DEVICE pointers.
 */
typedef struct {
  int32_t rows, cols;
  int64_t nnz;
  const int32_t* indptr;  /* [rows + 1] */
  const int32_t* indices; /* [nnz] */
  const float* data;      /* [nnz] */
} bppsa_csr;

/*
 * Appendix D.1: transposed Jacobian of a 3x3, padding-1, stride-1 convolution
 * (cross-correlation) with weight [co,ci,3,3] on a ci x h x w input.
 * Row (ci,y,x) holds, per output channel and per in-image neighbour
 * (y+dy, x+dx), dy,dx in {-1,0,1}, column co*h*w + (y+dy)*w + (x+dx) with value
 * weight[co][ci][1-dy][1-dx]; columns ascend.  Only in-image neighbours are
 * stored (nnz = ci*co*(3h-2)(3w-2) unpruned, the count behind Table 1's 0.99157).
 * `mask` ([co,ci,3,3] bytes, NULL = all kept) marks pruned weights (0) as
 * structurally absent; a kept weight whose value is 0.0 stays.
 * Two calls: *_indptr writes indptr[ci*h*w + 1]; the caller reads its last
 * entry (= nnz) to size indices/data, then *_fill writes them.
 */
bppsa_status bppsa_csr_conv3x3_indptr(int ci, int co, int h, int w, const uint8_t* mask,
                                      int32_t* indptr, void* stream);
bppsa_status bppsa_csr_conv3x3_fill(int ci, int co, int h, int w, const float* weight,
                                    const uint8_t* mask, const int32_t* indptr,
                                    int32_t* indices, float* data, void* stream);

/*
 * The same for a convolution of any kernel size, stride, zero padding and dilation (the generic
 * routine the footnote of Appendix D.1 leaves open): weight [co,ci,kh,kw] on a ci x h x w input,
 * output co x oh x ow with oh = (h + 2 pad_h - dil_h (kh - 1) - 1) / stride_h + 1 (ow alike).
 * Row (ci,y,x) holds column (co*oh + oy)*ow + ox with value weight[co][ci][ky][kx] wherever
 * y = oy stride_h - pad_h + ky dil_h and x = ox stride_w - pad_w + kx dil_w; an input and an output
 * meet through at most one tap, so no entry is a sum; columns ascend.  mask [co,ci,kh,kw] as
 * above.  With kh = kw = 3, stride 1, padding 1, dilation 1 the arrays equal those of
 * bppsa_csr_conv3x3_*.  BPPSA_ESHAPE if the dilated kernel is larger than the padded image,
 * BPPSA_EOVERFLOW if a size or co*oh*ow*ci*kh*kw does not fit 32 bits.  The same two calls;
 * indptr has ci*h*w + 1 entries.  The geometry struct is host memory.
 */
typedef struct bppsa_conv2d_geometry {
  int32_t kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} bppsa_conv2d_geometry;
bppsa_status bppsa_csr_conv2d_indptr(int ci, int co, int h, int w, const bppsa_conv2d_geometry* geometry,
                                     const uint8_t* mask, int32_t* indptr, void* stream);
bppsa_status bppsa_csr_conv2d_fill(int ci, int co, int h, int w, const bppsa_conv2d_geometry* geometry,
                                   const float* weight, const uint8_t* mask, const int32_t* indptr,
                                   int32_t* indices, float* data, void* stream);

/*
 * Appendix D.2 (Algorithms 5-7): ReLU on d elements.  indptr[i] = i,
 * indices[i] = i, data[i] = (x[i] > 0) ? 1 : 0 (explicit zeros are kept).
 * indptr [d+1], indices [d], data [d].
 */
bppsa_status bppsa_csr_relu(int d, const float* x, int32_t* indptr, int32_t* indices,
                            float* data, void* stream);

/*
 * Appendix D.3 (Algorithms 8-10): 2x2 / stride-2 max-pooling of x [c,h,w] (h, w
 * even).  One unit entry per output: row = the window's first maximum in
 * row-major window order, column = the output's flat index.  indptr [c*h*w+1],
 * indices and data [c*(h/2)*(w/2)].
 */
bppsa_status bppsa_csr_maxpool2x2(int c, int h, int w, const float* x, int32_t* indptr,
                                  int32_t* indices, float* data, void* stream);

/*
 * Fully connected layer y = W x with W [out,in]: the transposed Jacobian is W^T
 * (rows = inputs, cols = outputs) restricted to the kept weights.  Two calls as
 * for the convolution; indptr is [in + 1].
 */
bppsa_status bppsa_csr_linear_indptr(int out, int in, const uint8_t* mask, int32_t* indptr,
                                     void* stream);
bppsa_status bppsa_csr_linear_fill(int out, int in, const float* weight, const uint8_t* mask,
                                   const int32_t* indptr, int32_t* indices, float* data,
                                   void* stream);

/* y[rows] = A x[cols]: the matrix-vector form of A <> B (Section 3.1). */
bppsa_status bppsa_spmv(const bppsa_csr* A, const float* x, float* y, void* stream);

/*
 * Sparse scan (Section 3.3, Section 5.3).  Jt[0..n) are the transposed
 * Jacobians in SCAN ORDER: Jt[0] belongs to the last layer and
 * rows(Jt[k]) = cols(Jt[k+1]).  seed has cols(Jt[0]) entries.  On return
 * grads[k] (caller-allocated, rows(Jt[k]) floats) = Jt[k] ... Jt[0] seed, the
 * gradient with respect to the input of that layer, for k = 0..n-1; a NULL
 * entry is skipped (grads[n-1] is the inclusive tail Algorithm 1 does not
 * produce and costs one extra matrix-vector product).
 *
 * The schedule is Algorithm 1's with only `up_levels` up-sweep levels, a linear
 * scan of the block totals, and the matching down-sweep levels (Section 5.3);
 * up_levels = 0 is the pure matrix-vector chain.  Products whose result reaches
 * no gradient are not planned.  Products that contain the
 * gradient vector are CSR x vector, all others CSR x CSR with the structural
 * pattern (boolean product of the patterns, ascending columns, explicit zeros
 * kept).
 *
 * The index structure of every product depends only on the input patterns, so
 * it is computed once, ahead of the training loop, by bppsa_spscan_plan_create
 * (which reads only indptr/indices, synchronises the stream, and carves all
 * device storage for product structures, product values and intermediate
 * vectors from `arena`; BPPSA_EWORKSPACE if it does not fit).  The plan itself
 * is a small host object.  bppsa_spscan_run then only computes values and does
 * not synchronise; Jt passed to it must have the patterns the plan was built
 * from (sizes are checked).  cols(B) of any product must be <= 1048576.
 */
typedef struct bppsa_spscan_plan bppsa_spscan_plan;

bppsa_status bppsa_spscan_plan_create(int n, const bppsa_csr* Jt, int up_levels,
                                      void* arena, size_t arena_bytes, void* stream,
                                      bppsa_spscan_plan** plan);
void bppsa_spscan_plan_destroy(bppsa_spscan_plan* plan);
/* Arena bytes the plan occupies, number of CSR x CSR products, and their structure. */
size_t bppsa_spscan_plan_arena_used(const bppsa_spscan_plan* plan);
int bppsa_spscan_plan_num_products(const bppsa_spscan_plan* plan);
/* Product `idx` = left * right; operand ids < n name Jt[id], ids >= n name product id - n. */
bppsa_status bppsa_spscan_plan_product(const bppsa_spscan_plan* plan, int idx, bppsa_csr* out,
                                       int* left_id, int* right_id);
/* Floating-point operations (2 per multiply-add) of the planned matrix-matrix and
   matrix-vector steps: the static analysis of Section 4.3. */
bppsa_status bppsa_spscan_plan_flops(const bppsa_spscan_plan* plan, int64_t* mm_flops,
                                     int64_t* mv_flops);

/* The planned steps one by one, in the order bppsa_spscan_run issues them: the per-step view of
 * the static analysis of Section 4.3, which gives the FLOP-per-step series of Section 5.3.
 *   kind    BPPSA_STEP_SPMV (CSR x vector) or BPPSA_STEP_SPGEMM (CSR x CSR)
 *   phase   up-sweep, the serial chain over block totals, down-sweep, or the inclusive tail
 *   level   up-/down-sweep: tree level d (0 = neighbouring elements); chain: index of the block
 *   matrix  SPMV: id of the matrix applied; SPGEMM: id of the product formed (ids as in
 *           bppsa_spscan_plan_product)
 *   flops   2 per multiply-add: SPMV 2 nnz(matrix); SPGEMM 2 x sum over stored (i, k) of the left
 *           operand of the stored entries in row k of the right operand
 *   numeric_kind  SPGEMM: which kernel forms the values (0 nothing to sum, 1 one wave per row,
 *           2/3/4 one workgroup per row with accumulators per column / per entry / in global
 *           memory); -1 for SPMV
 */
enum { BPPSA_STEP_SPMV = 0, BPPSA_STEP_SPGEMM = 1 };
enum { BPPSA_PHASE_UP = 0, BPPSA_PHASE_CHAIN = 1, BPPSA_PHASE_DOWN = 2, BPPSA_PHASE_TAIL = 3 };
typedef struct bppsa_spscan_step {
  int32_t kind, phase, level, matrix;
  int64_t flops;
  int32_t numeric_kind;
} bppsa_spscan_step;
int bppsa_spscan_plan_num_steps(const bppsa_spscan_plan* plan);
bppsa_status bppsa_spscan_plan_step_flops(const bppsa_spscan_plan* plan, int idx, bppsa_spscan_step* out);

/* A cache of symbolic phases (Section 4.3: the structures depend on the architecture alone, so
 * they are worth keeping across plans).  bppsa_spscan_plan_create_cached behaves like
 * bppsa_spscan_plan_create, except that the product structures live in device memory the cache
 * allocates (hipMalloc, on a miss only) and keeps until bppsa_spscan_cache_destroy, and that a call
 * whose inputs have the fingerprint of an earlier call (n, up_levels, shapes, and a 128-bit hash of
 * every indptr and indices array, formed on the device) takes the structures from that call and
 * runs no symbolic kernel.  The arena then holds only product values and vectors.  Equality of
 * patterns is decided by the fingerprint, not by comparing the arrays.  A cache belongs to the
 * device that was current at bppsa_spscan_cache_create (BPPSA_EINVAL on another), may be used from
 * several host threads (calls are serialised), and must outlive the plans made through it.
 * bppsa_spscan_cache_stats: plans served from the cache, plans that ran the symbolic phase, the
 * number of products whose structure was computed, and the device bytes held.
 */
typedef struct bppsa_spscan_cache bppsa_spscan_cache;
bppsa_status bppsa_spscan_cache_create(bppsa_spscan_cache** cache);
void bppsa_spscan_cache_destroy(bppsa_spscan_cache* cache);
bppsa_status bppsa_spscan_cache_stats(bppsa_spscan_cache* cache, int64_t* hits, int64_t* misses,
                                      int64_t* symbolic_products, size_t* device_bytes);
bppsa_status bppsa_spscan_plan_create_cached(bppsa_spscan_cache* cache, int n, const bppsa_csr* Jt,
                                             int up_levels, void* arena, size_t arena_bytes,
                                             void* stream, bppsa_spscan_plan** plan);

bppsa_status bppsa_spscan_run(const bppsa_spscan_plan* plan, const bppsa_csr* Jt,
                              const float* seed, float* const* grads, void* stream);

/* One-shot convenience: plan (in `workspace`), run, destroy.  Synchronises. */
bppsa_status bppsa_spscan(int n, const bppsa_csr* Jt, const float* seed, float* const* grads,
                          int up_levels, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Measurement aid (not part of the method).
 * ---------------------------------------------------------------------- */

/*
 * bppsa_scan at H = 20 with its two internal choices exposed, for tests and for measurement; the
 * gradients are those of bppsa_scan (same kernels, same workspace size).
 *   absent_dies : bit mask (0..255) of compute dies whose workgroups stand aside, as if the
 *                 dispatcher had placed no workgroup there; their chains are then picked up by
 *                 the placement-independent path.  0 = normal operation.
 *   unit_halves : 0 = chosen from the sizes as bppsa_scan does; 1 or 2 = units of one or two
 *                 halves of 32 steps regardless of the sizes.
 *   lookback_stats : NULL, or device memory for three int64: the number of unit totals all
 *                 look-backs applied (matrix-vector hops), the number of look-backs, and the most
 *                 hops one look-back took.
 */
bppsa_status bppsa_scan_h20_diag(int T, int B, const float* Jt, const float* seed,
                                 float* G, float* g0,
                                 void* workspace, size_t workspace_bytes, void* stream,
                                 int absent_dies, int unit_halves, int64_t* lookback_stats);

/*
 * How bppsa_scan (generated = 0) or bppsa_gru_scan_fused (generated = 1) walks a chain of T steps
 * of H = 128 for B samples on the current device.  The chain is cut into segments of
 * `segment_steps` steps (Section 5.3's hybrid schedule); the `chain_steps` steps nearest the seed
 * are walked by one serial matrix-vector chain per sample while the totals of the remaining
 * segments are formed with matrix-matrix products, `slab_segments` segments at a time
 * (`slabs` slabs; 0 when no slab is formed, or when the batch alone fills the device and the
 * totals of all segments are formed at once and scanned recursively).  The slab farthest from the
 * seed is cut into segments of `last_slab_steps` steps (shorter than `segment_steps` when it
 * would otherwise fill less than half of the device; 0 when there is no slab).  `matrix_products` counts
 * the H x H matrix-matrix products of the call, `model_us` is the estimate the choice was made
 * on (0 where no choice is made).  Host only, no device work.
 * Errors: BPPSA_EINVAL (T or B below 1, out NULL).
 */
typedef struct {
  int segment_steps;
  int segments;
  int chain_steps;
  int slab_segments;
  int slabs;
  int last_slab_steps;
  int64_t matrix_products;
  double model_us;
} bppsa_h128_schedule;
bppsa_status bppsa_scan_h128_schedule(int T, int B, int want_g0, int generated, bppsa_h128_schedule* out);

/*
 * bppsa_scan at H = 128 with the schedule forced, for tests and for measurement; the gradients
 * are those of bppsa_scan (same kernels, same workspace size).
 *   chain_segments : segments nearest the seed walked by the serial chain (clamped to the number
 *                    of segments; all of them = no matrix-matrix product).  0 = the form without
 *                    the serial chain (totals of all interior segments, scanned recursively).
 *   slab_segments  : segments per slab of totals; 0 = as many as fill the compute units that the
 *                    serial chains leave free.  Raised if more than 32 slabs would result.
 *   last_slab_steps: 64, 32 or 16 = segment length inside the slab farthest from the seed; 0 =
 *                    whichever the cost model prefers.
 * Errors: those of bppsa_scan; BPPSA_EINVAL for another last_slab_steps; BPPSA_EUNSUPPORTED if
 * chain_segments > 0 and the device has fewer than 2 B compute units (the serial chains take one
 * each); BPPSA_ESHAPE if the last slab cut that fine would have more than 32 segments.
 */
bppsa_status bppsa_scan_h128_diag(int T, int B, const float* Jt, const float* seed,
                                  float* G, float* g0,
                                  void* workspace, size_t workspace_bytes, void* stream,
                                  int chain_segments, int slab_segments, int last_slab_steps);

/*
 * Plain streaming copy dst[i] = src[i] of n fp32 values (n a multiple of 4,
 * both pointers 16-byte aligned, non-overlapping).  It moves exactly 4n bytes
 * in and 4n bytes out of HBM, which makes it the unit against which hardware
 * traffic counters are scaled when the scan's HBM traffic is reported.
 * Errors: BPPSA_EINVAL (null pointer, n < 1), BPPSA_ESHAPE (n % 4 != 0 or a
 * misaligned pointer).
 */
bppsa_status bppsa_calibration_copy(const float* src, float* dst, int64_t n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BPPSA_H */
