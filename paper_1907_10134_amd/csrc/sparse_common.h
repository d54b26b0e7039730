// Internal launchers of the sparse kernels, shared by the builders and the sparse scan.
#pragma once

#include "bppsa_internal.h"

// In place: a[0..n) holds row lengths on entry, the exclusive prefix sum on exit; a[n] = total.
bppsa_status bppsa_lengths_to_indptr(int32_t* a, int n, hipStream_t stream);

// y = A x.  With a diagonal D given by its values d (one per row of A), y2 = D y is written
// as well: the product with a diagonal matrix that follows in a chain costs no launch.
bppsa_status bppsa_launch_spmv(const bppsa_csr& A, const float* x, float* y, hipStream_t stream,
                               const float* d = nullptr, float* y2 = nullptr);

// *flag (device int, preset to 1 by the caller) is cleared if A is not square with exactly the
// entries (i, i), i.e. indptr[i] = i and indices[i] = i.
bppsa_status bppsa_launch_check_diagonal(const bppsa_csr& A, int* flag, hipStream_t stream);

// Structural product C = A B.
// Pass 1 writes the length of every row of C into c_indptr[0..rows) and adds the number of
// multiply-adds of the product to *madds (device, 64-bit); the caller turns lengths into
// row pointers with bppsa_lengths_to_indptr.  Pass 2 writes the ascending column indices.
bppsa_status bppsa_launch_spgemm_count(const bppsa_csr& A, const bppsa_csr& B, int32_t* c_indptr,
                                       unsigned long long* madds, hipStream_t stream);
bppsa_status bppsa_launch_spgemm_indices(const bppsa_csr& A, const bppsa_csr& B, const int32_t* c_indptr,
                                         int32_t* c_indices, hipStream_t stream);
// Values of C for a known structure (c_indptr, c_indices); c_data is overwritten.  `kind` says
// which kernel forms them and is chosen once per product from the number of multiply-adds, nnz(C),
// the longest row of C (c_max_row, which the launch takes again to size LDS) and the number of
// columns of B; the BLOCK kinds also need the table b_split [3 * rows(B)] that
// bppsa_launch_row_splits writes for B.
enum {
  BPPSA_SPGEMM_SINGLE = 0,        // no value of C is a sum: nothing to order
  BPPSA_SPGEMM_WAVE = 1,          // one wave per row, the row staged in LDS
  BPPSA_SPGEMM_BLOCK_DENSE = 2,   // one workgroup per row, one LDS accumulator per column of B
  BPPSA_SPGEMM_BLOCK_STAGED = 3,  // one workgroup per row, one LDS accumulator per entry of the row
  BPPSA_SPGEMM_BLOCK_GLOBAL = 4   // one workgroup per row, accumulated in global memory
};
int bppsa_spgemm_numeric_kind(int64_t madds, int64_t c_nnz, int c_max_row, int b_cols);
bppsa_status bppsa_launch_row_splits(const bppsa_csr& B, int32_t* split, hipStream_t stream);
bppsa_status bppsa_launch_spgemm_numeric(int kind, const bppsa_csr& A, const bppsa_csr& B, const int32_t* b_split,
                                         const int32_t* c_indptr, const int32_t* c_indices, float* c_data,
                                         int c_max_row, hipStream_t stream);

// Adds a fingerprint of up to BPPSA_HASH_BATCH index arrays (values and their positions; `salt`
// tells arrays apart) to the two 64-bit words at out (device), in one launch.  The sums do not
// depend on the order of the additions.  The batch travels by value as a kernel argument.
#define BPPSA_HASH_BATCH 64
struct bppsa_hash_batch {
  const int32_t* array[BPPSA_HASH_BATCH];
  long long count[BPPSA_HASH_BATCH];
  unsigned long long salt[BPPSA_HASH_BATCH];
};
bppsa_status bppsa_launch_pattern_hash(const bppsa_hash_batch& batch, int n, unsigned long long* out,
                                       hipStream_t stream);

constexpr int kBppsaMaxSpgemmCols = 1 << 20;  // LDS bitmap: one bit per column of B
