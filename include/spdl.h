/*
 * libspdl -- CSR SpMM and SDDMM for deep-learning sparsity on AMD gfx950 (MI355X), with the
 * operations around them: fused bias + ReLU, softmax over CSR rows, transposed topology, value
 * scaling.
 *
 * C ABI.  Every pointer is marked HOST or DEVICE.  The library never allocates, frees or
 * keeps a caller's pointer, and never writes an input array.  Kernels are enqueued on
 * `stream` (a hipStream_t passed as void*; NULL = the default stream) with no host
 * synchronisation.  Every function returns an spdl_status and never throws, aborts or
 * prints.
 *
 * Common conventions
 *   A is an m x k sparse matrix in the standard compressed-sparse-row format
 *   (paper Sec. "Data Organization"):
 *     row_offsets     int32[m+1], row_offsets[0] == 0, non-decreasing, row_offsets[m] == nnz
 *     column_indices  int32[nnz], each in [0,k); any order inside a row (duplicates allowed:
 *                     SpMM sums them, SDDMM produces one output per stored entry).  Rows with
 *                     ascending indices take the fastest path.
 *     values          [nnz]
 *   Dense matrices are row-major with no padding (leading dimension == number of columns).
 *   Sizes: m, k, n, nnz >= 0 and m*n, k*n < 2^31.  m == 0, n == 0 and nnz == 0 are valid.
 *   Base pointers must be aligned to their element type; 16-byte aligned bases and n % 4 == 0
 *   (n % 8 == 0 for fp16) select the widest vector path, anything else a narrower one.
 *   Non-finite inputs.  With finite inputs every result is the definition's.  An Inf or NaN in
 *   a row of a dense operand reaches the outputs that the definition makes depend on that row
 *   in every kernel; all SDDMM kernels, the fp32 SpMM kernels and the direct fp16 SpMM kernel
 *   keep it away from every other output.  The fp16 matrix-core SpMM (chosen when at least one
 *   position in 32 of A is stored, n % 8 == 0, 16-byte aligned operands) multiplies the zeros of
 *   its expanded sparse panels by whole rows of B: there a non-finite B[k, j] turns C[i, j] into
 *   NaN for every row i (other columns of C are not affected).  Callers whose fp16 activations
 *   can overflow select the direct kernel with spdl_force_variant(0, 0), which follows the
 *   definition exactly.
 */
#ifndef SPDL_H_
#define SPDL_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPDL_OK = 0,
  SPDL_ERR_INVALID = -1,      /* negative size, null required pointer, size overflow          */
  SPDL_ERR_LAUNCH = -2,       /* the HIP runtime refused a launch (hipGetLastError != success) */
  SPDL_ERR_BAD_CSR = -3,      /* spdl_validate_csr_host: arrays are not a valid CSR topology   */
  SPDL_ERR_UNSUPPORTED = -4,  /* a forced kernel variant cannot run this problem              */
  SPDL_ERR_NOMEM = -5         /* a host routine could not allocate its working memory          */
} spdl_status;

/* SpMM:  C = A B.   (paper Sec. "Sparse Matrix--Matrix Multiplication Operation")
 *   C[i,j] = sum over stored entries p of row i of values[p] * B[column_indices[p], j].
 *   row_offsets, column_indices, values : DEVICE, CSR of A (m x k, nnz entries), fp32 values
 *   row_order : DEVICE int32[m], a permutation of [0,m) giving the order in which rows are
 *               handed to workgroups (paper Sec. "Row Swizzle Load Balancing"); NULL = identity.
 *               The result does not depend on it.
 *   B : DEVICE fp32[k*n];   C : DEVICE fp32[m*n], fully overwritten (empty rows become +0).
 *   Products and sums are fp32 (fused multiply-adds).  Most kernels add a row's products in
 *   stored order; when few long rows are spread over several lane groups, and in the kernel for
 *   attention-shaped problems (33..64 columns, which keeps a window of B around a band of A in
 *   on-chip memory and takes rows in their natural order), partial sums are added at the end.
 *   Either way the result is deterministic and does not depend on row_order. */
int spdl_spmm(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
              const float* values, const int* row_order, const float* B, float* C, void* stream);

/* SDDMM:  out = (L R^T) sampled at A's stored positions, without scaling by A's values.
 *   (paper Sec. "Sampled Dense--Dense Matrix Multiplication Operation")
 *   out_values[p] = sum_j L[i,j] * R[column_indices[p], j] for every entry p of row i.
 *   row_offsets, column_indices : DEVICE, topology of A (m x k)
 *   L : DEVICE fp32[m*n];  R : DEVICE fp32[k*n];  out_values : DEVICE fp32[nnz], CSR order,
 *   fully overwritten.  out_values may be the array that holds A's values (they are not read). */
int spdl_sddmm(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
               const float* L, const float* R, float* out_values, void* stream);

/* SpMM and SDDMM for a sparse matrix whose entries cluster around a band: the attention masks of
 * paper Sec. "Application: Sparse Transformer" (a dense band along the diagonal plus scattered
 * entries).  Same operations, arguments and results as spdl_spmm (without a row order: rows are
 * taken in their natural order, neighbours share the band) and spdl_sddmm; the only difference is
 * the choice of kernel, which the library cannot make by itself because it never reads the
 * topology on the host: a window of the dense operand around the band is kept in on-chip memory
 * and only the scattered entries are gathered.  Where the band is, and whether there is one, is
 * found on the device; without a band every entry is gathered and the result is still right.
 * Used as given for fp32 with n % 4 == 0, 16-byte aligned dense operands and k*n < 2^29 (SDDMM:
 * n <= 128); any other problem runs exactly as through spdl_spmm / spdl_sddmm.  spdl_spmm and
 * spdl_sddmm pick these kernels themselves for shapes like that of an attention head (thousands of
 * rows of a hundred entries or more, 33..128 columns), where they are also the faster way to
 * gather. */
int spdl_spmm_banded(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                     const float* values, const float* B, float* C, void* stream);
int spdl_sddmm_banded(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                      const float* L, const float* R, float* out_values, void* stream);

/* SpMM and SDDMM for a sparse matrix whose rows are of strongly unequal length (a few rows of
 * thousands of entries among rows of tens or hundreds: the heavy-tailed row lengths that paper
 * Sec. "Row Swizzle Load Balancing" is about, beyond what reordering rows evens out).  Same
 * operations, arguments and results as spdl_spmm (without a row order) and spdl_sddmm; the only
 * difference is the choice of kernel, which the library cannot make by itself because it never
 * reads the row lengths on the host: kernels whose work per wave does not depend on the length of
 * a row (SpMM: a wave per row, what a row holds beyond its share dealt to all waves of the
 * workgroup; SDDMM: the entries split evenly over the waves, or for dot products of more than 256
 * columns the kernel estimated faster without the one that keeps partial sums per row).  fp32,
 * n % 4 == 0, 16-byte aligned dense operands and k*n < 2^29; any other problem runs exactly as
 * through spdl_spmm / spdl_sddmm.  On matrices with rows of similar length these entry points are
 * up to twice as slow as spdl_spmm / spdl_sddmm. */
int spdl_spmm_skewed(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                     const float* values, const float* B, float* C, void* stream);
int spdl_sddmm_skewed(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                      const float* L, const float* R, float* out_values, void* stream);

/* SDDMM with the row order of SpMM (paper Sec. "Row Swizzle Load Balancing"; the paper applies the
 * swizzle to SpMM, the kernels here that give a sparse row to one lane group profit in the same way):
 *   row_order : DEVICE int32[m], a permutation of [0,m) (spdl_build_row_order), or NULL.
 *   It changes which workgroup computes which row, never a result; kernels that split the work by
 *   nonzeros ignore it.  Everything else as spdl_sddmm. */
int spdl_sddmm_ordered(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                       const int* row_order, const float* L, const float* R, float* out_values, void* stream);

/* General SDDMM (same section: the strict definition, with the element-wise scaling by the sparse
 * matrix that the deep-learning form leaves out; the footnote there prices it at one load and
 * one multiply before the store):
 *   out_values[p] = values[p] * sum_j L[i,j] * R[column_indices[p], j].
 *   values : DEVICE [nnz], the stored values of A; must not be the array out_values (an entry may
 *   be computed more than once when a row's indices are not ascending).  Everything else as
 *   spdl_sddmm.  The dot product is formed as in spdl_sddmm and multiplied once, in fp32; the
 *   fp16 version rounds to binary16 after the multiplication. */
int spdl_sddmm_scaled(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                      const float* values, const float* L, const float* R, float* out_values, void* stream);
int spdl_sddmm_scaled_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                          const uint16_t* values, const uint16_t* L, const uint16_t* R, uint16_t* out_values,
                          void* stream);

/* SDDMM with the right-hand operand not transposed (same footnote: the general form multiplies
 * L by an n x k matrix):
 *   out_values[p] = sum_j L[i,j] * Rn[j, column_indices[p]]   (times values[p] when values != NULL).
 *   Rn : DEVICE [n*k], row-major n x k.  values : DEVICE [nnz] or NULL; not the array out_values.
 *   Everything else as spdl_sddmm; k*n < 2^31.  Any n and alignment; fp32 with n % 4 == 0,
 *   n <= 128, k % 4 == 0 and 16-byte aligned L and Rn runs at about the speed of spdl_sddmm (slabs of
 *   Rn are transposed on the chip), everything else in a plain kernel an order of magnitude slower. */
int spdl_sddmm_nt(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                  const float* values, const float* L, const float* Rn, float* out_values, void* stream);
int spdl_sddmm_nt_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                      const uint16_t* values, const uint16_t* L, const uint16_t* Rn, uint16_t* out_values,
                      void* stream);

/* Mixed precision (paper Sec. "Mixed Precision"): operands and results are IEEE binary16
 * (passed as uint16_t bit patterns), every product and sum is fp32, results are rounded to
 * binary16 once (round to nearest even).  Column indices stay int32. */
int spdl_spmm_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                  const uint16_t* values, const int* row_order, const uint16_t* B, uint16_t* C,
                  void* stream);
int spdl_sddmm_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                   const uint16_t* L, const uint16_t* R, uint16_t* out_values, void* stream);
/* The same section's 16-bit column indices (they halve the index traffic of the sparse matrix):
 * spdl_spmm_f16 with column_indices : DEVICE int16[nnz], each in [0,k), k <= 32767 (larger k:
 * SPDL_ERR_INVALID).  Row offsets stay int32. */
int spdl_spmm_f16_i16(int m, int k, int n, int nnz, const int* row_offsets, const int16_t* column_indices,
                      const uint16_t* values, const int* row_order, const uint16_t* B, uint16_t* C,
                      void* stream);

/* SpMM with a fused epilogue (paper Sec. "Application: Sparse MobileNetV1": bias and ReLU are
 * fused into the sparse 1x1 convolution, whose weights are the sparse matrix and whose rows
 * are the output channels):
 *   C[i,j] = act( sum_p values[p] * B[column_indices[p], j] + bias[i] ),  act = max(., 0) when
 *   relu != 0, identity otherwise.
 *   bias : DEVICE [m], one value per row of A; NULL = no bias.  Everything else as spdl_spmm.
 *   The sum is formed exactly as in spdl_spmm, the bias is added to it in fp32, and in the fp16
 *   version the result is rounded to binary16 once, after the activation. */
int spdl_spmm_bias_relu(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                        const float* values, const int* row_order, const float* B, const float* bias,
                        int relu, float* C, void* stream);
int spdl_spmm_bias_relu_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                            const uint16_t* values, const int* row_order, const uint16_t* B,
                            const uint16_t* bias, int relu, uint16_t* C, void* stream);

/* Softmax over the stored entries of each row of a CSR matrix (paper Sec. "Application: Sparse
 * Transformer": the attention weights are the softmax of the sampled, scaled scores):
 *   probabilities[p] = exp(scale*logits[p] - M_i) / sum_q exp(scale*logits[q] - M_i),
 *   q over the entries of the row i that holds p, M_i = max_q scale*logits[q].
 *   row_offsets : DEVICE int32[m+1];  logits : DEVICE fp32[nnz];  probabilities : DEVICE
 *   fp32[nnz], fully overwritten, may be the same array as logits.  Empty rows produce nothing.
 *   A row that holds +inf or NaN produces NaN in that row (as the definition does). */
int spdl_csr_softmax(int m, int nnz, const int* row_offsets, const float* logits, float scale,
                     float* probabilities, void* stream);

/* Topology of the transpose (paper Sec. "Discussion & Conclusion": with a fixed topology the
 * transposed offsets and indices are computed once and cached, and the transposed values are
 * a permutation of the values).  Pure host code.
 *   row_offsets_host, column_indices_host : HOST, CSR topology of A (m x k, nnz entries)
 *   t_row_offsets_host : HOST int32[k+1], t_column_indices_host : HOST int32[nnz], written: the
 *     CSR topology of A^T (k x m); inside a row of A^T the entries are in ascending row index
 *     of A (entries of equal row in their stored order).
 *   perm_host : HOST int32[nnz], written: entry t of A^T is entry perm[t] of A.
 *   Returns SPDL_ERR_BAD_CSR when the input is not a valid topology (nothing defined is written).
 *   Allocates nothing. */
int spdl_build_transpose_host(int m, int k, int nnz, const int* row_offsets_host,
                              const int* column_indices_host, int* t_row_offsets_host,
                              int* t_column_indices_host, int* perm_host);

/* out[t] = values[perm[t]] for t in [0,nnz): the values of A^T from those of A (same passage).
 *   perm : DEVICE int32[nnz], each in [0,nnz);  values, out : DEVICE, nnz elements of elem_bytes
 *   (2 or 4) bytes each, distinct arrays.  With the arrays of spdl_build_transpose_host,
 *   spdl_spmm on (k, m, t_row_offsets, t_column_indices, out) computes A^T B. */
int spdl_permute_values(int nnz, int elem_bytes, const int* perm, const void* values, void* out,
                        void* stream);

/* Row swizzle (paper Sec. "Row Binning & Row Bundling Heuristics"): row indices sorted by
 * decreasing row length, equal lengths in ascending row index.  Pure host code.
 *   row_offsets_host : HOST int32[m+1];   row_order_host : HOST int32[m], written.
 *   SPDL_ERR_NOMEM if the sort cannot get its merge buffer. */
int spdl_build_row_order(int m, const int* row_offsets_host, int* row_order_host);

/* Host-side check of a CSR topology: offsets start at 0, never decrease, end at nnz; every
 * column index lies in [0,k).  Returns SPDL_OK or SPDL_ERR_BAD_CSR.  If sorted_out is not
 * NULL it receives 1 when every row's indices are strictly ascending, else 0.
 *   row_offsets_host : HOST int32[m+1];  column_indices_host : HOST int32[nnz]. */
int spdl_validate_csr_host(int m, int k, int nnz, const int* row_offsets_host,
                           const int* column_indices_host, int* sorted_out);

/* Kernel selection (paper Sec. "Experiments", first paragraph: tile sizes and vector widths
 * are picked from the problem shape).  spdl_select_* report what the dispatcher would launch;
 * spdl_force_variant overrides it for ablation runs (variant < 0 restores the heuristic); a
 * forced variant that cannot run the problem at hand falls back to one that can.  The override
 * is one process-wide setting per operation, read by every later call on any thread: it is not
 * meant to be changed while other threads are inside the library.
 * The variant ids are listed by spdl_variant_name. */
typedef struct {
  int variant;          /* kernel family id                                        */
  int vec;              /* elements per lane per memory instruction                */
  int lanes_per_row;    /* lanes cooperating on one output row / one dot product   */
  int rows_per_block;   /* SpMM: sparse rows per block.  SDDMM: waves per row, or for the   */
                        /* group variant the CSR entries owned by one wave                */
  int block_threads;
  int grid_x, grid_y;
} spdl_launch_info;
int spdl_select_spmm(int m, int k, int n, int nnz, int elem_bytes, const void* B, const void* C,
                     spdl_launch_info* info);
int spdl_select_sddmm(int m, int k, int n, int nnz, int elem_bytes, const void* L, const void* R,
                      spdl_launch_info* info);
int spdl_force_variant(int op /*0 = SpMM, 1 = SDDMM*/, int variant);
const char* spdl_variant_name(int op, int variant);   /* NULL if no such variant */

const char* spdl_status_string(int status);
int spdl_version(void);

#ifdef __cplusplus
}
#endif
#endif  /* SPDL_H_ */
