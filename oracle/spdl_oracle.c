/*
 * CPU oracle for CSR SpMM and SDDMM.  TEST INFRASTRUCTURE ONLY: nothing on the product
 * path may call this; only tests, the smoke check and the benchmark's cpu_baseline leg do.
 *
 * Both operations are finite sums fully determined by their inputs, so the oracle is the
 * definition written out, accumulated in double precision from the stored fp32 (or fp16)
 * inputs.  Next to every result it returns the tolerance scale S = sum of |product|.
 *
 *   SpMM  (paper Sec. "Sparse Matrix--Matrix Multiplication Operation":  A B => C,
 *          A in CSR, B and C dense row-major, Sec. "Data Organization")
 *   SDDMM (paper Sec. "Sampled Dense--Dense Matrix Multiplication Operation":
 *          L R^T sampled at the nonzero positions of A, with no scaling by A's values)
 *   Row order (paper Sec. "Row Binning & Row Bundling Heuristics": row indices sorted by
 *          decreasing row length; ties keep ascending row index)
 *
 * No blocking, fusion or reordering: loops run i, then the row's nonzeros p, then j.
 * Shares no code with the GPU library.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int t) {
#ifdef _OPENMP
  if (t > 0) omp_set_num_threads(t);
#else
  (void)t;
#endif
}

/* IEEE 754 binary16 -> double, written from the format definition:
 * 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits. */
static double half_bits_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1f;
  int f = h & 0x3ff;
  double mag;
  if (e == 0) {
    mag = ldexp((double)f, -24);                 /* subnormal: f * 2^-10 * 2^-14 */
  } else if (e == 31) {
    mag = f ? NAN : INFINITY;
  } else {
    mag = ldexp(1.0 + (double)f / 1024.0, e - 15);
  }
  return sign ? -mag : mag;
}

/* C[i,j] = sum_p values[p] * B[column_indices[p], j],  S[i,j] = sum_p |...| */
void oracle_spmm_f32(int m, int k, int n, const int32_t* row_offsets, const int32_t* column_indices,
                     const float* values, const float* B, double* C, double* S) {
  (void)k;
#pragma omp parallel for schedule(dynamic, 16)
  for (int i = 0; i < m; ++i) {
    double* c = C + (size_t)i * n;
    double* s = S + (size_t)i * n;
    for (int j = 0; j < n; ++j) { c[j] = 0.0; s[j] = 0.0; }
    for (int p = row_offsets[i]; p < row_offsets[i + 1]; ++p) {
      double a = (double)values[p];
      const float* b = B + (size_t)column_indices[p] * n;
      for (int j = 0; j < n; ++j) {
        double prod = a * (double)b[j];
        c[j] += prod;
        s[j] += fabs(prod);
      }
    }
  }
}

void oracle_spmm_f16(int m, int k, int n, const int32_t* row_offsets, const int32_t* column_indices,
                     const uint16_t* values, const uint16_t* B, double* C, double* S) {
  (void)k;
#pragma omp parallel for schedule(dynamic, 16)
  for (int i = 0; i < m; ++i) {
    double* c = C + (size_t)i * n;
    double* s = S + (size_t)i * n;
    for (int j = 0; j < n; ++j) { c[j] = 0.0; s[j] = 0.0; }
    for (int p = row_offsets[i]; p < row_offsets[i + 1]; ++p) {
      double a = half_bits_to_double(values[p]);
      const uint16_t* b = B + (size_t)column_indices[p] * n;
      for (int j = 0; j < n; ++j) {
        double prod = a * half_bits_to_double(b[j]);
        c[j] += prod;
        s[j] += fabs(prod);
      }
    }
  }
}

/* out[p] = sum_j L[i,j] * R[column_indices[p], j] for every stored position p of row i */
void oracle_sddmm_f32(int m, int k, int n, const int32_t* row_offsets, const int32_t* column_indices,
                      const float* L, const float* R, double* out, double* S) {
  (void)k;
#pragma omp parallel for schedule(dynamic, 16)
  for (int i = 0; i < m; ++i) {
    const float* l = L + (size_t)i * n;
    for (int p = row_offsets[i]; p < row_offsets[i + 1]; ++p) {
      const float* r = R + (size_t)column_indices[p] * n;
      double acc = 0.0, sc = 0.0;
      for (int j = 0; j < n; ++j) {
        double prod = (double)l[j] * (double)r[j];
        acc += prod;
        sc += fabs(prod);
      }
      out[p] = acc;
      S[p] = sc;
    }
  }
}

/* General SDDMM (paper Sec. "Sampled Dense--Dense Matrix Multiplication Operation", the strict
 * definition and its footnote): the sampled products scaled element-wise by the values of the
 * sparse matrix, out[p] = values[p] * sum_j L[i,j] R[c_p,j].  S[p] = |values[p]| * sum |L R|. */
void oracle_sddmm_scaled_f32(int m, int k, int n, const int32_t* row_offsets, const int32_t* column_indices,
                             const float* values, const float* L, const float* R, double* out, double* S) {
  oracle_sddmm_f32(m, k, n, row_offsets, column_indices, L, R, out, S);
  for (int p = 0; p < row_offsets[m]; ++p) {
    out[p] *= (double)values[p];
    S[p] *= fabs((double)values[p]);
  }
}

/* SDDMM with the right-hand operand not transposed (same section, footnote: the general form
 * takes the dense product L Rn with Rn of shape n x k, row-major):
 * out[p] = sum_j L[i,j] * Rn[j, c_p].  Not scaled by A's values. */
void oracle_sddmm_nt_f32(int m, int k, int n, const int32_t* row_offsets, const int32_t* column_indices,
                         const float* L, const float* Rn, double* out, double* S) {
#pragma omp parallel for schedule(dynamic, 16)
  for (int i = 0; i < m; ++i) {
    const float* l = L + (size_t)i * n;
    for (int p = row_offsets[i]; p < row_offsets[i + 1]; ++p) {
      const int c = column_indices[p];
      double acc = 0.0, sc = 0.0;
      for (int j = 0; j < n; ++j) {
        double prod = (double)l[j] * (double)Rn[(size_t)j * k + c];
        acc += prod;
        sc += fabs(prod);
      }
      out[p] = acc;
      S[p] = sc;
    }
  }
}

void oracle_sddmm_f16(int m, int k, int n, const int32_t* row_offsets, const int32_t* column_indices,
                      const uint16_t* L, const uint16_t* R, double* out, double* S) {
  (void)k;
#pragma omp parallel for schedule(dynamic, 16)
  for (int i = 0; i < m; ++i) {
    const uint16_t* l = L + (size_t)i * n;
    for (int p = row_offsets[i]; p < row_offsets[i + 1]; ++p) {
      const uint16_t* r = R + (size_t)column_indices[p] * n;
      double acc = 0.0, sc = 0.0;
      for (int j = 0; j < n; ++j) {
        double prod = half_bits_to_double(l[j]) * half_bits_to_double(r[j]);
        acc += prod;
        sc += fabs(prod);
      }
      out[p] = acc;
      S[p] = sc;
    }
  }
}

/* Rows by decreasing length; among equal lengths the smaller row index comes first.
 * Plain selection by length value: longest length first, rows scanned in ascending order. */
void oracle_row_order(int m, const int32_t* row_offsets, int32_t* row_order) {
  int max_len = 0;
  for (int i = 0; i < m; ++i) {
    int len = row_offsets[i + 1] - row_offsets[i];
    if (len > max_len) max_len = len;
  }
  /* bucket counts per length keep this O(m + max_len) without changing the definition */
  int64_t* start = (int64_t*)calloc((size_t)max_len + 2, sizeof(int64_t));
  for (int i = 0; i < m; ++i) start[row_offsets[i + 1] - row_offsets[i]]++;
  int64_t pos = 0;
  for (int len = max_len; len >= 0; --len) { int64_t c = start[len]; start[len] = pos; pos += c; }
  for (int i = 0; i < m; ++i) {
    int len = row_offsets[i + 1] - row_offsets[i];
    row_order[start[len]++] = i;
  }
  free(start);
}

/* Softmax over the stored entries of every CSR row, on scaled logits (paper Sec. "Application:
 * Sparse Transformer": softmax(Q K^T / sqrt(d_k)) restricted to the sparse topology):
 *   out[p] = exp(scale*x[p] - M_i) / sum_q exp(scale*x[q] - M_i),  M_i = max_q scale*x[q],
 * q ranging over the entries of the row that holds p.  Rows without entries produce nothing.
 * Double precision throughout; the maximum is subtracted as in the textbook formulation. */
void oracle_csr_softmax_f32(int m, const int32_t* row_offsets, const float* x, double scale, double* out) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int i = 0; i < m; ++i) {
    const int s = row_offsets[i], e = row_offsets[i + 1];
    if (e <= s) continue;
    double mx = scale * (double)x[s];
    for (int p = s + 1; p < e; ++p) {
      double v = scale * (double)x[p];
      if (v > mx) mx = v;
    }
    double sum = 0.0;
    for (int p = s; p < e; ++p) sum += exp(scale * (double)x[p] - mx);
    for (int p = s; p < e; ++p) out[p] = exp(scale * (double)x[p] - mx) / sum;
  }
}

/* Fused epilogue of the sparse 1x1 convolution (paper Sec. "Application: Sparse MobileNetV1":
 * bias and ReLU fused into the SpMM):  C[i,j] = max(0, sum_p values[p]*B[col[p],j] + bias[i]).
 * S[i,j] = sum_p |product| + |bias[i]| is the tolerance scale. */
void oracle_spmm_bias_relu_f32(int m, int k, int n, const int32_t* row_offsets, const int32_t* column_indices,
                               const float* values, const float* B, const float* bias, int relu, double* C,
                               double* S) {
  oracle_spmm_f32(m, k, n, row_offsets, column_indices, values, B, C, S);
#pragma omp parallel for
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) {
      double b = bias ? (double)bias[i] : 0.0;      /* no bias given: the epilogue adds nothing */
      double v = C[(size_t)i * n + j] + b;
      C[(size_t)i * n + j] = (relu && !(v > 0.0)) ? 0.0 : v;
      S[(size_t)i * n + j] += fabs(b);
    }
}

/* Transposed topology for A^T B (paper Sec. "Discussion & Conclusion": cache the row offsets
 * and column indices of A^T when the topology changes and move the values with a permutation).
 * Entry p of A at (i, c) becomes an entry of row c of A^T with column i; within a row of A^T
 * entries are ordered by ascending i (the order in which a row-major scan of A meets them).
 * perm[t] = position in A of the t-th entry of A^T. */
void oracle_transpose_topology(int m, int k, const int32_t* row_offsets, const int32_t* column_indices,
                               int32_t* t_row_offsets, int32_t* t_column_indices, int32_t* perm) {
  for (int c = 0; c <= k; ++c) t_row_offsets[c] = 0;
  for (int p = 0; p < row_offsets[m]; ++p) t_row_offsets[column_indices[p] + 1]++;
  for (int c = 0; c < k; ++c) t_row_offsets[c + 1] += t_row_offsets[c];
  int32_t* cursor = (int32_t*)malloc(sizeof(int32_t) * (size_t)(k > 0 ? k : 1));
  for (int c = 0; c < k; ++c) cursor[c] = t_row_offsets[c];
  for (int i = 0; i < m; ++i)
    for (int p = row_offsets[i]; p < row_offsets[i + 1]; ++p) {
      int t = cursor[column_indices[p]]++;
      t_column_indices[t] = i;
      perm[t] = p;
    }
  free(cursor);
}
