/*
 * Bi-GCN forward pass: plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, literal definition of what the
 * HIP library computes.  It shares no code with that library and must never be
 * called from the product path; only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg may load it.
 *
 * Everything is written as the paper's equations read (Sec. 3.1 Notations, Sec. 3.2
 * Eq. (1), Sec. 4.1 vector binarisation, Sec. 4.2.1-4.2.3): signs are kept as one
 * int8 per element (no bit packing), the +-1 products are literal integer
 * multiply-adds, and every floating-point quantity is accumulated in fp64.  The only
 * parallelism is an OpenMP "parallel for" over independent output rows.
 *
 * Readings of the paper taken here (each also listed in the design notes):
 *  - the scale of a binarised vector is its L1 norm divided by its own length t
 *    (Sec. 4.1, alpha* = ||V||_1 / t); the per-column weight scale therefore divides by
 *    d_in and the per-node feature scale by d_in as well, although the equations of
 *    Sec. 4.2.1 / 4.2.2 print 1/d_out and 1/N;
 *  - sign(0) is taken as +1 so that the binary vector lies in {-1,+1}^t: an element is
 *    +1 iff  x >= threshold, where the threshold is the standardisation mean of its
 *    column (0 when no standardisation is given), compared in fp32;
 *  - no bias, no ReLU, no dropout (Sec. 4.2.2: binarisation acts as the activation).
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stddef.h>
#include <stdint.h>

/* ------------------------------------------------------------------------- */
/* Sec. 3.1 / Eq. (1):  A~ = D^-1/2 (A + I) D^-1/2,  D_ii = sum_j (A+I)_ij.      */
/* The CSR pattern handed in is that of A + I (unweighted, self-loop present), */
/* so D_ii is the number of stored entries of row i.                          */
/* a_tilde[p] = 1 / sqrt(D_ii * D_kk) for the p-th stored entry (i, k).        */
/* ------------------------------------------------------------------------- */
void oracle_gcn_norm(int64_t n, const int64_t *row_ptr, const int32_t *col_idx, double *a_tilde)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n; ++i) {
        double d_i = (double)(row_ptr[i + 1] - row_ptr[i]);
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t k = col_idx[p];
            double d_k = (double)(row_ptr[k + 1] - row_ptr[k]);
            a_tilde[p] = 1.0 / sqrt(d_i * d_k);
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.1 (V_B* = sign(V), alpha* = ||V||_1 / t) applied to each row of a    */
/* strided fp32 matrix: element (r, c) is x[r*row_stride + c*col_stride].      */
/* Optional per-column standardisation (Sec. 4.4, step 1): x' = (x - shift[c]) */
/* * mul[c]; shift == NULL means 0, mul == NULL means 1.                        */
/*   sign[r*cols + c] = +1 if x >= shift[c] (fp32 compare) else -1             */
/*   scale[r]         = (1/cols) * sum_c |x'|                                  */
/* Rows of H give (F_i, beta_i) of Sec. 4.2.2; rows of W^T (row_stride = 1,    */
/* col_stride = d_out) give (B_j, alpha_j) of Sec. 4.2.1.                       */
/* ------------------------------------------------------------------------- */
void oracle_binarize_rows_f32(const float *x, int64_t rows, int64_t cols, int64_t row_stride,
                              int64_t col_stride, const float *shift, const float *mul,
                              int8_t *sign, double *scale)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double l1 = 0.0;
        for (int64_t c = 0; c < cols; ++c) {
            float v = x[r * row_stride + c * col_stride];
            float th = shift ? shift[c] : 0.0f;
            double m = mul ? (double)mul[c] : 1.0;
            sign[r * cols + c] = (v >= th) ? (int8_t)1 : (int8_t)-1;
            l1 += fabs(((double)v - (double)th) * m);
        }
        scale[r] = l1 / (double)cols;
    }
}

/* Same, for a dense row-major fp64 matrix (the oracle's own hidden activations).
 * The sign decision is taken on the value rounded to fp32, the precision in which the
 * activations exist in the method's fp32 arithmetic; the scale uses the fp64 value. */
void oracle_binarize_rows_f64(const double *h, int64_t rows, int64_t cols, const float *shift,
                              const float *mul, int8_t *sign, double *scale)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double l1 = 0.0;
        for (int64_t c = 0; c < cols; ++c) {
            double v = h[r * cols + c];
            float th = shift ? shift[c] : 0.0f;
            double m = mul ? (double)mul[c] : 1.0;
            sign[r * cols + c] = ((float)v >= th) ? (int8_t)1 : (int8_t)-1;
            l1 += fabs((v - (double)th) * m);
        }
        scale[r] = l1 / (double)cols;
    }
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.2.3, the inner product F_{i,:} . B_{:,j} of two +-1 vectors, written  */
/* as the literal sum of products.  f is (m, k) row-major, bt is (n, k)        */
/* row-major (row j of bt is column j of B).  acc[i*n + j] = sum_t f_it b_tj.  */
/* ------------------------------------------------------------------------- */
void oracle_sign_matmul(const int8_t *f, const int8_t *bt, int64_t m, int64_t k, int64_t n,
                        int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        for (int64_t j = 0; j < n; ++j) {
            int32_t s = 0;
            for (int64_t t = 0; t < k; ++t)
                s += (int32_t)f[i * k + t] * (int32_t)bt[j * k + t];
            acc[i * n + j] = s;
        }
    }
}

/* Sec. 4.2.3:  zeta_ij = beta_i * alpha_j * (F_{i,:} . B_{:,j}). */
void oracle_rescale(const int32_t *acc, const double *beta, const double *alpha, int64_t m,
                    int64_t n, double *zeta)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j)
            zeta[i * n + j] = beta[i] * alpha[j] * (double)acc[i * n + j];
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.2.3:  H_b^(l+1) = A~ zeta^(l), as an explicit sum over the stored     */
/* neighbours of each node (self-loop included), in CSR order.                 */
/*   out[i*d + j] = sum_{p in row i} a_tilde[p] * z[col_idx[p]*d + j]           */
/* ------------------------------------------------------------------------- */
void oracle_aggregate(int64_t n, const int64_t *row_ptr, const int32_t *col_idx,
                      const double *a_tilde, const double *z, int64_t d, double *out)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < d; ++j)
            out[i * d + j] = 0.0;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            const double *zk = z + (int64_t)col_idx[p] * d;
            double a = a_tilde[p];
            for (int64_t j = 0; j < d; ++j)
                out[i * d + j] += a * zk[j];
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1, first line:  dL/dzeta = A~^T dL/dH^(l+1), written as the          */
/* transpose of the sum above: entry p of row i sends a_tilde[p] * g[i, :] to     */
/* row col_idx[p].  No symmetry of the pattern is assumed.  Threads own disjoint  */
/* column ranges, so every output element is summed in CSR order by one thread.   */
/* ------------------------------------------------------------------------- */
void oracle_aggregate_transposed(int64_t n, const int64_t *row_ptr, const int32_t *col_idx,
                                 const double *a_tilde, const double *g, int64_t d, double *out)
{
    for (int64_t e = 0; e < n * d; ++e)
        out[e] = 0.0;
#pragma omp parallel
    {
#ifdef _OPENMP
        int64_t t = omp_get_thread_num(), nt = omp_get_num_threads();
#else
        int64_t t = 0, nt = 1;
#endif
        int64_t j0 = d * t / nt, j1 = d * (t + 1) / nt;
        for (int64_t i = 0; i < n; ++i) {
            for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
                double *ok = out + (int64_t)col_idx[p] * d;
                double a = a_tilde[p];
                for (int64_t j = j0; j < j1; ++j)
                    ok[j] += a * g[i * d + j];
            }
        }
    }
}

/* Number of threads the parallel loops above use (reported by the benchmark). */
#ifdef _OPENMP
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int t) { if (t > 0) omp_set_num_threads(t); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int t) { (void)t; }
#endif
