/*
 * CPU oracle for the forward pass of a low-rank binary factorized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the GPU library must compute.  It shares no code, header, table or
 * helper with the HIP library, and the product never calls it.
 *
 * What is computed (quantization scheme, Section 3.1, Eq. 1; restated as
 * Diag(s1) U V^T Diag(s2) in Appendix F.5):
 *
 *     W^[i][j] = s_out[i] * ( sum_{k<r} U[i][k] * V[j][k] ) * s_in[j]
 *     y[b][i]  = sum_{j<d_in} W^[i][j] * x[b][j]
 *
 * with U in {-1,+1}^{d_out x r}, V in {-1,+1}^{d_in x r}; s_out is the
 * output-channel scale s1 and s_in the input-channel scale s2.
 *
 * Sign storage (Fig. 2(c): -1 -> bit 0, +1 -> bit 1).  The paper does not fix
 * a word size or bit order; the reading used by this repository is:
 * row-major over the factor's rows, packed along the rank axis, column k
 * lives in 32-bit word k/32 at bit position k%32 counted from the least
 * significant bit; unused high bits of a row's last word are 0.
 *
 * Tier A (nqo_dense_weight / nqo_forward_dense*): the definition written out.
 * Tier B (nqo_forward_factored): the same product associated the way the
 * paper evaluates it (Section 3.3, Step 2: scales only at the input and the
 * output boundary, two chained products in between):
 *     x' = s_in (.) x ;  t = V^T x' ;  y = s_out (.) (U t)
 * Tier B exists because Tier A costs d_out*d_in*r operations.
 *
 * The three-scale variant of Appendix F.4 (a rank-wise scale s_mid between the
 * two binary products; the DBF / LittleBit format) has functions of its own at
 * the end of the file, pinned the same way (numpy reduction, closed forms,
 * complete enumeration, s_mid = 1 against the two-scale code); its storage
 * formula is pinned to totals worked by hand, to a count over the arrays such a
 * layer stores, and to the 1.33 GB that Table 1 prints for a 1.00-bit
 * Llama-2-7B in this format.
 *
 * All arithmetic is IEEE double.  Inputs arrive already widened to double
 * (bf16/fp16/fp32 -> double is exact).
 */
#include <stdint.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int64_t words_per_row(int64_t cols) { return (cols + 31) / 32; }

/* sign of column k in row `row` of a packed factor: +1.0 or -1.0 */
static inline double sign_at(const uint32_t* words, int64_t wpr, int64_t row, int64_t k)
{
    uint32_t w = words[row * wpr + k / 32];
    return ((w >> (k % 32)) & 1u) ? 1.0 : -1.0;
}

/* PackBinary (Algorithm 1, the sign-and-pack step): bit = 1 iff value >= 0
 * (both zeros map to +1), bit = 0 iff value < 0.  NaN is rejected: returns -1. */
int nqo_pack_f64(const double* vals, int64_t rows, int64_t cols, uint32_t* words)
{
    int64_t wpr = words_per_row(cols);
    for (int64_t i = 0; i < rows * wpr; ++i) words[i] = 0u;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t k = 0; k < cols; ++k) {
            double v = vals[i * cols + k];
            if (isnan(v)) return -1;
            if (v >= 0.0) words[i * wpr + k / 32] |= (uint32_t)1u << (k % 32);
        }
    return 0;
}

/* Same for int8 input, which must be exactly -1 or +1: anything else returns -1. */
int nqo_pack_i8(const int8_t* vals, int64_t rows, int64_t cols, uint32_t* words)
{
    int64_t wpr = words_per_row(cols);
    for (int64_t i = 0; i < rows * wpr; ++i) words[i] = 0u;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t k = 0; k < cols; ++k) {
            int8_t v = vals[i * cols + k];
            if (v != 1 && v != -1) return -1;
            if (v == 1) words[i * wpr + k / 32] |= (uint32_t)1u << (k % 32);
        }
    return 0;
}

void nqo_unpack(const uint32_t* words, int64_t rows, int64_t cols, int8_t* out)
{
    int64_t wpr = words_per_row(cols);
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t k = 0; k < cols; ++k)
            out[i * cols + k] = (int8_t)sign_at(words, wpr, i, k);
}

/* (U V^T)[i][j]: an exact integer in [-r, r] */
static double uv_dot(const uint32_t* U, const uint32_t* V, int64_t wpr, int64_t r, int64_t i, int64_t j)
{
    double acc = 0.0;
    for (int64_t k = 0; k < r; ++k) acc += sign_at(U, wpr, i, k) * sign_at(V, wpr, j, k);
    return acc;
}

/* Tier A: dense reconstruction W^[d_out][d_in] of Eq. 1 */
void nqo_dense_weight(const uint32_t* U, const uint32_t* V, const double* s_out, const double* s_in,
                      int64_t d_out, int64_t d_in, int64_t r, double* W)
{
    int64_t wpr = words_per_row(r);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < d_out; ++i)
        for (int64_t j = 0; j < d_in; ++j)
            W[i * d_in + j] = s_out[i] * uv_dot(U, V, wpr, r, i, j) * s_in[j];
}

/* Tier A on chosen output rows: y[b][q] = sum_j W^[rows[q]][j] x[b][j] */
void nqo_forward_dense_rows(const uint32_t* U, const uint32_t* V, const double* s_out, const double* s_in,
                            int64_t d_out, int64_t d_in, int64_t r,
                            const double* x, int64_t batch,
                            const int64_t* rows, int64_t n_rows, double* y)
{
    int64_t wpr = words_per_row(r);
    (void)d_out;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < n_rows; ++q) {
        int64_t i = rows[q];
        double* Wrow = (double*)malloc(sizeof(double) * (size_t)d_in);
        for (int64_t j = 0; j < d_in; ++j)
            Wrow[j] = s_out[i] * uv_dot(U, V, wpr, r, i, j) * s_in[j];
        for (int64_t b = 0; b < batch; ++b) {
            double acc = 0.0;
            for (int64_t j = 0; j < d_in; ++j) acc += Wrow[j] * x[b * d_in + j];
            y[b * n_rows + q] = acc;
        }
        free(Wrow);
    }
}

/* Tier A, all rows */
void nqo_forward_dense(const uint32_t* U, const uint32_t* V, const double* s_out, const double* s_in,
                       int64_t d_out, int64_t d_in, int64_t r,
                       const double* x, int64_t batch, double* y)
{
    int64_t* rows = (int64_t*)malloc(sizeof(int64_t) * (size_t)d_out);
    for (int64_t i = 0; i < d_out; ++i) rows[i] = i;
    nqo_forward_dense_rows(U, V, s_out, s_in, d_out, d_in, r, x, batch, rows, d_out, y);
    free(rows);
}

/* Tier B: x' = s_in (.) x ; t = V^T x' ; y = s_out (.) (U t).
 * `t_out` (may be NULL) receives the intermediate t[batch][r].
 * Returns the number of threads that worked. */
int nqo_forward_factored(const uint32_t* U, const uint32_t* V, const double* s_out, const double* s_in,
                         int64_t d_out, int64_t d_in, int64_t r,
                         const double* x, int64_t batch, double* y, double* t_out, int threads)
{
    int64_t wpr = words_per_row(r);
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    double* xp = (double*)malloc(sizeof(double) * (size_t)d_in);
    double* t = (double*)malloc(sizeof(double) * (size_t)r);
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t j = 0; j < d_in; ++j) xp[j] = s_in[j] * x[b * d_in + j];
#pragma omp parallel
        {
#ifdef _OPENMP
#pragma omp single
            used = omp_get_num_threads();
#endif
#pragma omp for schedule(static)
            for (int64_t k = 0; k < r; ++k) {
                double acc = 0.0;
                for (int64_t j = 0; j < d_in; ++j) acc += sign_at(V, wpr, j, k) * xp[j];
                t[k] = acc;
            }
#pragma omp for schedule(static)
            for (int64_t i = 0; i < d_out; ++i) {
                double acc = 0.0;
                for (int64_t k = 0; k < r; ++k) acc += sign_at(U, wpr, i, k) * t[k];
                y[b * d_out + i] = s_out[i] * acc;
            }
        }
        if (t_out) for (int64_t k = 0; k < r; ++k) t_out[b * r + k] = t[k];
    }
    free(xp);
    free(t);
    return used;
}

/* ---- three-scale variant (the DBF / LittleBit format of Appendix F.4) ----
 *     W^ = Diag(s1) ( U Diag(s_mid) V^T ) Diag(s2),   s_mid in R^r
 * i.e. W^[i][j] = s_out[i] * ( sum_k U[i][k] * s_mid[k] * V[j][k] ) * s_in[j].
 * Separate functions: the two-scale code above stays exactly what its pins check. */

/* Tier A on chosen output rows, the definition written out */
void nqo_forward_dense_rows_mid(const uint32_t* U, const uint32_t* V, const double* s_out, const double* s_mid,
                                const double* s_in, int64_t d_out, int64_t d_in, int64_t r,
                                const double* x, int64_t batch,
                                const int64_t* rows, int64_t n_rows, double* y)
{
    int64_t wpr = words_per_row(r);
    (void)d_out;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < n_rows; ++q) {
        int64_t i = rows[q];
        double* Wrow = (double*)malloc(sizeof(double) * (size_t)d_in);
        for (int64_t j = 0; j < d_in; ++j) {
            double inner = 0.0;
            for (int64_t k = 0; k < r; ++k) inner += sign_at(U, wpr, i, k) * s_mid[k] * sign_at(V, wpr, j, k);
            Wrow[j] = s_out[i] * inner * s_in[j];
        }
        for (int64_t b = 0; b < batch; ++b) {
            double acc = 0.0;
            for (int64_t j = 0; j < d_in; ++j) acc += Wrow[j] * x[b * d_in + j];
            y[b * n_rows + q] = acc;
        }
        free(Wrow);
    }
}

/* Tier B: x' = s_in (.) x ; t = V^T x' ; t' = s_mid (.) t ; y = s_out (.) (U t').
 * `t_out` (may be NULL) receives t (before the rank-wise scale). */
int nqo_forward_factored_mid(const uint32_t* U, const uint32_t* V, const double* s_out, const double* s_mid,
                             const double* s_in, int64_t d_out, int64_t d_in, int64_t r,
                             const double* x, int64_t batch, double* y, double* t_out, int threads)
{
    int64_t wpr = words_per_row(r);
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    double* xp = (double*)malloc(sizeof(double) * (size_t)d_in);
    double* t = (double*)malloc(sizeof(double) * (size_t)r);
    double* tm = (double*)malloc(sizeof(double) * (size_t)r);
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t j = 0; j < d_in; ++j) xp[j] = s_in[j] * x[b * d_in + j];
#pragma omp parallel
        {
#ifdef _OPENMP
#pragma omp single
            used = omp_get_num_threads();
#endif
#pragma omp for schedule(static)
            for (int64_t k = 0; k < r; ++k) {
                double acc = 0.0;
                for (int64_t j = 0; j < d_in; ++j) acc += sign_at(V, wpr, j, k) * xp[j];
                t[k] = acc;
                tm[k] = s_mid[k] * acc;
            }
#pragma omp for schedule(static)
            for (int64_t i = 0; i < d_out; ++i) {
                double acc = 0.0;
                for (int64_t k = 0; k < r; ++k) acc += sign_at(U, wpr, i, k) * tm[k];
                y[b * d_out + i] = s_out[i] * acc;
            }
        }
        if (t_out) for (int64_t k = 0; k < r; ++k) t_out[b * r + k] = t[k];
    }
    free(xp);
    free(t);
    free(tm);
    return used;
}

/* Storage of the three-scale variant in bits: r(n+m) + 16(n+r+m)  (Appendix F.4) */
int64_t nqo_layer_bits_mid(int64_t d_out, int64_t d_in, int64_t r)
{
    return r * (d_out + d_in) + 16 * (d_out + r + d_in);
}

/* Storage of one factorized layer in bits: r(n+m) + 16(n+m)  (Appendix F.5) */
int64_t nqo_layer_bits(int64_t d_out, int64_t d_in, int64_t r)
{
    return r * (d_out + d_in) + 16 * (d_out + d_in);
}
