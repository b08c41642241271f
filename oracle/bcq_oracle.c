/*
 * CPU oracle for the binary-coding-quantized (BCQ) linear layer of AlphaTuning
 * (arXiv 2210.03858).  TEST INFRASTRUCTURE ONLY: the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the GPU library never does and
 * shares no code, header, table or helper with it.
 *
 * Everything is written as the plain definition: fp64 arithmetic, naive loops,
 * one sequential sum per output, no blocking, no fusion, no reordering.  OpenMP
 * only distributes independent outputs (rows or tokens) over cores; it never
 * splits a sum.
 *
 * Notation (paper -> here): h_out -> N rows of W, h_in -> K columns of W,
 * n_b -> T tokens, q bit planes.  Row-wise quantization (group size g = K,
 * Section 3 "BCQ Format", Eq. 1):
 *      W ~= sum_{i=1..q} diag(alpha_i) * B_i ,  B_i in {-1,+1}^{N x K}.
 * Shapes follow Table 1: alpha[q][N], planes[q][N][K].
 *
 * Readings of silent points (stated once here, used everywhere below):
 *   - sign(0) = +1, i.e. b = (r >= 0) ? +1 : -1, so -0.0 -> +1 as well.
 *   - Eq. ap3 (Appendix C) has lost its parentheses in print; it is read as
 *     alpha_i = (w - sum_{j<i} alpha_j b_j)^T b_i / n = mean_k |r_k|,
 *     which agrees with Eq. ap1 at i = 1.
 *   - alpha is an FP32 parameter (Section 4.2): the mean is formed in fp64,
 *     rounded once to fp32, and that rounded value is both stored and
 *     subtracted from the residual.
 *   - Eq. 4 is read as the true gradient of Eq. 2:
 *     dalpha_i[n] = s * sum_t dY[t,n] * (X B_i^T)[t,n]; the empirical 1/g_L of
 *     Eq. 4 is the caller's factor s.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Relative distance of v (> 0) to the nearer of the two fp32 rounding boundaries
 * that enclose the interval rounding to (float)v.  A tiny value means that a sum
 * formed in another order may round to a neighbouring fp32. */
static double round_margin(double v) {
    float a = (float)v;
    if (!(v > 0.0) || !isfinite(a)) return 1.0;
    double up = (double)nextafterf(a, INFINITY);
    double dn = (double)nextafterf(a, -INFINITY);
    double m1 = 0.5 * ((double)a + up), m2 = 0.5 * ((double)a + dn);
    double d1 = fabs(v - m1), d2 = fabs(v - m2);
    return (d1 < d2 ? d1 : d2) / v;
}

/* Greedy BCQ of one row (Appendix C, Eq. ap1 for i = 1, Eq. ap2 and ap3 for i > 1).
 * force[i] != 0 replaces the computed alpha_i by alpha_in[i] (used to re-run a row
 * with a given scale); force may be NULL. */
static void greedy_row(const float* w, int64_t K, int q, const float* alpha_in,
                       const uint8_t* force, float* alpha_out, int8_t* b_out /*[q][K] stride K*/,
                       int64_t plane_stride, double* margin_out, double* r) {
    for (int64_t k = 0; k < K; ++k) r[k] = (double)w[k];
    for (int i = 0; i < q; ++i) {
        int8_t* b = b_out + (int64_t)i * plane_stride;
        double S = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            b[k] = (r[k] >= 0.0) ? (int8_t)1 : (int8_t)-1; /* Eq. ap2: b_i = sign(residual) */
            S += fabs(r[k]);                               /* r^T b_i = sum |r_k|           */
        }
        double mean = S / (double)K;                       /* Eq. ap3: alpha_i = r^T b_i / n */
        float a = (float)mean;
        if (margin_out) margin_out[i] = round_margin(mean);
        if (force && force[i]) a = alpha_in[i];
        alpha_out[i] = a;
        for (int64_t k = 0; k < K; ++k) r[k] -= (double)a * (double)b[k];
    }
}

/* a1. W[N][K] fp32 -> alpha[q][N] fp32, planes[q][N][K] in {-1,+1}; margin[q][N] optional. */
void orc_quantize(const float* W, int64_t N, int64_t K, int q, float* alpha, int8_t* planes,
                  double* margin) {
#pragma omp parallel
    {
        double* r = (double*)malloc(sizeof(double) * (size_t)K);
        float a[64];
        double m[64];
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            greedy_row(W + n * K, K, q, NULL, NULL, a, planes + n * K, N * K, m, r);
            for (int i = 0; i < q; ++i) {
                alpha[(int64_t)i * N + n] = a[i];
                if (margin) margin[(int64_t)i * N + n] = m[i];
            }
        }
        free(r);
    }
}

/* One row with some alpha_i forced; planes_row[q][K]. */
void orc_quantize_row_forced(const float* w, int64_t K, int q, const float* alpha_in,
                             const uint8_t* force, float* alpha_out, int8_t* planes_row) {
    double* r = (double*)malloc(sizeof(double) * (size_t)K);
    greedy_row(w, K, q, alpha_in, force, alpha_out, planes_row, K, NULL, r);
    free(r);
}

/* a2. 32 signs -> one uint32 along K; bit j of word w is the sign of column 32w+j, 1 <=> +1.
 * The sign of the int8 decides (v >= 0 -> +1). */
void orc_pack(const int8_t* planes, int64_t N, int64_t K, int q, uint32_t* packed) {
    int64_t rows = (int64_t)q * N, Kw = K / 32;
#pragma omp parallel for schedule(static)
    for (int64_t rn = 0; rn < rows; ++rn)
        for (int64_t w = 0; w < Kw; ++w) {
            uint32_t word = 0;
            for (int j = 0; j < 32; ++j)
                if (planes[rn * K + 32 * w + j] >= 0) word |= (uint32_t)1 << j;
            packed[rn * Kw + w] = word;
        }
}

void orc_unpack(const uint32_t* packed, int64_t N, int64_t K, int q, int8_t* planes) {
    int64_t rows = (int64_t)q * N, Kw = K / 32;
#pragma omp parallel for schedule(static)
    for (int64_t rn = 0; rn < rows; ++rn)
        for (int64_t k = 0; k < K; ++k)
            planes[rn * K + k] = ((packed[rn * Kw + k / 32] >> (k % 32)) & 1u) ? (int8_t)1 : (int8_t)-1;
}

/* Eq. 1: What[n][k] = sum_i alpha_i[n] * B_i[n][k], fp64. */
static void dequant_row(const float* alpha, const int8_t* planes, int64_t N, int64_t K, int q,
                        int64_t n, double* wrow) {
    for (int64_t k = 0; k < K; ++k) {
        double s = 0.0;
        for (int i = 0; i < q; ++i)
            s += (double)alpha[(int64_t)i * N + n] * (double)planes[((int64_t)i * N + n) * K + k];
        wrow[k] = s;
    }
}

void orc_dequant(const float* alpha, const int8_t* planes, int64_t N, int64_t K, int q, double* What) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) dequant_row(alpha, planes, N, K, q, n, What + n * K);
}

/* a3. Eq. 2: y[t][n] = sum_k x[t][k] * What[n][k].  x holds the exact input values
 * (fp32, or bf16 values widened exactly to fp32); y stays fp64. */
void orc_fwd(const float* alpha, const int8_t* planes, const float* x, int64_t T, int64_t N,
             int64_t K, int q, double* y) {
#pragma omp parallel
    {
        double* wrow = (double*)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            dequant_row(alpha, planes, N, K, q, n, wrow);
            for (int64_t t = 0; t < T; ++t) {
                double s = 0.0;
                for (int64_t k = 0; k < K; ++k) s += (double)x[t * K + k] * wrow[k];
                y[t * N + n] = s;
            }
        }
        free(wrow);
    }
}

/* a3 on listed entries only: out[j] = y[tt[j]][nn[j]]. */
void orc_fwd_at(const float* alpha, const int8_t* planes, const float* x, int64_t T, int64_t N,
                int64_t K, int q, const int64_t* tt, const int64_t* nn, int64_t cnt, double* out) {
    (void)T;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < cnt; ++j) {
        int64_t t = tt[j], n = nn[j];
        double s = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double w = 0.0;
            for (int i = 0; i < q; ++i)
                w += (double)alpha[(int64_t)i * N + n] * (double)planes[((int64_t)i * N + n) * K + k];
            s += (double)x[t * K + k] * w;
        }
        out[j] = s;
    }
}

/* a4. Eq. 3: dx[t][k] = sum_n dy[t][n] * What[n][k]. */
void orc_bwd_input(const float* alpha, const int8_t* planes, const float* dy, int64_t T, int64_t N,
                   int64_t K, int q, double* dx) {
    double* What = (double*)malloc(sizeof(double) * (size_t)N * (size_t)K);
    orc_dequant(alpha, planes, N, K, q, What);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t k = 0; k < K; ++k) {
            double s = 0.0;
            for (int64_t n = 0; n < N; ++n) s += (double)dy[t * N + n] * What[n * K + k];
            dx[t * K + k] = s;
        }
    free(What);
}

void orc_bwd_input_at(const float* alpha, const int8_t* planes, const float* dy, int64_t T, int64_t N,
                      int64_t K, int q, const int64_t* tt, const int64_t* kk, int64_t cnt, double* out) {
    (void)T;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < cnt; ++j) {
        int64_t t = tt[j], k = kk[j];
        double s = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            double w = 0.0;
            for (int i = 0; i < q; ++i)
                w += (double)alpha[(int64_t)i * N + n] * (double)planes[((int64_t)i * N + n) * K + k];
            s += (double)dy[t * N + n] * w;
        }
        out[j] = s;
    }
}

/* a5. Eq. 4 read as the gradient of Eq. 2:
 * dalpha[i][n] = s * sum_t dy[t][n] * (sum_k B_i[n][k] x[t][k]),  i < q_train. */
void orc_bwd_alpha(const int8_t* planes, const float* x, const float* dy, int64_t T, int64_t N,
                   int64_t K, int q, int q_train, double grad_scale, double* dalpha) {
    (void)q;
#pragma omp parallel for schedule(static) collapse(2)
    for (int i = 0; i < q_train; ++i)
        for (int64_t n = 0; n < N; ++n) {
            const int8_t* b = planes + ((int64_t)i * N + n) * K;
            double g = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double p = 0.0;
                for (int64_t k = 0; k < K; ++k) p += (double)b[k] * (double)x[t * K + k];
                g += (double)dy[t * N + n] * p;
            }
            dalpha[(int64_t)i * N + n] = grad_scale * g;
        }
}

/* a5 on listed rows only: out[i][j] = dalpha[i][rows[j]]. */
void orc_bwd_alpha_rows(const int8_t* planes, const float* x, const float* dy, int64_t T, int64_t N,
                        int64_t K, int q, int q_train, double grad_scale, const int64_t* rows,
                        int64_t cnt, double* out) {
    (void)q;
#pragma omp parallel for schedule(static) collapse(2)
    for (int i = 0; i < q_train; ++i)
        for (int64_t j = 0; j < cnt; ++j) {
            int64_t n = rows[j];
            const int8_t* b = planes + ((int64_t)i * N + n) * K;
            double g = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double p = 0.0;
                for (int64_t k = 0; k < K; ++k) p += (double)b[k] * (double)x[t * K + k];
                g += (double)dy[t * N + n] * p;
            }
            out[(int64_t)i * cnt + j] = grad_scale * g;
        }
}

/* ------------------------------------------------------------------------------------------
 * Group-wise scales (Appendix C "group-wise quantization"; Table 1 rows with g < h_in;
 * Section 4.1, remark after Eq. 4): every row of W is cut into K/g consecutive vectors
 * of length g and each vector has its own q scales.  Shapes: alpha[q][N][K/g],
 * planes[q][N][K] as before.  g must divide K.  The functions below are the definitions
 * above with alpha_i[n] replaced by alpha_i[n][k / g]; g = K gives the row-wise case.
 * ------------------------------------------------------------------------------------------ */

/* Greedy BCQ of every length-g vector on its own (Eq. ap1-ap3 applied per vector). */
void orc_quantize_g(const float* W, int64_t N, int64_t K, int64_t g, int q, float* alpha,
                    int8_t* planes, double* margin) {
    int64_t G = K / g;
#pragma omp parallel
    {
        double* r = (double*)malloc(sizeof(double) * (size_t)g);
        float a[64];
        double m[64];
#pragma omp for schedule(static)
        for (int64_t v = 0; v < N * G; ++v) { /* v = n * G + group: vectors are consecutive in memory */
            greedy_row(W + v * g, g, q, NULL, NULL, a, planes + v * g, N * K, m, r);
            for (int i = 0; i < q; ++i) {
                alpha[(int64_t)i * N * G + v] = a[i];
                if (margin) margin[(int64_t)i * N * G + v] = m[i];
            }
        }
        free(r);
    }
}

/* Eq. 1 per vector: What[n][k] = sum_i alpha_i[n][k/g] * B_i[n][k]. */
static double what_g(const float* alpha, const int8_t* planes, int64_t N, int64_t K, int64_t g,
                     int q, int64_t n, int64_t k) {
    int64_t G = K / g;
    double s = 0.0;
    for (int i = 0; i < q; ++i)
        s += (double)alpha[((int64_t)i * N + n) * G + k / g] * (double)planes[((int64_t)i * N + n) * K + k];
    return s;
}

void orc_dequant_g(const float* alpha, const int8_t* planes, int64_t N, int64_t K, int64_t g, int q,
                   double* What) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) What[n * K + k] = what_g(alpha, planes, N, K, g, q, n, k);
}

/* Eq. 2 with group-wise scales, on listed entries: out[j] = y[tt[j]][nn[j]];
 * tt == NULL means all entries in row-major order (cnt = T * N). */
void orc_fwd_g_at(const float* alpha, const int8_t* planes, const float* x, int64_t T, int64_t N,
                  int64_t K, int64_t g, int q, const int64_t* tt, const int64_t* nn, int64_t cnt,
                  double* out) {
    (void)T;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < cnt; ++j) {
        int64_t t = tt ? tt[j] : j / N, n = tt ? nn[j] : j % N;
        double s = 0.0;
        for (int64_t k = 0; k < K; ++k) s += (double)x[t * K + k] * what_g(alpha, planes, N, K, g, q, n, k);
        out[j] = s;
    }
}

/* Eq. 3 with group-wise scales, on listed entries (tt == NULL: all, cnt = T * K). */
void orc_bwd_input_g_at(const float* alpha, const int8_t* planes, const float* dy, int64_t T,
                        int64_t N, int64_t K, int64_t g, int q, const int64_t* tt, const int64_t* kk,
                        int64_t cnt, double* out) {
    (void)T;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < cnt; ++j) {
        int64_t t = tt ? tt[j] : j / K, k = tt ? kk[j] : j % K;
        double s = 0.0;
        for (int64_t n = 0; n < N; ++n) s += (double)dy[t * N + n] * what_g(alpha, planes, N, K, g, q, n, k);
        out[j] = s;
    }
}

/* Eq. 4 as the gradient of Eq. 2 with group-wise scales, on listed rows (rows == NULL: all N):
 * out[i][j][c] = s * sum_t dy[t][n_j] * sum_{k in group c} B_i[n_j][k] x[t][k]. */
void orc_bwd_alpha_g_rows(const int8_t* planes, const float* x, const float* dy, int64_t T, int64_t N,
                          int64_t K, int64_t g, int q, int q_train, double grad_scale,
                          const int64_t* rows, int64_t cnt, double* out) {
    (void)q;
    int64_t G = K / g;
#pragma omp parallel for schedule(static) collapse(2)
    for (int i = 0; i < q_train; ++i)
        for (int64_t j = 0; j < cnt; ++j) {
            int64_t n = rows ? rows[j] : j;
            const int8_t* b = planes + ((int64_t)i * N + n) * K;
            for (int64_t c = 0; c < G; ++c) {
                double acc = 0.0;
                for (int64_t t = 0; t < T; ++t) {
                    double p = 0.0;
                    for (int64_t k = c * g; k < (c + 1) * g; ++k) p += (double)b[k] * (double)x[t * K + k];
                    acc += (double)dy[t * N + n] * p;
                }
                out[((int64_t)i * cnt + j) * G + c] = grad_scale * acc;
            }
        }
}

/* ------------------------------------------------------------------------------------------
 * Alternating quantizer (Appendix C, "Alternating Method", Eq. ap4).  Per vector w of length n:
 *   start from the greedy (alpha, B);
 *   repeat `iters` times (the paper uses 15):
 *     (1) alpha <- (B^T B)^{-1} B^T w                      least-squares refit, Eq. ap4
 *     (2) every element takes the sign pattern whose level sum_i +-alpha_i is nearest to w_k
 *         (the paper finds it by binary search over the sorted 2^q levels; here all 2^q levels
 *         are compared, which gives the same pattern)
 * Readings of silent points:
 *   - the iteration arithmetic is fp64; alpha is rounded to fp32 once, at the end;
 *   - the returned alpha is the one of the last refit (1) and the returned B the one of the last
 *     re-assignment (2); no extra refit follows;
 *   - if step (2) changes nothing the pair is a fixed point and the loop stops (more iterations
 *     would repeat it exactly);
 *   - if B^T B is singular (two planes equal or opposite, e.g. an all-zero vector) the loop stops
 *     before that refit and the current (alpha, B) stay; singular = a Cholesky pivot <= 1e-9 n;
 *   - ties between two levels go to the larger level, ties between equal levels to the larger
 *     pattern index c = sum_i [b_i = +1] 2^i (consistent with sign(0) = +1).
 * margin[0]: smallest relative gap between the best and the second-best level over all elements
 *            and iterations (exact ties at w_k = 0 between the mirror levels +-v are not counted:
 *            they are resolved by the rule above, whatever the rounding of alpha);
 * margin[1]: smallest round_margin() of the returned alpha_i.
 * ------------------------------------------------------------------------------------------ */
static void alternating_row(const float* w, int64_t n, int q, int iters, float* alpha_out,
                            int8_t* b_out, int64_t plane_stride, double* margin, double* err_trace,
                            int* iters_done, double* r, uint8_t* code) {
    double a[8], m_dec = 1.0;
    greedy_row(w, n, q, NULL, NULL, alpha_out, b_out, plane_stride, NULL, r);
    for (int i = 0; i < q; ++i) a[i] = (double)alpha_out[i];
    for (int64_t k = 0; k < n; ++k) {
        uint8_t c = 0;
        for (int i = 0; i < q; ++i)
            if (b_out[(int64_t)i * plane_stride + k] > 0) c |= (uint8_t)(1u << i);
        code[k] = c;
    }
    const int levels = 1 << q;
    int done = 0;
    for (int it = 0; it < iters; ++it) {
        if (err_trace) { /* squared error before this iteration */
            double e = 0.0;
            for (int64_t k = 0; k < n; ++k) {
                double v = 0.0;
                for (int i = 0; i < q; ++i) v += ((code[k] >> i) & 1) ? a[i] : -a[i];
                e += ((double)w[k] - v) * ((double)w[k] - v);
            }
            err_trace[2 * it] = e;
        }
        /* (1) Eq. ap4: Gram matrix and right-hand side, then Cholesky solve */
        double G[8][8], rhs[8], L[8][8], y[8];
        for (int i = 0; i < q; ++i) {
            for (int j = 0; j <= i; ++j) {
                double s = 0.0;
                for (int64_t k = 0; k < n; ++k)
                    s += (((code[k] >> i) & 1) == ((code[k] >> j) & 1)) ? 1.0 : -1.0;
                G[i][j] = s;
            }
            double s = 0.0;
            for (int64_t k = 0; k < n; ++k) s += ((code[k] >> i) & 1) ? (double)w[k] : -(double)w[k];
            rhs[i] = s;
        }
        int singular = 0;
        for (int j = 0; j < q && !singular; ++j) {
            double d = G[j][j];
            for (int p = 0; p < j; ++p) d -= L[j][p] * L[j][p];
            if (!(d > 1e-9 * (double)n)) { singular = 1; break; }
            L[j][j] = sqrt(d);
            for (int i = j + 1; i < q; ++i) {
                double s = G[i][j];
                for (int p = 0; p < j; ++p) s -= L[i][p] * L[j][p];
                L[i][j] = s / L[j][j];
            }
        }
        if (singular) break;
        for (int i = 0; i < q; ++i) {
            double s = rhs[i];
            for (int p = 0; p < i; ++p) s -= L[i][p] * y[p];
            y[i] = s / L[i][i];
        }
        for (int i = q - 1; i >= 0; --i) {
            double s = y[i];
            for (int p = i + 1; p < q; ++p) s -= L[p][i] * a[p];
            a[i] = s / L[i][i];
        }
        if (err_trace) { /* squared error after the refit */
            double e = 0.0;
            for (int64_t k = 0; k < n; ++k) {
                double v = 0.0;
                for (int i = 0; i < q; ++i) v += ((code[k] >> i) & 1) ? a[i] : -a[i];
                e += ((double)w[k] - v) * ((double)w[k] - v);
            }
            err_trace[2 * it + 1] = e;
        }
        /* (2) nearest level for every element */
        double lv[256], scale = 0.0;
        for (int c = 0; c < levels; ++c) {
            double v = 0.0;
            for (int i = 0; i < q; ++i) v += ((c >> i) & 1) ? a[i] : -a[i];
            lv[c] = v;
        }
        for (int i = 0; i < q; ++i) scale += fabs(a[i]);
        int changed = 0;
        for (int64_t k = 0; k < n; ++k) {
            double x = (double)w[k];
            int best = levels - 1;
            double bd = fabs(x - lv[best]);
            for (int c = levels - 2; c >= 0; --c) {
                double d = fabs(x - lv[c]);
                if (d < bd || (d == bd && lv[c] > lv[best])) { best = c; bd = d; }
            }
            double second = INFINITY;
            for (int c = 0; c < levels; ++c)
                if (c != best) { double d = fabs(x - lv[c]); if (d < second) second = d; }
            double gap = second - bd;
            int mirror_tie = (gap == 0.0 && x == 0.0);
            if (!mirror_tie && scale > 0.0 && gap / scale < m_dec) m_dec = gap / scale;
            if ((uint8_t)best != code[k]) { code[k] = (uint8_t)best; changed = 1; }
        }
        done = it + 1;
        if (!changed) break;
    }
    double m_round = 1.0;
    for (int i = 0; i < q; ++i) {
        alpha_out[i] = (float)a[i];
        double rm = round_margin(fabs(a[i]));
        if (rm < m_round) m_round = rm;
        for (int64_t k = 0; k < n; ++k)
            b_out[(int64_t)i * plane_stride + k] = ((code[k] >> i) & 1) ? (int8_t)1 : (int8_t)-1;
    }
    if (margin) { margin[0] = m_dec; margin[1] = m_round; }
    if (iters_done) *iters_done = done;
}

/* W[N][K] -> alpha[q][N][K/g], planes[q][N][K]; margin[N*K/g][2], iters_done[N*K/g] optional. */
void orc_quantize_alternating(const float* W, int64_t N, int64_t K, int64_t g, int q, int iters,
                              float* alpha, int8_t* planes, double* margin, int* iters_done) {
    int64_t V = N * (K / g);
#pragma omp parallel
    {
        double* r = (double*)malloc(sizeof(double) * (size_t)g);
        uint8_t* code = (uint8_t*)malloc((size_t)g);
        float a[8];
#pragma omp for schedule(static)
        for (int64_t v = 0; v < V; ++v) {
            alternating_row(W + v * g, g, q, iters, a, planes + v * g, N * K, margin ? margin + 2 * v : NULL,
                            NULL, iters_done ? iters_done + v : NULL, r, code);
            for (int i = 0; i < q; ++i) alpha[(int64_t)i * V + v] = a[i];
        }
        free(r);
        free(code);
    }
}

/* One vector with the squared error before every iteration and after every refit:
 * err_trace[2 it], err_trace[2 it + 1], it < iters (unused entries stay as passed in). */
void orc_alternating_row_trace(const float* w, int64_t n, int q, int iters, float* alpha_out,
                               int8_t* planes_row, double* err_trace, int* iters_done) {
    double* r = (double*)malloc(sizeof(double) * (size_t)n);
    uint8_t* code = (uint8_t*)malloc((size_t)n);
    alternating_row(w, n, q, iters, alpha_out, planes_row, n, NULL, err_trace, iters_done, r, code);
    free(r);
    free(code);
}
