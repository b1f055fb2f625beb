/*
 * FreqKV reference oracle (TEST INFRASTRUCTURE ONLY - never on the product path).
 *
 * Plain fp64, single-threaded, direct O(n^2) sums of the paper's definitions:
 *   - orthonormal DCT-II along the token axis            (Appendix A, DCT-II definition; Sec. 3.3 Eq. 2)
 *   - keep the lowest Lc coefficients                    (Sec. 3.3, "retaining ratio")
 *   - Lc-point inverse DCT of the kept coefficients      (Appendix A, inverse definition, with N := Lc)
 *   - rescale by sqrt(Lc/n)                              (Sec. 3.3 Eq. 3, rescaling ablation appendix)
 *
 * No FFT, no matrix library, no blocking, no reordering.  The cosine argument
 * pi*t*(2j+1)/(2N) is reduced in 64-bit integers: q = t*(2j+1) mod 4N, and the
 * cosine comes from a table cos(pi*q/(2N)), q in [0,4N), filled in fp64.
 *
 * Shares no code, table or constant with the HIP library.
 *
 * Parity pins: see tests/test_oracle_pins.py (round trip at ratio 1, constant
 * sequence, Parseval, explicit-matrix brute force, pure-cosine closed form,
 * Dirichlet-kernel closed form, scipy special case).  Numeric values of
 * compressed K/V for real text: parity unpinned (the paper prints none).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef M_PI
#define M_PI 3.14159265358979323846
#endif

/* cos(pi*q/(2N)) for q = 0 .. 4N-1 */
static double *cos_table(int N)
{
    int64_t len = 4 * (int64_t)N;
    double *tab = (double *)malloc((size_t)len * sizeof(double));
    if (!tab) return NULL;
    for (int64_t q = 0; q < len; ++q)
        tab[q] = cos(M_PI * (double)q / (2.0 * (double)N));
    return tab;
}

/*
 * Orthonormal DCT-II (Appendix A, first equation).
 *   x : [n][d] row-major (rows = tokens, columns = channels)
 *   z : [n_out][d], coefficients t = 0 .. n_out-1  (n_out <= n)
 *   z[t][c] = alpha_t * sum_j x[j][c] * cos(pi t (2j+1) / (2n)),
 *   alpha_0 = sqrt(1/n), alpha_t = sqrt(2/n) otherwise.
 * Returns 0, or -1 on allocation failure / bad sizes.
 */
int freqkv_oracle_dct2(const double *x, int n, int d, int n_out, double *z)
{
    if (n <= 0 || d <= 0 || n_out < 0 || n_out > n) return -1;
    double *tab = cos_table(n);
    if (!tab) return -1;
    const int64_t period = 4 * (int64_t)n;
    for (int t = 0; t < n_out; ++t) {
        double *zt = z + (size_t)t * d;
        for (int c = 0; c < d; ++c) zt[c] = 0.0;
        for (int j = 0; j < n; ++j) {
            int64_t q = ((int64_t)t * (2 * (int64_t)j + 1)) % period;
            double w = tab[q];
            const double *xj = x + (size_t)j * d;
            for (int c = 0; c < d; ++c) zt[c] += xj[c] * w;
        }
        double alpha = (t == 0) ? sqrt(1.0 / (double)n) : sqrt(2.0 / (double)n);
        for (int c = 0; c < d; ++c) zt[c] *= alpha;
    }
    free(tab);
    return 0;
}

/*
 * Inverse of the orthonormal DCT-II (Appendix A, second equation), L-point.
 *   z : [L][d] coefficients, y : [L][d] samples
 *   y[m][c] = sum_t alpha_t * z[t][c] * cos(pi t (2m+1) / (2L)),  alpha as above with N = L.
 */
int freqkv_oracle_idct2(const double *z, int L, int d, double *y)
{
    if (L <= 0 || d <= 0) return -1;
    double *tab = cos_table(L);
    if (!tab) return -1;
    const int64_t period = 4 * (int64_t)L;
    const double a0 = sqrt(1.0 / (double)L), a1 = sqrt(2.0 / (double)L);
    for (int m = 0; m < L; ++m) {
        double *ym = y + (size_t)m * d;
        for (int c = 0; c < d; ++c) ym[c] = 0.0;
        for (int t = 0; t < L; ++t) {
            int64_t q = ((int64_t)t * (2 * (int64_t)m + 1)) % period;
            double w = tab[q] * (t == 0 ? a0 : a1);
            const double *zt = z + (size_t)t * d;
            for (int c = 0; c < d; ++c) ym[c] += zt[c] * w;
        }
    }
    free(tab);
    return 0;
}

/*
 * One compression of one span (Sec. 3.3 Eq. 2 and Eq. 3):
 *   x : [n][d]  ->  y : [Lc][d],
 *   y = scale * IDCT_Lc( DCT_n(x)[0:Lc] ),  scale = sqrt(Lc/n) when rescale != 0, else 1.
 * Optionally returns the kept coefficients in z_keep ([Lc][d], may be NULL).
 */
int freqkv_oracle_compress_span(const double *x, int n, int Lc, int d, int rescale,
                                double *y, double *z_keep)
{
    if (n <= 0 || Lc <= 0 || Lc > n || d <= 0) return -1;
    double *z = (double *)malloc((size_t)Lc * d * sizeof(double));
    if (!z) return -1;
    int rc = freqkv_oracle_dct2(x, n, d, Lc, z);      /* coefficients t >= Lc are discarded */
    if (rc == 0) rc = freqkv_oracle_idct2(z, Lc, d, y);
    if (rc == 0 && rescale) {
        double s = sqrt((double)Lc / (double)n);
        for (size_t i = 0; i < (size_t)Lc * d; ++i) y[i] *= s;
    }
    if (rc == 0 && z_keep) memcpy(z_keep, z, (size_t)Lc * d * sizeof(double));
    free(z);
    return rc;
}

/*
 * One trigger on one head-tensor of the cache (Sec. 3.4; Fig. 2b):
 *   cache : [cur_len][d] rows = tokens.  Rows [0,S) stay, rows [S,W) are the
 *   span that is compressed to Lc rows, rows [W,cur_len) (a recent tail) are
 *   kept bit-for-bit behind the compressed rows.
 *   out   : [S + Lc + (cur_len - W)][d]
 */
int freqkv_oracle_compress_head(const double *cache, int cur_len, int d, int W, int S, int Lc,
                                int rescale, double *out)
{
    int n = W - S;
    if (S < 0 || n <= 0 || cur_len < W || Lc <= 0 || Lc > n) return -1;
    memcpy(out, cache, (size_t)S * d * sizeof(double));
    int rc = freqkv_oracle_compress_span(cache + (size_t)S * d, n, Lc, d, rescale,
                                         out + (size_t)S * d, NULL);
    if (rc) return rc;
    memcpy(out + (size_t)(S + Lc) * d, cache + (size_t)W * d,
           (size_t)(cur_len - W) * d * sizeof(double));
    return 0;
}
