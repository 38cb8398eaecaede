/* Driver that walks the C oracle over small ragged problems - every activation and row op, with
 * and without the optional vectors - for a build with -fsanitize=address,undefined
 * (tests/test_sanitizers_host.py).  Buffers are heap blocks of exactly the documented sizes, so
 * any index past an extent is an out-of-bounds report.  Prints a checksum. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int fge_oracle_chain(const double *X, const double *W, const double *b, const double *gamma, const double *beta,
                     long M, long N, long K, double alpha, double post_scale, int act, double lo, double hi,
                     int norm, double eps, double *out, double *aux);
int fge_oracle_gated_chain(const double *X, const double *W1, const double *W2, const double *b1, const double *b2,
                           const double *gamma, const double *beta, long M, long N, long K, double alpha,
                           double post_scale, int act, double lo, double hi, int norm, double eps, double *out,
                           double *aux, double *work);

static double *fill(long n, unsigned *s)
{
    double *p = malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    for (long i = 0; i < n; ++i) {
        *s = *s * 1664525u + 1013904223u;
        p[i] = ((double)(*s >> 8) / 16777216.0) * 2.0 - 1.0;
    }
    return p;
}

int main(void)
{
    const long shapes[][3] = {{1, 1, 1}, {3, 5, 7}, {17, 33, 9}, {8, 64, 16}};
    unsigned s = 12345u;
    double sum = 0.0;
    for (unsigned q = 0; q < sizeof(shapes) / sizeof(shapes[0]); ++q) {
        const long M = shapes[q][0], N = shapes[q][1], K = shapes[q][2];
        double *X = fill(M * K, &s), *W = fill(N * K, &s), *W2 = fill(N * K, &s), *b = fill(N, &s), *g = fill(N, &s),
               *be = fill(N, &s), *out = fill(M * N, &s), *aux = fill(M, &s), *work = fill(M * N, &s);
        for (int act = 0; act <= 5; ++act)
            for (int norm = 0; norm <= 4; ++norm)
                for (int opt = 0; opt < 2; ++opt) {
                    if (fge_oracle_chain(X, W, opt ? b : NULL, opt ? g : NULL, opt ? be : NULL, M, N, K, 0.5, 1.5, act,
                                         -0.5, 0.75, norm, 1e-5, out, aux))
                        return 2;
                    for (long i = 0; i < M * N; ++i) sum += out[i];
                    if (fge_oracle_gated_chain(X, W, W2, opt ? b : NULL, opt ? be : NULL, opt ? g : NULL, NULL, M, N, K,
                                               0.5, 1.5, act, -0.5, 0.75, norm, 1e-5, out, aux, work))
                        return 3;
                    for (long i = 0; i < M * N; ++i) sum += out[i];
                }
        if (fge_oracle_chain(X, W, b, g, be, M, N, K, 1.0, 1.0, 9, 0.0, 0.0, 0, 0.0, out, aux) == 0) return 4;   /* bad code is refused */
        free(X); free(W); free(W2); free(b); free(g); free(be); free(out); free(aux); free(work);
    }
    if (!isfinite(sum)) return 5;
    printf("checksum %.6f\n", sum);
    return 0;
}
