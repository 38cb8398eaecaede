/*
 * Float64 CPU oracle for the fused operator chain
 *
 *     out = rowop_N( act( post_scale * (alpha * X.W^T + b) ) )
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is compared against; it
 * is never part of the product path and shares no code with it.  Only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may call it.
 *
 * Everything is the plain mathematical definition evaluated in IEEE double, one step after
 * the other, with no blocking, fusion or reordering:
 *
 *   - the chain itself (a dense contraction, a bias, an elementwise activation, a row-wise
 *     normalisation) is the "fused operator" pattern of the paper's benchmark section
 *     (Section 3.6: matmul, activations, Softmax, LayerNorm, RMSNorm and fused variants) and of
 *     its performance discussion (Section 4.3: eager mode composes LayerNorm from mean,
 *     variance and normalisation steps);
 *   - RMSNorm follows the paper's Unified-Sketch example (Fig. 2): sum of squares over the
 *     reduced axis, divide by its length, add eps, square root, divide the input by it;
 *   - the reference is "the framework-level implementation" (Section 3.1), so GELU without
 *     suffix is the erf form and LayerNorm uses the biased variance with eps inside the root.
 *
 * Pins (tests/test_oracle_pins.py): brute-force loops in another order, closed forms and
 * invariants of each step, library routines on special cases.  The paper prints no worked
 * numeric example, so the whole chain at workload scale is pinned only through its steps.
 *
 * Layout: X is M x K row-major, W is N x K row-major (both K-contiguous), b/gamma/beta have
 * length N (NULL = absent), out is M x N row-major, aux has length M (row logsumexp) or NULL.
 */
#include <math.h>
#include <stddef.h>

enum { ACT_NONE = 0, ACT_RELU, ACT_GELU_TANH, ACT_GELU_ERF, ACT_SILU, ACT_CLAMP };
enum { NORM_NONE = 0, NORM_SOFTMAX, NORM_LAYERNORM, NORM_RMSNORM, NORM_LOGSUMEXP };

/* Step 1: G[i][j] = sum_k X[i][k] * W[j][k]   (k ascending). */
void fge_oracle_gemm(const double *X, const double *W, long M, long N, long K, double *G)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i)
        for (long j = 0; j < N; ++j) {
            double acc = 0.0;
            for (long k = 0; k < K; ++k)
                acc += X[i * K + k] * W[j * K + k];
            G[i * N + j] = acc;
        }
}

/* Step 2: Y = post_scale * (alpha * G + b[j]).  alpha multiplies the product only; post_scale
 * multiplies the biased sum. */
void fge_oracle_scale_bias(double *G, const double *b, long M, long N, double alpha, double post_scale)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i)
        for (long j = 0; j < N; ++j)
            G[i * N + j] = post_scale * (alpha * G[i * N + j] + (b ? b[j] : 0.0));
}

/* Step 3: elementwise activation. */
double fge_oracle_act1(double y, int act, double lo, double hi)
{
    switch (act) {
    case ACT_NONE:      return y;
    case ACT_RELU:      return y > 0.0 ? y : 0.0;
    case ACT_GELU_TANH: return 0.5 * y * (1.0 + tanh(sqrt(2.0 / M_PI) * (y + 0.044715 * y * y * y)));
    case ACT_GELU_ERF:  return 0.5 * y * (1.0 + erf(y / sqrt(2.0)));
    case ACT_SILU:      return y / (1.0 + exp(-y));
    case ACT_CLAMP:     return y < lo ? lo : (y > hi ? hi : y);
    default:            return NAN;
    }
}

void fge_oracle_act(double *Y, long count, int act, double lo, double hi)
{
#pragma omp parallel for schedule(static)
    for (long t = 0; t < count; ++t)
        Y[t] = fge_oracle_act1(Y[t], act, lo, hi);
}

/* Step 4: row-wise operation over the N columns of each row, in place.
 *   softmax   : p_j = exp(a_j - m) / sum_l exp(a_l - m),  m = max_j a_j
 *   layernorm : mu = sum a / N;  var = sum (a - mu)^2 / N (biased, two passes);
 *               out_j = (a_j - mu) / sqrt(var + eps) * gamma_j + beta_j
 *   rmsnorm   : out_j = a_j / sqrt(sum a^2 / N + eps) * gamma_j      (Fig. 2 of the paper)
 *   logsumexp : out = a unchanged;  aux_i = m + ln sum_j exp(a_j - m)
 */
void fge_oracle_rowop(double *A, long M, long N, int norm, double eps,
                      const double *gamma, const double *beta, double *aux)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        double *a = A + i * N;
        if (norm == NORM_SOFTMAX || norm == NORM_LOGSUMEXP) {
            double m = a[0];
            for (long j = 1; j < N; ++j)
                if (a[j] > m) m = a[j];
            double s = 0.0;
            for (long j = 0; j < N; ++j)
                s += exp(a[j] - m);
            if (norm == NORM_SOFTMAX) {
                for (long j = 0; j < N; ++j)
                    a[j] = exp(a[j] - m) / s;
            } else if (aux) {
                aux[i] = m + log(s);
            }
        } else if (norm == NORM_LAYERNORM) {
            double mu = 0.0;
            for (long j = 0; j < N; ++j) mu += a[j];
            mu /= (double)N;
            double var = 0.0;
            for (long j = 0; j < N; ++j) var += (a[j] - mu) * (a[j] - mu);
            var /= (double)N;
            double sd = sqrt(var + eps);
            for (long j = 0; j < N; ++j)
                a[j] = (a[j] - mu) / sd * (gamma ? gamma[j] : 1.0) + (beta ? beta[j] : 0.0);
        } else if (norm == NORM_RMSNORM) {
            double ss = 0.0;
            for (long j = 0; j < N; ++j) ss += a[j] * a[j];
            double rms = sqrt(ss / (double)N + eps);
            for (long j = 0; j < N; ++j)
                a[j] = a[j] / rms * (gamma ? gamma[j] : 1.0);
        }
    }
}

/* The whole chain: steps 1-4 in order.  Returns 0, or -1 on an unknown enum. */
int fge_oracle_chain(const double *X, const double *W, const double *b,
                     const double *gamma, const double *beta,
                     long M, long N, long K, double alpha, double post_scale,
                     int act, double clamp_lo, double clamp_hi, int norm, double eps,
                     double *out, double *aux)
{
    if (act < ACT_NONE || act > ACT_CLAMP || norm < NORM_NONE || norm > NORM_LOGSUMEXP)
        return -1;
    fge_oracle_gemm(X, W, M, N, K, out);
    fge_oracle_scale_bias(out, b, M, N, alpha, post_scale);
    fge_oracle_act(out, M * N, act, clamp_lo, clamp_hi);
    fge_oracle_rowop(out, M, N, norm, eps, gamma, beta, aux);
    return 0;
}

#ifdef _OPENMP
#include <omp.h>
int fge_oracle_threads(void) { return omp_get_max_threads(); }
#else
int fge_oracle_threads(void) { return 1; }
#endif

/* Gated variant (the "SiLU-and-Mul" / "GELU-and-Mul" fused operators the paper's benchmark
 * section lists among the fused operations, Section 3.6): two products sharing X,
 *     G = post_scale * (alpha * X.W1^T + b1),   U = post_scale * (alpha * X.W2^T + b2),
 *     A = act(G) * U   elementwise,             out = rowop_N(A).
 * Gate step: A[t] = act(G[t]) * U[t], written into G. */
void fge_oracle_gate(double *G, const double *U, long count, int act, double lo, double hi)
{
#pragma omp parallel for schedule(static)
    for (long t = 0; t < count; ++t)
        G[t] = fge_oracle_act1(G[t], act, lo, hi) * U[t];
}

/* The gated chain, step after step.  `work` is M x N scratch for U.  Returns 0, or -1 on an
 * unknown enum. */
int fge_oracle_gated_chain(const double *X, const double *W1, const double *W2,
                           const double *b1, const double *b2,
                           const double *gamma, const double *beta,
                           long M, long N, long K, double alpha, double post_scale,
                           int act, double clamp_lo, double clamp_hi, int norm, double eps,
                           double *out, double *aux, double *work)
{
    if (act < ACT_NONE || act > ACT_CLAMP || norm < NORM_NONE || norm > NORM_LOGSUMEXP)
        return -1;
    fge_oracle_gemm(X, W1, M, N, K, out);
    fge_oracle_scale_bias(out, b1, M, N, alpha, post_scale);
    fge_oracle_gemm(X, W2, M, N, K, work);
    fge_oracle_scale_bias(work, b2, M, N, alpha, post_scale);
    fge_oracle_gate(out, work, M * N, act, clamp_lo, clamp_hi);
    fge_oracle_rowop(out, M, N, norm, eps, gamma, beta, aux);
    return 0;
}
