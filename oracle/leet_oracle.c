/*
 * fp64 CPU oracle for exponentially decaying causal linear attention.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call this file;
 * it exists so that the HIP kernels can be checked against a slow, plain,
 * obviously correct statement of what the paper's operator computes.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * Operator (Section 2.2, Eq. "BCMV" with B = Q, C = K):
 *     O = ((Q K^T) .* M) V,   M[i][j] = gamma^(i-j) if i >= j else 0.
 * No softmax, no row normalisation, no 1/sqrt(d) (Section 2.1 drops it).
 * gamma is one value per head; gamma = 1 is plain causal linear attention.
 * 0^0 is taken as 1, so the diagonal weight is always 1.
 *
 * Two independent forms are given:
 *   form 1  leet_oracle_quadratic*  the definition written out (the paper's
 *           "vanilla" method), O(N^2 d);
 *   form 2  leet_oracle_recurrent / leet_oracle_decode_step  the row-based
 *           algorithm (Appendix B.1, Alg. 1) with the discount of the
 *           lambda-cumsum recurrence O_i = V_i + lambda O_{i-1}
 *           (Appendix C.1):   U <- gamma U + k_i^T v_i ;  o_i = q_i U.
 *           The state is updated before the output is taken, so token i
 *           sees itself with weight gamma^0 = 1, as M[i][i] = 1 demands.
 *
 * Layout everywhere: q, k, v, out are [B][H][N][d] row-major doubles; gamma
 * is [H]; a state is [B][H][d][d] with rows = key index, cols = value index.
 *
 * The operator is defined for B, C in R^(N x r) and V in R^(N x d) with a rank r
 * that need not equal d (Section 2.2); the *_rd entry points take q, k as
 * [B][H][N][r] and v, out as [B][H][N][dv], state [B][H][r][dv].  The entry
 * points with a single d are the same code with r = dv = d.
 * All parity pins live in tests/ (not here).
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

/* gamma^n for integer n >= 0, by the library pow, with 0^0 = 1. */
static double decay_weight(double gamma, long n)
{
    if (n == 0) return 1.0;
    return pow(gamma, (double)n);
}

/* Form 1 for one output row i of one (b,h): o_i = sum_{j<=i} gamma^(i-j) (q_i.k_j) v_j. */
static void quadratic_row(const double *q, const double *k, const double *v,
                          double gamma, long i, int r, int dv, double *o)
{
    for (int c = 0; c < dv; ++c) o[c] = 0.0;
    for (long j = 0; j <= i; ++j) {
        double a = 0.0;
        for (int e = 0; e < r; ++e) a += q[i * r + e] * k[j * r + e];
        a *= decay_weight(gamma, i - j);
        for (int c = 0; c < dv; ++c) o[c] += a * v[j * dv + c];
    }
}

/* Form 1, whole tensors. */
int leet_oracle_quadratic_rd(const double *q, const double *k, const double *v,
                             const double *gamma, double *out,
                             int B, int H, long N, int r, int dv)
{
    if (!gamma || B <= 0 || H <= 0 || N < 0 || r <= 0 || dv <= 0) return 1;
    if (N == 0) return 0; /* no rows */
    if (!q || !k || !v || !out) return 1;
    long BH = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (long bh = 0; bh < BH; ++bh) {
        for (long i = 0; i < N; ++i) {
            size_t qk = (size_t)bh * N * r, vo = (size_t)bh * N * dv;
            quadratic_row(q + qk, k + qk, v + vo, gamma[bh % H], i, r, dv,
                          out + vo + (size_t)i * dv);
        }
    }
    return 0;
}

int leet_oracle_quadratic(const double *q, const double *k, const double *v,
                          const double *gamma, double *out,
                          int B, int H, long N, int d)
{
    return leet_oracle_quadratic_rd(q, k, v, gamma, out, B, H, N, d, d);
}

/* Form 1 on selected rows only: rows[r] = {b*H+h, i}; out_rows is [nrows][d]. */
int leet_oracle_quadratic_rows(const double *q, const double *k, const double *v,
                               const double *gamma, const long *rows, long nrows,
                               double *out_rows, int B, int H, long N, int d)
{
    if (!q || !k || !v || !gamma || !rows || !out_rows || B <= 0 || H <= 0 || N <= 0 || d <= 0) return 1;
    for (long r = 0; r < nrows; ++r) {
        long bh = rows[2 * r], i = rows[2 * r + 1];
        if (bh < 0 || bh >= (long)B * H || i < 0 || i >= N) return 1;
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < nrows; ++r) {
        long bh = rows[2 * r], i = rows[2 * r + 1];
        size_t base = (size_t)bh * N * d;
        quadratic_row(q + base, k + base, v + base, gamma[bh % H], i, d, d,
                      out_rows + (size_t)r * d);
    }
    return 0;
}

/* One token of form 2 on one (b,h) state U[r][dv]. */
static void recurrent_token(double *U, const double *qi, const double *ki,
                            const double *vi, double gamma, int r, int dv, double *oi)
{
    for (int e = 0; e < r; ++e)
        for (int c = 0; c < dv; ++c)
            U[(size_t)e * dv + c] = gamma * U[(size_t)e * dv + c] + ki[e] * vi[c];
    for (int c = 0; c < dv; ++c) oi[c] = 0.0;
    for (int e = 0; e < r; ++e)
        for (int c = 0; c < dv; ++c)
            oi[c] += qi[e] * U[(size_t)e * dv + c];
}

/*
 * Form 2, whole tensors.  state_in may be NULL (zero state); state_out may be
 * NULL.  state_out receives the state after the last token.
 */
int leet_oracle_recurrent_rd(const double *q, const double *k, const double *v,
                             const double *gamma, const double *state_in,
                             double *out, double *state_out,
                             int B, int H, long N, int r, int dv)
{
    /* N = 0: the loop over tokens does not run and the state leaves as it entered */
    if (!gamma || B <= 0 || H <= 0 || N < 0 || r <= 0 || dv <= 0) return 1;
    if (N > 0 && (!q || !k || !v || !out)) return 1;
    long BH = (long)B * H;
    size_t ssz = (size_t)r * dv;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        double *U = (double *)malloc(sizeof(double) * ssz);
        if (!U) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        if (state_in) memcpy(U, state_in + (size_t)bh * ssz, sizeof(double) * ssz);
        else memset(U, 0, sizeof(double) * ssz);
        size_t qk = (size_t)bh * N * r, vo = (size_t)bh * N * dv;
        for (long i = 0; i < N; ++i)
            recurrent_token(U, q + qk + i * r, k + qk + i * r, v + vo + i * dv,
                            gamma[bh % H], r, dv, out + vo + i * dv);
        if (state_out) memcpy(state_out + (size_t)bh * ssz, U, sizeof(double) * ssz);
        free(U);
    }
    return failed;
}

int leet_oracle_recurrent(const double *q, const double *k, const double *v,
                          const double *gamma, const double *state_in,
                          double *out, double *state_out,
                          int B, int H, long N, int d)
{
    return leet_oracle_recurrent_rd(q, k, v, gamma, state_in, out, state_out, B, H, N, d, d);
}

/*
 * One decode step: q, k, v, out are [B][H][d]; state is updated in place.
 * This is form 2 applied to a single token per (b,h).
 */
int leet_oracle_decode_step_rd(const double *q, const double *k, const double *v,
                               const double *gamma, double *state_inout, double *out,
                               int B, int H, int r, int dv)
{
    if (!q || !k || !v || !gamma || !state_inout || !out || B <= 0 || H <= 0 || r <= 0 || dv <= 0) return 1;
    long BH = (long)B * H;
#pragma omp parallel for schedule(static)
    for (long bh = 0; bh < BH; ++bh)
        recurrent_token(state_inout + (size_t)bh * r * dv, q + bh * r, k + bh * r,
                        v + bh * dv, gamma[bh % H], r, dv, out + bh * dv);
    return 0;
}

int leet_oracle_decode_step(const double *q, const double *k, const double *v,
                            const double *gamma, double *state_inout, double *out,
                            int B, int H, int d)
{
    return leet_oracle_decode_step_rd(q, k, v, gamma, state_inout, out, B, H, d, d);
}

int leet_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
