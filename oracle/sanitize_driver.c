/*
 * Runs the fp64 oracle (leet_oracle.c, compiled into this program) on one case read from a
 * file, for a build with -fsanitize=address,undefined: every buffer is heap-allocated at its
 * exact size, so an access outside q, k, v, gamma, a state or an output trips the sanitizer.
 * TEST INFRASTRUCTURE ONLY, like the oracle itself; tests/test_oracle_sanitized.py writes the
 * case, runs this program and compares what it writes with the pins.
 *
 * Case file (native endianness):
 *   7 longs   B, H, N, r, dv, has_state, nrows
 *   doubles   q[B*H*N*r], k[B*H*N*r], v[B*H*N*dv], gamma[H], state_in[B*H*r*dv] if has_state
 *   longs     rows[2*nrows]          (b*H+h, i) pairs for the row-sampled quadratic form (r = dv only)
 * Result file:
 *   doubles   quadratic[B*H*N*dv], recurrent[B*H*N*dv], state_out[B*H*r*dv],
 *             quadratic_rows[nrows*dv], decode_out[B*H*dv], decode_state[B*H*r*dv]
 *   (decode: one step of the recurrence on token 0 from state_in or zero)
 */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int leet_oracle_quadratic_rd(const double *, const double *, const double *, const double *, double *,
                             int, int, long, int, int);
int leet_oracle_quadratic_rows(const double *, const double *, const double *, const double *, const long *, long,
                               double *, int, int, long, int);
int leet_oracle_recurrent_rd(const double *, const double *, const double *, const double *, const double *,
                             double *, double *, int, int, long, int, int);
int leet_oracle_decode_step_rd(const double *, const double *, const double *, const double *, double *, double *,
                               int, int, int, int);

static double *read_doubles(FILE *f, size_t n)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    if (!p || fread(p, sizeof(double), n, f) != n) { fprintf(stderr, "short case file\n"); exit(3); }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s case.bin result.bin\n", argv[0]); return 2; }
    FILE *f = fopen(argv[1], "rb");
    if (!f) { perror("case"); return 2; }
    long hdr[7];
    if (fread(hdr, sizeof(long), 7, f) != 7) { fprintf(stderr, "short header\n"); return 3; }
    const long B = hdr[0], H = hdr[1], N = hdr[2], r = hdr[3], dv = hdr[4], has_state = hdr[5], nrows = hdr[6];
    const size_t nqk = (size_t)(B * H * N * r), nv = (size_t)(B * H * N * dv), ns = (size_t)(B * H * r * dv);
    double *q = read_doubles(f, nqk), *k = read_doubles(f, nqk), *v = read_doubles(f, nv);
    double *gamma = read_doubles(f, (size_t)H);
    double *state_in = has_state ? read_doubles(f, ns) : NULL;
    long *rows = (long *)malloc(sizeof(long) * (size_t)(2 * nrows ? 2 * nrows : 1));
    if (!rows || fread(rows, sizeof(long), (size_t)(2 * nrows), f) != (size_t)(2 * nrows)) return 3;
    fclose(f);

    double *quad = (double *)malloc(sizeof(double) * nv), *rec = (double *)malloc(sizeof(double) * nv);
    double *s_out = (double *)malloc(sizeof(double) * ns);
    double *qrows = (double *)malloc(sizeof(double) * (size_t)(nrows * dv ? nrows * dv : 1));
    double *dec_out = (double *)malloc(sizeof(double) * (size_t)(B * H * dv));
    double *dec_state = (double *)malloc(sizeof(double) * ns);
    if (!quad || !rec || !s_out || !qrows || !dec_out || !dec_state) return 4;

    int rc = leet_oracle_quadratic_rd(q, k, v, gamma, quad, (int)B, (int)H, N, (int)r, (int)dv);
    rc |= leet_oracle_recurrent_rd(q, k, v, gamma, state_in, rec, s_out, (int)B, (int)H, N, (int)r, (int)dv);
    if (nrows) rc |= leet_oracle_quadratic_rows(q, k, v, gamma, rows, nrows, qrows, (int)B, (int)H, N, (int)r);

    /* one decode step on token 0 of every (b, h): q, k, v of that token gathered into [B][H][.] */
    double *q0 = (double *)malloc(sizeof(double) * (size_t)(B * H * r)), *k0 = (double *)malloc(sizeof(double) * (size_t)(B * H * r));
    double *v0 = (double *)malloc(sizeof(double) * (size_t)(B * H * dv));
    if (!q0 || !k0 || !v0) return 4;
    for (long bh = 0; bh < B * H; ++bh) {
        memcpy(q0 + bh * r, q + (size_t)bh * N * r, sizeof(double) * (size_t)r);
        memcpy(k0 + bh * r, k + (size_t)bh * N * r, sizeof(double) * (size_t)r);
        memcpy(v0 + bh * dv, v + (size_t)bh * N * dv, sizeof(double) * (size_t)dv);
    }
    if (state_in) memcpy(dec_state, state_in, sizeof(double) * ns);
    else memset(dec_state, 0, sizeof(double) * ns);
    rc |= leet_oracle_decode_step_rd(q0, k0, v0, gamma, dec_state, dec_out, (int)B, (int)H, (int)r, (int)dv);
    if (rc) { fprintf(stderr, "an oracle call reported failure\n"); return 5; }

    f = fopen(argv[2], "wb");
    if (!f) { perror("result"); return 2; }
    fwrite(quad, sizeof(double), nv, f);
    fwrite(rec, sizeof(double), nv, f);
    fwrite(s_out, sizeof(double), ns, f);
    fwrite(qrows, sizeof(double), (size_t)(nrows * dv), f);
    fwrite(dec_out, sizeof(double), (size_t)(B * H * dv), f);
    fwrite(dec_state, sizeof(double), ns, f);
    fclose(f);
    free(q); free(k); free(v); free(gamma); free(state_in); free(rows); free(quad); free(rec); free(s_out);
    free(qrows); free(dec_out); free(dec_state); free(q0); free(k0); free(v0);
    return 0;
}
