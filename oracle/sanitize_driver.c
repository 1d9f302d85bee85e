/*
 * Driver for a sanitizer run of the CPU oracle (test infrastructure, like the oracle itself).
 * Built together with sb_oracle.c under -fsanitize=address,undefined by
 * tests/test_oracle_sanitizers.py and run as a stand-alone executable: every buffer is
 * allocated with exactly the size the oracle's interface states, so an access outside it, a
 * read of uninitialised heap that reaches a branch in the checks below, or undefined
 * arithmetic aborts the run.  Exit status 0 = clean.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int sb_oracle_num_threads(void);
int sb_oracle_weights(const double *q, const double *k, int T, int d,
                      double *A_out, double *beta_out, double *rem_out);
int sb_oracle_fwd(const double *q, const double *k, const double *v, const double *r,
                  double *o, double *rem, int B, int H, int T, int d, int row_begin, int row_end);
int sb_oracle_bwd(const double *q, const double *k, const double *v, const double *r,
                  const double *dout, double *dq, double *dk, double *dv, double *dr,
                  int B, int H, int T, int d);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void)
{   /* xorshift, uniform in (-2, 2): enough to exercise both signs of the logits */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return ((double)(state >> 11) / 9007199254740992.0) * 4.0 - 2.0;
}
static double *filled(size_t n)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    if (!p) exit(2);
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
static int finite_all(const double *p, size_t n)
{
    for (size_t i = 0; i < n; ++i) if (!isfinite(p[i])) return 0;
    return 1;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int one_shape(int B, int H, int T, int d, int with_r)
{
    const size_t n = (size_t)B * H * T * d, nr = (size_t)H * d, nm = (size_t)B * H * T;
    double *q = filled(n), *k = filled(n), *v = filled(n), *g = filled(n);
    double *r = with_r ? filled(nr) : NULL;
    double *o = filled(n), *rem = filled(nm);
    /* full rows, then a row range into a second buffer, then without rem */
    CHECK(sb_oracle_fwd(q, k, v, r, o, rem, B, H, T, d, 0, T) == 0);
    CHECK(finite_all(o, n) && finite_all(rem, nm));
    if (!with_r) for (size_t c = 0; c < (size_t)d; ++c) CHECK(o[c] == 0.0);   /* first token: empty sum */
    double *o2 = filled(n);
    const int r0 = T / 3, r1 = T - T / 4;
    CHECK(sb_oracle_fwd(q, k, v, r, o2, NULL, B, H, T, d, r0, r1) == 0);
    for (int j = r0; j < r1; ++j)
        for (int c = 0; c < d; ++c) CHECK(o2[(size_t)j * d + c] == o[(size_t)j * d + c]);
    CHECK(sb_oracle_fwd(q, k, v, r, o2, NULL, B, H, T, d, T, T) == 0);        /* empty range */
    /* backward */
    double *dq = filled(n), *dk = filled(n), *dv = filled(n), *dr = with_r ? filled(nr) : NULL;
    CHECK(sb_oracle_bwd(q, k, v, r, g, dq, dk, dv, dr, B, H, T, d) == 0);
    CHECK(finite_all(dq, n) && finite_all(dk, n) && finite_all(dv, n));
    if (with_r) CHECK(finite_all(dr, nr));
    /* dense weights of the first head */
    double *A = filled((size_t)T * T), *beta = filled((size_t)T * T), *rm = filled((size_t)T);
    CHECK(sb_oracle_weights(q, k, T, d, A, beta, rm) == 0);
    CHECK(sb_oracle_weights(q, k, T, d, A, NULL, NULL) == 0);
    for (int j = 0; j < T; ++j) {
        double s = 0.0;
        for (int i = 0; i < T; ++i) s += A[(size_t)j * T + i];
        CHECK(s <= 1.0 + 1e-12 && fabs(s + rm[j] - 1.0) < 1e-12);             /* row sum = 1 - stick left */
    }
    /* error paths return codes, nothing else */
    CHECK(sb_oracle_fwd(NULL, k, v, r, o, rem, B, H, T, d, 0, T) < 0);
    CHECK(sb_oracle_fwd(q, k, v, r, o, rem, B, H, T, d, 0, T + 1) < 0);
    CHECK(sb_oracle_bwd(q, k, v, r, g, dq, dk, dv, with_r ? NULL : dq, B, H, T, d) < 0);
    free(q); free(k); free(v); free(g); free(r); free(o); free(o2); free(rem);
    free(dq); free(dk); free(dv); free(dr); free(A); free(beta); free(rm);
    return 0;
}

int main(void)
{
    if (sb_oracle_num_threads() < 1) return 1;
    const int shapes[][4] = {{1, 1, 1, 4}, {1, 2, 2, 8}, {2, 3, 17, 5}, {1, 2, 40, 16}, {2, 1, 33, 64}};
    for (size_t s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s)
        for (int with_r = 0; with_r < 2; ++with_r)
            if (one_shape(shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][3], with_r)) {
                fprintf(stderr, "shape %zu with_r %d failed\n", s, with_r);
                return 1;
            }
    printf("oracle sanitizer run clean\n");
    return 0;
}
