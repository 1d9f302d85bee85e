/*
 * CPU float64 oracle for causal stick-breaking attention.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the GPU library and to be
 * timed as a CPU baseline.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product path never does.  It shares no code,
 * header, table or constant with the GPU sources.
 *
 * What is computed is the paper's Eq. 1 (section 2) written out directly:
 *
 *     z[i,j]  = q_j . k_i / sqrt(d_head)
 *     beta    = sigma(z),  sigma(x) = 1 / (1 + exp(-x))         (Fig. 1 caption)
 *     A[i,j]  = beta[i,j] * prod_{i<k<j} (1 - beta[k,j])        (Eq. 1)
 *     o_j     = sum_{i<j} A[i,j] v_i                            (Eq. 1; o_1 = 0)
 *
 * with the product evaluated as a running product while walking the keys from
 * j-1 down to 1: no log-space rewrite, no tiling, no reordering.  The
 * backward follows Eq. 4 (section 4, "Backward") with the sum taken over the
 * keys at or before i (the reading that the tiled backward algorithm's
 * left-to-right cumulative sum implements, and that finite differences of the
 * forward confirm):
 *
 *     G[i,j]  = A[i,j] * (dO_j . v_i)                  dL/d(log A), Eq. 4 left
 *     dZ[i,j] = G[i,j] - beta[i,j] * sum_{i'<=i} G[i',j]          Eq. 4 right
 *     dQ_j = s * sum_i dZ[i,j] k_i,  dK_i = s * sum_j dZ[i,j] q_j,
 *     dV_i = sum_j A[i,j] dO_j,      s = 1/sqrt(d_head)
 *
 * Remainder bias (Appendix C, the remainder-bias output equation): with one embedding
 * r per head, o_j gets the unused part of the stick times r,
 *
 *     o_j = sum_{i<j} A[i,j] v_i + rem_j r,   rem_j = 1 - sum_i A[i,j] = prod_{k<j} (1 - beta[k,j]).
 *
 * Its gradients follow from d rem_j / d z[i,j] = -beta[i,j] rem_j (each factor of the
 * product depends on one logit):  dr = sum_j rem_j dO_j (over every batch entry of the
 * head), and dZ[i,j] gains -beta[i,j] rem_j (dO_j . r): the remainder behaves like one
 * more term in front of the cumulative sum of G.
 *
 * Indices here are 0-based: query row j attends to keys 0..j-1.
 * Layout of every tensor: [B, H, T, d] contiguous, d fastest.  All host memory,
 * owned by the caller.  Threads: OpenMP over (head, row).
 *
 * Pins (tests/test_oracle_*.py): brute-force product in pure Python, the
 * log-space form (Eq. 2), the gated recurrence of section 3, the geometric
 * closed form for constant logits, row sums, the first-token zero, saturation
 * limits, and central finite differences for every gradient.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* logistic function, evaluated without overflow on either side */
static double sb_sigma(double x)
{
    if (x >= 0.0) {
        return 1.0 / (1.0 + exp(-x));
    } else {
        double e = exp(x);
        return e / (1.0 + e);
    }
}

static double sb_dot(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += a[c] * b[c];
    return s;
}

/*
 * One query row j of one head: fills A[0..j-1] (and beta[0..j-1] when beta is
 * not NULL) and returns the remaining stick prod_{k<j} (1 - beta[k,j]).
 * 1 - beta is taken as sigma(-z), never as 1.0 - beta, so it keeps its
 * relative precision when beta is close to 1.
 */
static double sb_row(const double *qj, const double *K, int j, int d,
                     double *A, double *beta)
{
    const double scale = 1.0 / sqrt((double)d);
    double stick = 1.0; /* prod over the keys already passed (those nearer to j) */
    for (int i = j - 1; i >= 0; --i) {
        double z = sb_dot(qj, K + (size_t)i * d, d) * scale;
        double b = sb_sigma(z);
        A[i] = b * stick;
        if (beta) beta[i] = b;
        stick *= sb_sigma(-z);
    }
    return stick;
}

int sb_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Attention weights of one head as dense T x T matrices, row = query j,
 * column = key i (so A_out[j*T + i] is the paper's A[i,j]); entries with
 * i >= j are zero.  beta_out may be NULL.  For small T (tests).
 */
int sb_oracle_weights(const double *q, const double *k, int T, int d,
                      double *A_out, double *beta_out, double *rem_out)
{
    if (!q || !k || !A_out || T < 1 || d < 1) return -1;
    memset(A_out, 0, sizeof(double) * (size_t)T * T);
    if (beta_out) memset(beta_out, 0, sizeof(double) * (size_t)T * T);
    for (int j = 0; j < T; ++j) {
        double r = sb_row(q + (size_t)j * d, k, j, d, A_out + (size_t)j * T,
                          beta_out ? beta_out + (size_t)j * T : NULL);
        if (rem_out) rem_out[j] = r;
    }
    return 0;
}

/*
 * Forward for query rows row_begin <= j < row_end of every (b,h).
 * o   [B,H,T,d]: rows in the range are written, others untouched.
 * rem [B,H,T]  : remaining stick prod_{k<j}(1-beta[k,j]) = 1 - sum_i A[i,j];
 *                may be NULL.
 * r   [H,d]    : remainder-bias embeddings, or NULL for plain Eq. 1.
 */
int sb_oracle_fwd(const double *q, const double *k, const double *v, const double *r,
                  double *o, double *rem,
                  int B, int H, int T, int d, int row_begin, int row_end)
{
    if (!q || !k || !v || !o) return -1;
    if (B < 1 || H < 1 || T < 1 || d < 1) return -2;
    if (row_begin < 0 || row_end > T || row_begin > row_end) return -2;
    const long nrows = (long)(row_end - row_begin);
    const long total = (long)B * H * nrows;
    int failed = 0;
#pragma omp parallel
    {
        double *A = (double *)malloc(sizeof(double) * (size_t)T);
        if (!A) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 8)
        for (long w = 0; w < total; ++w) {
            if (!A) continue;
            long bh = w / nrows;
            /* long rows first: better balance under dynamic scheduling */
            int j = row_end - 1 - (int)(w % nrows);
            const double *Q = q + (size_t)bh * T * d;
            const double *K = k + (size_t)bh * T * d;
            const double *V = v + (size_t)bh * T * d;
            double *oj = o + ((size_t)bh * T + j) * d;
            double stick = sb_row(Q + (size_t)j * d, K, j, d, A, NULL);
            for (int c = 0; c < d; ++c) oj[c] = 0.0;
            for (int i = 0; i < j; ++i) {
                const double a = A[i];
                const double *vi = V + (size_t)i * d;
                for (int c = 0; c < d; ++c) oj[c] += a * vi[c];
            }
            if (r) {
                const double *rh = r + (size_t)(bh % H) * d;
                for (int c = 0; c < d; ++c) oj[c] += stick * rh[c];
            }
            if (rem) rem[(size_t)bh * T + j] = stick;
        }
        free(A);
    }
    return failed ? -3 : 0;
}

/*
 * Backward: all rows of every (b,h).  dq, dk, dv [B,H,T,d] are overwritten.
 * Works head by head with dense T x T scratch for A and dZ (16*T*T bytes).
 * r [H,d] and dr [H,d] (overwritten): remainder bias, both NULL for plain Eq. 1.
 */
int sb_oracle_bwd(const double *q, const double *k, const double *v, const double *r,
                  const double *dout, double *dq, double *dk, double *dv, double *dr,
                  int B, int H, int T, int d)
{
    if (!q || !k || !v || !dout || !dq || !dk || !dv) return -1;
    if ((r == NULL) != (dr == NULL)) return -1;
    if (B < 1 || H < 1 || T < 1 || d < 1) return -2;
    if (dr) memset(dr, 0, sizeof(double) * (size_t)H * d);
    const double scale = 1.0 / sqrt((double)d);
    double *Amat = (double *)malloc(sizeof(double) * (size_t)T * T);
    double *Zmat = (double *)malloc(sizeof(double) * (size_t)T * T);
    if (!Amat || !Zmat) { free(Amat); free(Zmat); return -3; }
    int failed = 0;

    for (long bh = 0; bh < (long)B * H; ++bh) {
        const double *Q = q + (size_t)bh * T * d;
        const double *K = k + (size_t)bh * T * d;
        const double *V = v + (size_t)bh * T * d;
        const double *DO = dout + (size_t)bh * T * d;
        double *DQ = dq + (size_t)bh * T * d;
        double *DK = dk + (size_t)bh * T * d;
        double *DV = dv + (size_t)bh * T * d;

        /* per query row: A, G, dZ (Eq. 4), dQ */
#pragma omp parallel
        {
            double *beta = (double *)malloc(sizeof(double) * (size_t)T);
            if (!beta) {
#pragma omp atomic write
                failed = 1;
            }
#pragma omp for schedule(dynamic, 8)
            for (int jj = 0; jj < T; ++jj) {
                if (!beta) continue;
                int j = T - 1 - jj;
                double *A = Amat + (size_t)j * T;
                double *dZ = Zmat + (size_t)j * T;
                const double stick = sb_row(Q + (size_t)j * d, K, j, d, A, beta);
                /* sum_{i'<=i} G[i',j]; with a remainder bias the unused stick comes first */
                double prefix = r ? stick * sb_dot(DO + (size_t)j * d, r + (size_t)(bh % H) * d, d) : 0.0;
                if (dr) {
                    double *drh = dr + (size_t)(bh % H) * d;
                    for (int c = 0; c < d; ++c) {
#pragma omp atomic
                        drh[c] += stick * DO[(size_t)j * d + c];
                    }
                }
                for (int i = 0; i < j; ++i) {
                    double g = A[i] * sb_dot(DO + (size_t)j * d, V + (size_t)i * d, d);
                    prefix += g;
                    dZ[i] = g - beta[i] * prefix;
                }
                double *dqj = DQ + (size_t)j * d;
                for (int c = 0; c < d; ++c) dqj[c] = 0.0;
                for (int i = 0; i < j; ++i) {
                    const double *ki = K + (size_t)i * d;
                    for (int c = 0; c < d; ++c) dqj[c] += dZ[i] * ki[c];
                }
                for (int c = 0; c < d; ++c) dqj[c] *= scale;
            }
            free(beta);
        }
        if (failed) break;

        /* per key row: dK, dV summed over the later queries */
#pragma omp parallel for schedule(dynamic, 8)
        for (int i = 0; i < T; ++i) {
            double *dki = DK + (size_t)i * d;
            double *dvi = DV + (size_t)i * d;
            for (int c = 0; c < d; ++c) { dki[c] = 0.0; dvi[c] = 0.0; }
            for (int j = i + 1; j < T; ++j) {
                const double dz = Zmat[(size_t)j * T + i];
                const double a = Amat[(size_t)j * T + i];
                const double *qj = Q + (size_t)j * d;
                const double *doj = DO + (size_t)j * d;
                for (int c = 0; c < d; ++c) {
                    dki[c] += dz * qj[c];
                    dvi[c] += a * doj[c];
                }
            }
            for (int c = 0; c < d; ++c) dki[c] *= scale;
        }
    }
    free(Amat);
    free(Zmat);
    return failed ? -3 : 0;
}
