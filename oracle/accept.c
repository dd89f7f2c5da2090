/*
 * CPU ORACLE (test infrastructure, not part of the product path).
 *
 * Speculative-sampling acceptance test, written out as its plain definition in
 * fp64 with sequential loops.  The paper names the rule only as VERIFY /
 * "speculative sampling" (Problem Formulation, Sec. 3.1; the VERIFY loop with
 * its break in Algorithm 1) and requires that the target's output
 * distribution be preserved (Abstract, Conclusion).  The rule itself is the
 * standard one: accept draft token x with probability min(1, p[x]/q[x]); at
 * the first rejection draw one token from norm(max(0, p - q)); if every draft
 * token is accepted and the verifier has one more row, draw the bonus token
 * from that row.
 *
 * Nothing here is blocked, fused or reordered: one softmax per position,
 * one left-to-right ratio test, one left-to-right running sum for the draw.
 *
 * Built by oracle/build.py with gcc; called through ctypes from
 * oracle/accept.py.  Only tests, the smoke check and the bench's CPU-baseline
 * leg may use it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define FLAG_NEAR_TIE 1      /* some tested position had |u - rho| < tie_eps   */
#define FLAG_ZERO_RESIDUAL 2 /* residual mass was 0: the draw fell back to p   */

/* softmax(l / T) for one row, the textbook way: subtract the max, exp, divide. */
static void softmax_row(const double *l, int V, double T, double *out)
{
    double m = -INFINITY;
    for (int i = 0; i < V; ++i) {
        double s = l[i] / T;
        if (s > m) m = s;
    }
    double Z = 0.0;
    for (int i = 0; i < V; ++i) {
        out[i] = exp(l[i] / T - m);
        Z += out[i];
    }
    for (int i = 0; i < V; ++i) out[i] /= Z;
}

/* Inverse-CDF draw from the unnormalised non-negative weights r[0..V):
 * the smallest k whose running sum exceeds u * sum(r); if rounding leaves no
 * such k, the last index with positive weight. */
static int32_t draw_inverse_cdf(const double *r, int V, double u)
{
    double total = 0.0;
    for (int i = 0; i < V; ++i) total += r[i];
    double t = u * total;
    double C = 0.0;
    int32_t last_pos = -1;
    for (int i = 0; i < V; ++i) {
        if (r[i] > 0.0) last_pos = i;
        C += r[i];
        if (C > t) return i;
    }
    return last_pos;
}

/*
 * One sequence.
 *   lp      [n_p_rows][V]  verifier logits, n_p_rows is gamma or gamma+1
 *   lq      [gamma][V]     drafter logits
 *   x       [gamma]        draft tokens
 *   u       [gamma+1]      uniforms in [0,1): u[j] for ratio test j, u[gamma] for the one draw
 *   T       temperature > 0
 * Outputs: *out_n accepted count in [0,gamma]; *out_tok emitted token
 * (resampled, bonus, or -1 when all accepted and there is no bonus row);
 * *out_flags FLAG_* bits; rho[gamma] (optional) the ratios p[x]/q[x] of the
 * positions that were tested, NaN for the untested ones.
 */
static void accept_one(const double *lp, int n_p_rows, const double *lq, const int32_t *x,
                       int gamma, int V, const double *u, double T, double tie_eps,
                       int32_t *out_n, int32_t *out_tok, int32_t *out_flags, double *rho,
                       double *p, double *q, double *r)
{
    int n = 0;
    int32_t flags = 0;
    if (rho)
        for (int j = 0; j < gamma; ++j) rho[j] = NAN;

    for (int j = 0; j < gamma; ++j) {
        softmax_row(lp + (size_t)j * V, V, T, p);
        softmax_row(lq + (size_t)j * V, V, T, q);
        double pj = p[x[j]], qj = q[x[j]];
        double ratio = (qj == 0.0) ? INFINITY : pj / qj;
        if (rho) rho[j] = ratio;
        if (fabs(u[j] - ratio) < tie_eps) flags |= FLAG_NEAR_TIE;
        double a = ratio < 1.0 ? ratio : 1.0;
        if (u[j] < a) {
            ++n;
        } else {
            break;
        }
    }

    int32_t tok = -1;
    if (n < gamma) {
        /* p and q still hold the softmaxes of the rejected position n */
        double Rsum = 0.0;
        for (int i = 0; i < V; ++i) {
            double d = p[i] - q[i];
            r[i] = d > 0.0 ? d : 0.0;
            Rsum += r[i];
        }
        if (!(Rsum > 0.0)) {
            flags |= FLAG_ZERO_RESIDUAL;
            for (int i = 0; i < V; ++i) r[i] = p[i];
        }
        tok = draw_inverse_cdf(r, V, u[gamma]);
    } else if (n_p_rows > gamma) {
        softmax_row(lp + (size_t)gamma * V, V, T, p);
        tok = draw_inverse_cdf(p, V, u[gamma]);
    }
    *out_n = n;
    *out_tok = tok;
    *out_flags = flags;
}

/*
 * rows independent sequences, densely packed:
 *   lp [rows][n_p_rows][V], lq [rows][gamma][V], x [rows][gamma], u [rows][gamma+1],
 *   out_n/out_tok/out_flags [rows], rho [rows][gamma] or NULL.
 * Returns 0, or -1 on a bad argument (nothing written).
 */
int oracle_spec_accept(const double *lp, const double *lq, const int32_t *x, const double *u,
                       int rows, int gamma, int n_p_rows, int V, double T, double tie_eps,
                       int32_t *out_n, int32_t *out_tok, int32_t *out_flags, double *rho)
{
    if (rows < 0 || gamma < 0 || V <= 0 || !(T > 0.0)) return -1;
    if (n_p_rows != gamma && n_p_rows != gamma + 1) return -1;
    for (size_t i = 0; i < (size_t)rows * gamma; ++i)
        if (x[i] < 0 || x[i] >= V) return -1;
    double *p = malloc(sizeof(double) * V);
    double *q = malloc(sizeof(double) * V);
    double *r = malloc(sizeof(double) * V);
    if (!p || !q || !r) {
        free(p); free(q); free(r);
        return -1;
    }
    for (int b = 0; b < rows; ++b) {
        accept_one(lp + (size_t)b * n_p_rows * V, n_p_rows, lq + (size_t)b * gamma * V,
                   x + (size_t)b * gamma, gamma, V, u + (size_t)b * (gamma + 1), T, tie_eps,
                   out_n + b, out_tok + b, out_flags + b, rho ? rho + (size_t)b * gamma : NULL,
                   p, q, r);
    }
    free(p); free(q); free(r);
    return 0;
}

/*
 * Greedy verification (the verification rule the paper lists beside speculative
 * sampling in Sec. 3.1 and compares against in its ablation on acceptance-length
 * variance): a draft token is kept iff it is the verifier's most likely token,
 * argmax_v lp_j[v], the lowest index among equal maxima; the first mismatch is
 * replaced by that argmax; if every draft token matches and the verifier has one
 * more row, its argmax is the bonus token, else -1.  No temperature, no uniforms,
 * no drafter distribution.
 *   lp [rows][n_p_rows][V], x [rows][gamma], out_n / out_tok [rows].
 */
int oracle_greedy_accept(const double *lp, const int32_t *x, int rows, int gamma, int n_p_rows, int V,
                         int32_t *out_n, int32_t *out_tok)
{
    if (rows < 0 || gamma < 0 || V <= 0) return -1;
    if (n_p_rows != gamma && n_p_rows != gamma + 1) return -1;
    for (int b = 0; b < rows; ++b) {
        const double *l = lp + (size_t)b * n_p_rows * V;
        int n = gamma;
        int32_t tok = -1;
        for (int j = 0; j < n_p_rows; ++j) {
            int best = 0;
            for (int v = 1; v < V; ++v)
                if (l[(size_t)j * V + v] > l[(size_t)j * V + best]) best = v;
            if (j < gamma && x[(size_t)b * gamma + j] == best) continue;
            n = j;            /* j < gamma: first mismatch; j == gamma: the bonus row */
            tok = best;
            break;
        }
        out_n[b] = n;
        out_tok[b] = tok;
    }
    return 0;
}
