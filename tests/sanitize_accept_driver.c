/* Driver for the sanitizer run of the CPU oracle's C part (tests/test_oracle_sanitizers.py builds it together with
 * oracle/accept.c under -fsanitize=address,undefined and runs it): seeded pseudo-random logits over several
 * shapes, edge sizes included, through both entry points; prints one line per case so that the test can compare
 * the results with those of the ordinary build. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_spec_accept(const double *lp, const double *lq, const int32_t *x, const double *u,
                       int rows, int gamma, int n_p_rows, int V, double T, double tie_eps,
                       int32_t *out_n, int32_t *out_tok, int32_t *out_flags, double *rho);
int oracle_greedy_accept(const double *lp, const int32_t *x, int rows, int gamma, int n_p_rows, int V,
                         int32_t *out_n, int32_t *out_tok);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double uniform01(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0;
}

static int run_case(int rows, int gamma, int n_p_rows, int V, double T)
{
    size_t np = (size_t)rows * n_p_rows * V, nq = (size_t)rows * gamma * V;
    double *lp = malloc(sizeof(double) * (np ? np : 1)), *lq = malloc(sizeof(double) * (nq ? nq : 1));
    int32_t *x = malloc(sizeof(int32_t) * ((size_t)rows * gamma + 1));
    double *u = malloc(sizeof(double) * (size_t)rows * (gamma + 1));
    int32_t *n = malloc(sizeof(int32_t) * rows), *tok = malloc(sizeof(int32_t) * rows), *fl = malloc(sizeof(int32_t) * rows);
    double *rho = malloc(sizeof(double) * ((size_t)rows * gamma + 1));
    if (!lp || !lq || !x || !u || !n || !tok || !fl || !rho) return 2;
    for (size_t i = 0; i < np; ++i) lp[i] = 4.0 * uniform01() - 2.0;
    for (size_t i = 0; i < nq; ++i) lq[i] = lp[(i / ((size_t)gamma * V)) * n_p_rows * V + i % ((size_t)gamma * V)] + uniform01() - 0.5;
    for (size_t i = 0; i < (size_t)rows * gamma; ++i) x[i] = (int32_t)(uniform01() * V) % V;
    for (size_t i = 0; i < (size_t)rows * (gamma + 1); ++i) u[i] = uniform01();
    if (V > 3 && np) lp[1] = -INFINITY;                  /* an impossible entry */
    int rc = oracle_spec_accept(lp, lq, x, u, rows, gamma, n_p_rows, V, T, 1e-5, n, tok, fl, rho);
    long sum = 0;
    for (int b = 0; b < rows; ++b) sum = sum * 31 + n[b] * 7 + tok[b] + fl[b];
    printf("sample rows %d gamma %d n_p %d V %d T %.2f rc %d checksum %ld\n", rows, gamma, n_p_rows, V, T, rc, sum);
    rc |= oracle_greedy_accept(lp, x, rows, gamma, n_p_rows, V, n, tok);
    sum = 0;
    for (int b = 0; b < rows; ++b) sum = sum * 31 + n[b] * 7 + tok[b];
    printf("greedy rows %d gamma %d n_p %d V %d rc %d checksum %ld\n", rows, gamma, n_p_rows, V, rc, sum);
    free(lp); free(lq); free(x); free(u); free(n); free(tok); free(fl); free(rho);
    return rc;
}

int main(void)
{
    int bad = 0;
    bad |= run_case(5, 4, 5, 1000, 1.0);
    bad |= run_case(3, 4, 4, 1003, 0.7);
    bad |= run_case(1, 16, 17, 8192, 1.0);
    bad |= run_case(7, 1, 2, 1, 1.0);        /* one-entry vocabulary */
    bad |= run_case(4, 0, 1, 17, 2.0);       /* gamma = 0: plain sampling */
    bad |= run_case(2, 64, 65, 300, 1.0);    /* the longest block the boundary accepts */
    /* bad arguments are refused, nothing is written */
    int32_t dummy = -5;
    if (oracle_spec_accept(NULL, NULL, NULL, NULL, 1, 2, 4, 8, 1.0, 1e-5, &dummy, &dummy, &dummy, NULL) != -1) bad = 1;
    if (oracle_spec_accept(NULL, NULL, NULL, NULL, 1, 2, 3, 8, 0.0, 1e-5, &dummy, &dummy, &dummy, NULL) != -1) bad = 1;
    if (dummy != -5) bad = 1;
    printf("done bad %d\n", bad);
    return bad;
}
