/* Host-only driver that runs the CPU oracle's three entry points under AddressSanitizer and
 * UndefinedBehaviorSanitizer on small, odd-shaped problems (vectors, rank above a dimension,
 * identical workers, an isolated worker, gradients).  Built and run by tests/test_host_api.py;
 * it checks nothing about the values -- the sanitizers' verdict is the result. */
#include <stdio.h>

#include "../oracle/pg_oracle.c"

static unsigned long long rng_state = 88172645463325252ull;
static double rnd(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state % 2000001ull) / 1000000.0 - 1.0;
}

static int run_case(int n, int n_edges, const int32_t *edges, int p, int q, int rank, int steps, int same)
{
    int r = rank < p ? rank : p;
    if (r > q) r = q;
    double w[16];
    real_t *X[8], *G[8], *Q[16], *Ph[16], *Vp[16];
    int32_t flags[16 * 8];
    for (int e = 0; e < n_edges; ++e) w[e] = 0.2;
    for (int i = 0; i < n; ++i) {
        X[i] = malloc(sizeof(real_t) * (size_t)p * q);
        G[i] = malloc(sizeof(real_t) * (size_t)p * q);
        for (int t = 0; t < p * q; ++t) {
            X[i][t] = (real_t)(same ? (double)(t % 7) : rnd());
            G[i][t] = (real_t)rnd();
        }
    }
    for (int e = 0; e < n_edges; ++e) {
        Q[e] = malloc(sizeof(real_t) * (size_t)q * r);
        Ph[e] = malloc(sizeof(real_t) * (size_t)p * r);
        Vp[e] = malloc(sizeof(real_t) * (size_t)p * r);
        for (int t = 0; t < q * r; ++t) Q[e][t] = (real_t)rnd();
        for (int t = 0; t < p * r; ++t) Vp[e][t] = (real_t)0;
    }
    int rc = pgo_round_layer(n, n_edges, edges, w, p, q, rank, steps, X, Q, Ph, flags);
    rc |= pgo_round_layer_sgd(n, n_edges, edges, w, p, q, rank, steps, X, Q, NULL, NULL,
                              (const real_t *const *)G, 0.1);
    rc |= pgo_alg2_layer(n, n_edges, edges, w, p, q, rank, 0, 3, X, Q, Vp, flags,
                         (const real_t *const *)G, 0.1);
    rc |= pgo_alg2_layer(n, n_edges, edges, w, p, q, rank, 3, 1, X, Q, Vp, NULL, NULL, 0.0);
    for (int i = 0; i < n; ++i) { free(X[i]); free(G[i]); }
    for (int e = 0; e < n_edges; ++e) { free(Q[e]); free(Ph[e]); free(Vp[e]); }
    return rc;
}

int main(void)
{
    const int32_t ring4[] = {0, 1, 1, 2, 2, 3, 3, 0};
    const int32_t path[] = {0, 1, 2, 1};           /* worker 3 isolated */
    int rc = 0;
    rc |= run_case(4, 4, ring4, 7, 5, 1, 1, 0);
    rc |= run_case(4, 4, ring4, 5, 9, 3, 2, 0);
    rc |= run_case(4, 4, ring4, 6, 1, 2, 1, 0);   /* vector */
    rc |= run_case(4, 4, ring4, 1, 6, 4, 1, 0);   /* single row */
    rc |= run_case(4, 4, ring4, 3, 4, 8, 2, 0);   /* rank above both dimensions */
    rc |= run_case(4, 4, ring4, 6, 4, 2, 2, 1);   /* identical workers: every column dropped */
    rc |= run_case(4, 2, path, 5, 4, 2, 1, 0);
    rc |= run_case(3, 0, path, 5, 4, 2, 1, 0);    /* no edges */
    printf(rc == 0 ? "oracle sanitize ok\n" : "oracle sanitize FAILED rc=%d\n", rc);
    return rc != 0;
}
