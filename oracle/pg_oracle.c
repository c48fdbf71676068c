/*
 * PowerGossip CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, single-threaded, deliberately slow statement of one gossip round of
 * PowerGossip (Vogels, Karimireddy, Jaggi, "Practical Low-Rank Communication
 * Compression in Decentralized Deep Learning", arXiv 2008.01425) for ONE
 * parameter matrix shared by all workers.  Nothing in the product path may
 * call it; only tests, the smoke check and the benchmark's CPU-baseline leg do.
 * It shares no code with the GPU library.
 *
 * What is computed, and where the paper defines it:
 *   - the model is a list of matrices X in R^{p x q}, each handled separately
 *     (Section 2: every weight and every bias is its own matrix; conv
 *     weights are p = output channels, q = inputs x kernel size); the caller
 *     loops over layers;
 *   - compressed gossip, Eq. (2) (the unnumbered display after Eq. (1) in
 *     Section 3) and the consensus form Eq. (4) (Section 4.2, "Compressed
 *     consensus"): every worker adds W_ij * C(X_j - X_i) over its neighbours,
 *     all differences taken from the parameters at the start of the round;
 *   - the compressor is the low-rank projection of Section 3 driven by the
 *     alternating power iteration of Eq. (3) and Algorithm 2: a product with
 *     the difference (computed as X_a v - X_b v, "Linearity", Section 3.1),
 *     a normalisation, a product with the transposed difference;
 *   - rank r > 1 replaces the normalisation by an orthogonalisation of the
 *     r columns (Appendix "Changing rank vs changing # power iterations";
 *     the rank-k operators of Section 4.1).
 *
 * One "power step" here is a PAIR of Algorithm 2's iterations (odd then
 * even): P = D Q, Phat = orth(P), Q' = D^T Phat.  The approximation applied is
 * the one the even iteration returns, Phat Q'^T = Phat Phat^T D.  With s power
 * steps the pair is repeated s times on the SAME (frozen) parameters and only
 * the last approximation is applied, as Algorithm 2 overwrites and returns
 * its approximation once.  Q' (unnormalised, as Algorithm 2 stores p_j - p_i)
 * is the warm start of the next round.  Normalising Q before the product, as
 * Algorithm 2 does, is skipped: orth(D (cQ)) = orth(D Q) for c > 0.
 *
 * Edge e = (a, b) uses D_e = X_a - X_b; one state per undirected edge, so
 * Algorithm 2's v_ij = -v_ji and C(X_j - X_i) = -C(X_i - X_j) hold by
 * construction, and worker a receives -w_e U, worker b +w_e U (Lemma 1).
 *
 * Orthogonalisation: modified Gram-Schmidt, columns left to right, unit
 * 2-norm, no sign changes.  A column whose residual has squared norm below
 * max(FLT_MIN, 1e-10 * its squared norm before projection) is "degenerate":
 * its Phat column is zero, it contributes nothing to the update (Section 3.1:
 * a zero difference gives a zero update) and its Q column is left as it was.
 *
 * Precision: storage type real_t (float by default, double with
 * -DPGO_ALL_DOUBLE); every sum is accumulated in double in increasing index
 * order; P and the Gram-Schmidt run in double; Phat and Q' are rounded to
 * real_t when stored; the update of an element is summed in double over the
 * worker's incident edges in edge-list order and rounded once.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef PGO_ALL_DOUBLE
typedef double real_t;
#else
typedef float real_t;
#endif

#define PGO_OK 0
#define PGO_ERR_ARG (-1)
#define PGO_ERR_NOMEM (-4)

int pgo_real_bytes(void) { return (int)sizeof(real_t); }

/* y[row] = sum_c X[row, c] * v[c]; X is p x q row-major (Algorithm 2, odd iteration). */
static void mat_vec(const real_t *X, int p, int q, const real_t *v, double *y)
{
    for (int row = 0; row < p; ++row) {
        double acc = 0.0;
        for (int c = 0; c < q; ++c)
            acc += (double)X[(size_t)row * q + c] * (double)v[c];
        y[row] = acc;
    }
}

/* y[c] = sum_row X[row, c] * u[row] (Algorithm 2, even iteration: the product with X transposed). */
static void mat_t_vec(const real_t *X, int p, int q, const real_t *u, double *y)
{
    for (int c = 0; c < q; ++c)
        y[c] = 0.0;
    for (int row = 0; row < p; ++row) {
        double ur = (double)u[row];
        for (int c = 0; c < q; ++c)
            y[c] += (double)X[(size_t)row * q + c] * ur;
    }
}

/*
 * One gossip round for one p x q parameter matrix held by every worker.
 *
 *   edges      [2*n_edges] pairs (a, b), a != b, each undirected edge once
 *   edge_w     [n_edges]   W_ab = W_ba
 *   X          [n_workers] pointers to p*q row-major matrices, updated in place
 *   Q          [n_edges]   pointers to r_l columns of length q (column k at +k*q),
 *                          r_l = min(rank, p, q); in: Q, out: Q'
 *   Phat       NULL, or [n_edges] pointers (entries may be NULL) receiving the last
 *              step's r_l orthonormal columns of length p (column k at +k*p)
 *   degenerate NULL, or [n_edges * r_l] flags of the last step
 *   G, eta     NULL, or [n_workers] pointers to p*q stochastic gradients and the learning rate:
 *              the update step of Algorithm 1, X_i <- X_i + sum_j W_ij C(X_j - X_i) - eta * G_i, the
 *              gradient term added to the same single rounding as the gossip term
 */
int pgo_round_layer_sgd(int n_workers, int n_edges, const int32_t *edges, const double *edge_w,
                        int p, int q, int rank, int power_steps,
                        real_t *const *X, real_t *const *Q, real_t *const *Phat, int32_t *degenerate,
                        const real_t *const *G, double eta)
{
    if (n_workers < 1 || n_edges < 0 || p < 1 || q < 1 || rank < 1 || power_steps < 1)
        return PGO_ERR_ARG;
    for (int e = 0; e < n_edges; ++e) {
        int a = edges[2 * e], b = edges[2 * e + 1];
        if (a < 0 || b < 0 || a >= n_workers || b >= n_workers || a == b)
            return PGO_ERR_ARG;
    }
    int r = rank;
    if (r > p) r = p;
    if (r > q) r = q;

    const size_t pq = (size_t)p * q;
    double *pa = malloc(sizeof(double) * p), *pb = malloc(sizeof(double) * p);
    double *qa = malloc(sizeof(double) * q), *qb = malloc(sizeof(double) * q);
    double *P = malloc(sizeof(double) * (size_t)p * r);          /* one edge, r columns, in double */
    real_t *Ph = malloc(sizeof(real_t) * (size_t)n_edges * p * r); /* stored Phat of every edge */
    real_t *Qc = malloc(sizeof(real_t) * (size_t)n_edges * q * r); /* Q carried through the steps */
    int32_t *deg = malloc(sizeof(int32_t) * (size_t)n_edges * r + 4);
    double *dX = malloc(sizeof(double) * pq);
    if (!pa || !pb || !qa || !qb || !P || !Ph || !Qc || !deg || !dX) {
        free(pa); free(pb); free(qa); free(qb); free(P); free(Ph); free(Qc); free(deg); free(dX);
        return PGO_ERR_NOMEM;
    }
    for (int e = 0; e < n_edges; ++e)
        memcpy(Qc + (size_t)e * q * r, Q[e], sizeof(real_t) * (size_t)q * r);

    for (int step = 0; step < power_steps; ++step) {
        /* odd iteration on every edge: P = X_a Q - X_b Q, then orthonormalise */
        for (int e = 0; e < n_edges; ++e) {
            const real_t *Xa = X[edges[2 * e]], *Xb = X[edges[2 * e + 1]];
            for (int k = 0; k < r; ++k) {
                const real_t *v = Qc + ((size_t)e * r + k) * q;
                mat_vec(Xa, p, q, v, pa);
                mat_vec(Xb, p, q, v, pb);
                for (int row = 0; row < p; ++row)
                    P[(size_t)k * p + row] = pa[row] - pb[row];
            }
            for (int k = 0; k < r; ++k) {
                double *col = P + (size_t)k * p;
                double norm2_in = 0.0;
                for (int row = 0; row < p; ++row)
                    norm2_in += col[row] * col[row];
                for (int j = 0; j < k; ++j) {
                    const double *prev = P + (size_t)j * p; /* already orthonormal (or zero) */
                    double dot = 0.0;
                    for (int row = 0; row < p; ++row)
                        dot += prev[row] * col[row];
                    for (int row = 0; row < p; ++row)
                        col[row] -= dot * prev[row];
                }
                double norm2 = 0.0;
                for (int row = 0; row < p; ++row)
                    norm2 += col[row] * col[row];
                double floor2 = 1e-10 * norm2_in;
                if (floor2 < (double)FLT_MIN) floor2 = (double)FLT_MIN;
                int is_deg = !(norm2 >= floor2); /* also true for NaN */
                deg[(size_t)e * r + k] = is_deg;
                if (is_deg) {
                    for (int row = 0; row < p; ++row) col[row] = 0.0;
                } else {
                    double nrm = sqrt(norm2);
                    for (int row = 0; row < p; ++row) col[row] = col[row] / nrm;
                }
                real_t *dst = Ph + ((size_t)e * r + k) * p;
                for (int row = 0; row < p; ++row) dst[row] = (real_t)col[row];
            }
        }
        /* even iteration on every edge: Q' = X_a^T Phat - X_b^T Phat (not normalised) */
        for (int e = 0; e < n_edges; ++e) {
            const real_t *Xa = X[edges[2 * e]], *Xb = X[edges[2 * e + 1]];
            for (int k = 0; k < r; ++k) {
                if (deg[(size_t)e * r + k]) continue; /* keep the old column */
                const real_t *u = Ph + ((size_t)e * r + k) * p;
                mat_t_vec(Xa, p, q, u, qa);
                mat_t_vec(Xb, p, q, u, qb);
                real_t *dst = Qc + ((size_t)e * r + k) * q;
                for (int c = 0; c < q; ++c) dst[c] = (real_t)(qa[c] - qb[c]);
            }
        }
    }

    /* symmetric rank-r correction from the start-of-round parameters, worker by worker */
    for (int i = 0; i < n_workers; ++i) {
        for (size_t t = 0; t < pq; ++t) dX[t] = 0.0;
        int touched = 0;
        for (int e = 0; e < n_edges; ++e) {
            double sign;
            if (edges[2 * e] == i) sign = -1.0;          /* first endpoint: X_a -= w U */
            else if (edges[2 * e + 1] == i) sign = 1.0;  /* second endpoint: X_b += w U */
            else continue;
            touched = 1;
            for (int k = 0; k < r; ++k) {
                if (deg[(size_t)e * r + k]) continue;
                const real_t *u = Ph + ((size_t)e * r + k) * p;
                const real_t *v = Qc + ((size_t)e * r + k) * q;
                for (int row = 0; row < p; ++row) {
                    double su = sign * edge_w[e] * (double)u[row];
                    for (int c = 0; c < q; ++c)
                        dX[(size_t)row * q + c] += su * (double)v[c];
                }
            }
        }
        if (G && G[i]) {
            for (size_t t = 0; t < pq; ++t) dX[t] -= eta * (double)G[i][t];
            touched = 1;
        }
        if (touched)
            for (size_t t = 0; t < pq; ++t)
                X[i][t] = (real_t)((double)X[i][t] + dX[t]);
    }
    /* The corrections depend only on Ph and Qc, both fixed before any X was written,
       so updating the workers one after another is still the synchronous update of Eq. (4). */
    for (int e = 0; e < n_edges; ++e) {
        memcpy(Q[e], Qc + (size_t)e * q * r, sizeof(real_t) * (size_t)q * r);
        if (Phat && Phat[e])
            memcpy(Phat[e], Ph + (size_t)e * p * r, sizeof(real_t) * (size_t)p * r);
    }
    if (degenerate)
        memcpy(degenerate, deg, sizeof(int32_t) * (size_t)n_edges * r);

    free(pa); free(pb); free(qa); free(qb); free(P); free(Ph); free(Qc); free(deg); free(dX);
    return PGO_OK;
}

/* The gossip-only round (compressed consensus, Eq. (4)). */
int pgo_round_layer(int n_workers, int n_edges, const int32_t *edges, const double *edge_w,
                    int p, int q, int rank, int power_steps,
                    real_t *const *X, real_t *const *Q, real_t *const *Phat, int32_t *degenerate)
{
    return pgo_round_layer_sgd(n_workers, n_edges, edges, edge_w, p, q, rank, power_steps,
                               X, Q, Phat, degenerate, NULL, 0.0);
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 2 taken literally: `iterations` single mat-vec iterations, numbered k_done + 1 ...
 * k_done + iterations, on the unchanged parameters; the approximation of the LAST one is applied
 * (the procedure overwrites its approximation in the loop and returns it once).
 *   odd k : vhat = v / |v| in R^q;  p = X_a vhat - X_b vhat;  approximation p vhat^T;  v <- p
 *   even k: the same with X transposed: vhat = v / |v| in R^p;  p' = X_a^T vhat - X_b^T vhat;
 *           approximation vhat p'^T;  v <- p'
 * The vector therefore alternates between R^q and R^p; it is kept in two buffers, Vq (r columns
 * of length q) and Vp (r columns of length p): the one of the current space is read, the other is
 * written.  rank > 1 replaces the normalisation by the same Gram-Schmidt as above.  A column
 * whose normalisation fails (the dropped-column rule above) contributes nothing in that
 * iteration and leaves the buffer it would have written untouched.
 * With (k_done even, iterations = 2) this applies exactly the approximation of one power step.
 * G, eta: optional gradient term of Algorithm 1, as above.
 * ------------------------------------------------------------------------------------------ */
static void orthonormalise_cols(const real_t *V, int len, int r, double *work, real_t *U, int32_t *dropped)
{
    for (int k = 0; k < r; ++k)
        for (int t = 0; t < len; ++t) work[(size_t)k * len + t] = (double)V[(size_t)k * len + t];
    for (int k = 0; k < r; ++k) {
        double *col = work + (size_t)k * len;
        double norm2_in = 0.0;
        for (int t = 0; t < len; ++t) norm2_in += col[t] * col[t];
        for (int j = 0; j < k; ++j) {
            const double *prev = work + (size_t)j * len;
            double dot = 0.0;
            for (int t = 0; t < len; ++t) dot += prev[t] * col[t];
            for (int t = 0; t < len; ++t) col[t] -= dot * prev[t];
        }
        double norm2 = 0.0;
        for (int t = 0; t < len; ++t) norm2 += col[t] * col[t];
        double floor2 = 1e-10 * norm2_in;
        if (floor2 < (double)FLT_MIN) floor2 = (double)FLT_MIN;
        int is_drop = !(norm2 >= floor2);
        dropped[k] = is_drop;
        double nrm = sqrt(norm2);
        for (int t = 0; t < len; ++t) col[t] = is_drop ? 0.0 : col[t] / nrm;
        for (int t = 0; t < len; ++t) U[(size_t)k * len + t] = (real_t)col[t];
    }
}

int pgo_alg2_layer(int n_workers, int n_edges, const int32_t *edges, const double *edge_w,
                   int p, int q, int rank, long long k_done, int iterations,
                   real_t *const *X, real_t *const *Vq, real_t *const *Vp, int32_t *dropped_out,
                   const real_t *const *G, double eta)
{
    if (n_workers < 1 || n_edges < 0 || p < 1 || q < 1 || rank < 1 || iterations < 1 || k_done < 0)
        return PGO_ERR_ARG;
    int r = rank;
    if (r > p) r = p;
    if (r > q) r = q;
    const size_t pq = (size_t)p * q;
    const int mx = p > q ? p : q;
    double *ya = malloc(sizeof(double) * mx), *yb = malloc(sizeof(double) * mx);
    double *work = malloc(sizeof(double) * (size_t)mx * r);
    real_t *U = malloc(sizeof(real_t) * (size_t)n_edges * mx * r + 8); /* unit vectors of the last iteration */
    int32_t *drop = malloc(sizeof(int32_t) * (size_t)n_edges * r + 4);
    double *dX = malloc(sizeof(double) * pq);
    if (!ya || !yb || !work || !U || !drop || !dX) {
        free(ya); free(yb); free(work); free(U); free(drop); free(dX);
        return PGO_ERR_NOMEM;
    }
    int last_odd = 0;
    for (int it = 1; it <= iterations; ++it) {
        const long long k = k_done + it;
        last_odd = (int)(k & 1);
        for (int e = 0; e < n_edges; ++e) {
            const real_t *Xa = X[edges[2 * e]], *Xb = X[edges[2 * e + 1]];
            real_t *Ue = U + (size_t)e * mx * r;
            int32_t *de = drop + (size_t)e * r;
            if (last_odd) {
                orthonormalise_cols(Vq[e], q, r, work, Ue, de);
                for (int c = 0; c < r; ++c) {
                    if (de[c]) continue;
                    mat_vec(Xa, p, q, Ue + (size_t)c * q, ya);
                    mat_vec(Xb, p, q, Ue + (size_t)c * q, yb);
                    for (int row = 0; row < p; ++row) Vp[e][(size_t)c * p + row] = (real_t)(ya[row] - yb[row]);
                }
            } else {
                orthonormalise_cols(Vp[e], p, r, work, Ue, de);
                for (int c = 0; c < r; ++c) {
                    if (de[c]) continue;
                    mat_t_vec(Xa, p, q, Ue + (size_t)c * p, ya);
                    mat_t_vec(Xb, p, q, Ue + (size_t)c * p, yb);
                    for (int t = 0; t < q; ++t) Vq[e][(size_t)c * q + t] = (real_t)(ya[t] - yb[t]);
                }
            }
        }
    }
    for (int i = 0; i < n_workers; ++i) {
        for (size_t t = 0; t < pq; ++t) dX[t] = 0.0;
        int touched = 0;
        for (int e = 0; e < n_edges; ++e) {
            double sign;
            if (edges[2 * e] == i) sign = -1.0;
            else if (edges[2 * e + 1] == i) sign = 1.0;
            else continue;
            touched = 1;
            const real_t *Ue = U + (size_t)e * mx * r;
            for (int c = 0; c < r; ++c) {
                if (drop[(size_t)e * r + c]) continue;
                /* odd: (D vhat) vhat^T = Vp Uq^T ; even: vhat (D^T vhat)^T = Up Vq^T */
                const real_t *left = last_odd ? Vp[e] + (size_t)c * p : Ue + (size_t)c * p;
                const real_t *right = last_odd ? Ue + (size_t)c * q : Vq[e] + (size_t)c * q;
                for (int row = 0; row < p; ++row) {
                    double su = sign * edge_w[e] * (double)left[row];
                    for (int t = 0; t < q; ++t) dX[(size_t)row * q + t] += su * (double)right[t];
                }
            }
        }
        if (G && G[i]) {
            for (size_t t = 0; t < pq; ++t) dX[t] -= eta * (double)G[i][t];
            touched = 1;
        }
        if (touched)
            for (size_t t = 0; t < pq; ++t) X[i][t] = (real_t)((double)X[i][t] + dX[t]);
    }
    if (dropped_out) memcpy(dropped_out, drop, sizeof(int32_t) * (size_t)n_edges * r);
    free(ya); free(yb); free(work); free(U); free(drop); free(dX);
    return PGO_OK;
}
