"""Pins of the CPU oracle against what the paper and the mathematics fix.

Each test names the passage it leans on.  None of them re-types the oracle's
formula and compares it with itself: the expected values come from closed forms,
library routines (numpy SVD / QR / dense matrix products) or invariants.
"""
import os

import numpy as np
import pytest

from oracle import pg_oracle as O
from paper_2008_01425_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def ring(n):
    return W.ring_edges(n)


def make(n, edges, w, shapes, rank=1, steps=1):
    ew = np.full(len(edges), w) if np.isscalar(w) else np.asarray(w, dtype=np.float64)
    return O.Problem(n, np.asarray(edges), ew, shapes, rank, steps)


def rand_state(prob, rng, dtype=np.float64, sigma=0.3):
    bases = [rng.standard_normal(s) for s in prob.shapes]
    X = [[(b + sigma * rng.standard_normal(b.shape)).astype(dtype) for b in bases]
         for _ in range(prob.n_workers)]
    Q = [[rng.standard_normal((prob.layer_rank(l), prob.shapes[l][1])).astype(dtype)
          for l in range(len(prob.shapes))] for _ in range(prob.n_edges)]
    return X, Q


def copy_state(X, Q):
    return [[a.copy() for a in r] for r in X], [[a.copy() for a in r] for r in Q]


def consensus_distance(X):
    n = len(X)
    tot = 0.0
    for l in range(len(X[0])):
        mean = sum(X[i][l].astype(np.float64) for i in range(n)) / n
        tot += sum(((X[i][l].astype(np.float64) - mean) ** 2).sum() for i in range(n))
    return tot / n


# ---------------------------------------------------------------- Lemma 1
@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-13), (np.float32, 2e-6)])
@pytest.mark.parametrize("topo", ["ring5", "torus3x3", "star"])
def test_average_is_preserved(dtype, tol, topo):
    """Lemma 1 (appendix, 'Preserves average'): the worker mean never moves."""
    rng = np.random.default_rng(1)
    if topo == "ring5":
        n, edges, w = 5, ring(5), 1 / 3
    elif topo == "torus3x3":
        n, edges, w = 9, W.torus_edges(3, 3), 1 / 5
    else:
        n, edges, w = 4, np.array([[0, 1], [2, 0], [0, 3]]), 0.25
    prob = make(n, edges, w, [(12, 7), (5, 9), (6, 1)], rank=2, steps=2)
    X, Q = rand_state(prob, rng, dtype)
    before = [sum(X[i][l].astype(np.float64) for i in range(n)) for l in range(3)]
    for _ in range(3):
        O.gossip_round(prob, X, Q)
    for l in range(3):
        after = sum(X[i][l].astype(np.float64) for i in range(n))
        assert np.abs(after - before[l]).max() <= tol * np.abs(before[l]).max()


# ------------------------------------------------- best rank-1 (Section 3)
def test_exact_rank_one_difference_is_recovered_in_one_step():
    """Section 3: with v the top right singular vector, C_v(D) is the best rank-1
    approximation; a difference that IS rank 1 is therefore reproduced exactly after
    one power step from any start not orthogonal to it, and w = 1/2 lands both
    workers on their mean."""
    rng = np.random.default_rng(2)
    p, q = 9, 6
    u, v = rng.standard_normal(p), rng.standard_normal(q)
    base = rng.standard_normal((p, q))
    Xa, Xb = base + 0.5 * np.outer(u, v), base - 0.5 * np.outer(u, v)
    prob = make(2, [[0, 1]], 0.5, [(p, q)])
    X, Q = [[Xa.copy()], [Xb.copy()]], [[rng.standard_normal((1, q))]]
    info = O.gossip_round(prob, X, Q, want_phat=True)
    ph = info.phat[0][0][0]
    sgn = np.sign(ph @ u)
    assert np.allclose(ph, sgn * u / np.linalg.norm(u), atol=1e-12)
    # Q' = D^T Phat = +-||u|| v
    assert np.allclose(Q[0][0][0], sgn * np.linalg.norm(u) * v, atol=1e-12)
    assert np.allclose(X[0][0], base, atol=1e-12)
    assert np.allclose(X[1][0], base, atol=1e-12)


# ------------------------------------------- Eq. (3): power iteration -> SVD
@pytest.mark.parametrize("rank", [1, 2, 3])
def test_frozen_parameters_converge_to_top_singular_triplets(rank):
    """Eq. (3): when the difference does not change, the scheme is power iteration.
    With zero edge weight X is frozen; many warm-started rounds must reach the top-r
    left singular vectors (columns of Phat) and Q'_k = sigma_k * right singular vector."""
    rng = np.random.default_rng(3)
    p, q = 14, 10
    U, _ = np.linalg.qr(rng.standard_normal((p, p)))
    V, _ = np.linalg.qr(rng.standard_normal((q, q)))
    sv = np.array([5.0, 3.0, 1.5, 0.4, 0.3, 0.2, 0.1, 0.05, 0.02, 0.01])
    D = (U[:, :q] * sv) @ V.T
    base = rng.standard_normal((p, q))
    prob = make(2, [[0, 1]], 0.0, [(p, q)], rank=rank)
    X, Q = [[base + D], [base.copy()]], [[rng.standard_normal((rank, q))]]
    D = X[0][0] - X[1][0]
    Us, ss, Vts = np.linalg.svd(D)
    for _ in range(60):
        info = O.gossip_round(prob, X, Q, want_phat=True)
    assert np.array_equal(X[0][0] - X[1][0], D)          # w = 0: nothing moved
    ph = info.phat[0][0]
    for k in range(rank):
        s = np.sign(ph[k] @ Us[:, k])
        assert np.allclose(ph[k], s * Us[:, k], atol=1e-8)
        assert np.allclose(Q[0][0][k], s * ss[k] * Vts[k], atol=1e-8)
        assert abs(np.linalg.norm(Q[0][0][k]) - ss[k]) < 1e-9


def test_subspace_error_shrinks_at_power_iteration_rate():
    """Eq. (3) again, quantitatively: the angle to the top left singular vector shrinks
    by about (sigma_2/sigma_1)^2 per power step (one step = two of the paper's iterations)."""
    rng = np.random.default_rng(4)
    p, q = 12, 8
    U, _ = np.linalg.qr(rng.standard_normal((p, p)))
    V, _ = np.linalg.qr(rng.standard_normal((q, q)))
    sv = np.array([2.0, 1.0, 0.1, 0.05, 0.02, 0.01, 0.005, 0.001])
    D = (U[:, :q] * sv) @ V.T
    prob = make(2, [[0, 1]], 0.0, [(p, q)])
    X, Q = [[D.copy()], [np.zeros((p, q))]], [[rng.standard_normal((1, q))]]
    Us = np.linalg.svd(D)[0]
    errs = []
    for _ in range(8):
        info = O.gossip_round(prob, X, Q, want_phat=True)
        ph = info.phat[0][0][0]
        errs.append(np.sqrt(max(0.0, 1 - (ph @ Us[:, 0]) ** 2)))
    ratios = np.array(errs[2:7]) / np.array(errs[1:6])
    assert np.all(ratios < 0.27) and np.all(ratios > 0.23)   # (1/2)^2 = 0.25


# ------------------------------------------------ Theorem 1 / Lemma 2 step
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_consensus_distance_never_increases_on_tiny_ring(dtype):
    """Theorem 1 bounds the expected contraction; with projections Pi <= I (the step used in
    Lemma 2) the round is x <- (I - M) x with 0 <= M <= (I - W) (x) I <= 2I, so the distance
    to the mean cannot grow in any single round.  Checked on the 4-worker ring workload."""
    wl = W.get("tiny")
    prob = O.Problem(wl.n_workers, wl.edges, wl.edge_w.astype(np.float64), wl.shapes, 1, 1)
    X = [[a.astype(dtype) for a in row] for row in wl.all_params()]
    Q = [[a.astype(dtype) for a in row] for row in wl.all_q()]
    prev = consensus_distance(X)
    first = prev
    for _ in range(wl.rounds):
        O.gossip_round(prob, X, Q)
        cur = consensus_distance(X)
        assert cur <= prev * (1 + 1e-12)
        prev = cur
    assert prev < 0.7 * first


# --------------------------------------------- Eq. (1): uncompressed gossip
@pytest.mark.parametrize("steps", [1, 2])
def test_full_rank_reduces_to_plain_gossip(steps):
    """Eq. (1) without the gradient: when r >= p <= q the projector Phat Phat^T is the
    identity and a round is the textbook X <- W X over workers."""
    rng = np.random.default_rng(5)
    n, p, q = 6, 4, 9
    edges = ring(n)
    w = 0.3
    prob = make(n, edges, w, [(p, q)], rank=p, steps=steps)
    X, Q = rand_state(prob, rng)
    Wm = np.zeros((n, n))
    for a, b in edges:
        Wm[a, b] = Wm[b, a] = w
    Wm += np.diag(1 - Wm.sum(1))
    stacked = np.stack([X[i][0] for i in range(n)])               # (n, p, q)
    expect = np.einsum("ij,jpq->ipq", Wm, stacked)
    O.gossip_round(prob, X, Q)
    got = np.stack([X[i][0] for i in range(n)])
    assert np.allclose(got, expect, atol=1e-12)


def test_vectors_follow_exact_gossip_whatever_the_rank():
    """The parameter tables list bias vectors with compression 'None': a p x 1 layer has
    r_l = 1 and the rank-1 projection of a vector is the vector itself."""
    rng = np.random.default_rng(6)
    n = 5
    edges = ring(n)
    w = 1 / 3
    prob = make(n, edges, w, [(11, 1)], rank=3, steps=1)
    X, Q = rand_state(prob, rng)
    Wm = np.zeros((n, n))
    for a, b in edges:
        Wm[a, b] = Wm[b, a] = w
    Wm += np.diag(1 - Wm.sum(1))
    expect = np.einsum("ij,jpq->ipq", Wm, np.stack([X[i][0] for i in range(n)]))
    O.gossip_round(prob, X, Q)
    assert np.allclose(np.stack([X[i][0] for i in range(n)]), expect, atol=1e-13)


# --------------------------------------------------- Section 3.1 fixed point
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_consensus_is_a_fixed_point(dtype):
    """Section 3.1: if two workers agree, the compressed update is zero.  Identical workers
    stay bit-identical, the projection vectors are kept, nothing becomes NaN."""
    rng = np.random.default_rng(7)
    prob = make(4, ring(4), 1 / 3, [(8, 5), (3, 1)], rank=2)
    base = [rng.standard_normal(s).astype(dtype) for s in prob.shapes]
    X = [[b.copy() for b in base] for _ in range(4)]
    Q = [[rng.standard_normal((prob.layer_rank(l), prob.shapes[l][1])).astype(dtype)
          for l in range(2)] for _ in range(4)]
    Q0 = [[a.copy() for a in r] for r in Q]
    info = O.gossip_round(prob, X, Q, want_phat=True)
    for i in range(4):
        for l in range(2):
            assert np.array_equal(X[i][l], base[l])
    for e in range(4):
        for l in range(2):
            assert np.array_equal(Q[e][l], Q0[e][l])
            assert not np.any(info.phat[e][l])
    assert all(d.all() for d in info.degenerate)


# --------------------------- assumption A5: the applied operator is a projection
@pytest.mark.parametrize("rank", [1, 3])
def test_applied_update_is_the_left_projection_of_the_difference(rank):
    """Section 4.1 (left projection L(X) = v v^T X, rank-k form) and Eq. (2): the correction a
    round applies on an edge is w * Phat Phat^T (X_a - X_b), subtracted from a and added to b;
    Phat is orthonormal and equals the QR factor of D Q (library QR, signs fixed)."""
    rng = np.random.default_rng(8)
    p, q, w = 10, 7, 0.4
    prob = make(2, [[0, 1]], w, [(p, q)], rank=rank)
    X, Q = rand_state(prob, rng)
    Xa, Xb, Q0 = X[0][0].copy(), X[1][0].copy(), Q[0][0].copy()
    D = Xa - Xb
    info = O.gossip_round(prob, X, Q, want_phat=True)
    ph = info.phat[0][0]                                    # (r, p)
    assert np.allclose(ph @ ph.T, np.eye(rank), atol=1e-13)
    Qf, Rf = np.linalg.qr(D @ Q0.T)                        # p x r
    Qf = Qf * np.sign(np.diag(Rf))
    assert np.allclose(ph.T, Qf, atol=1e-11)
    proj = ph.T @ ph                                        # p x p projector
    assert np.allclose(X[0][0], Xa - w * proj @ D, atol=1e-13)
    assert np.allclose(X[1][0], Xb + w * proj @ D, atol=1e-13)
    assert np.allclose(Q[0][0], (D.T @ ph.T).T, atol=1e-13)
    # idempotent and contractive (A5: C(C(X)) = C(X); Pi <= I)
    assert np.allclose(proj @ proj, proj, atol=1e-12)
    assert np.linalg.norm(D - proj @ D) <= np.linalg.norm(D) * (1 + 1e-14)


def test_compressor_is_linear_in_the_difference():
    """A5, first identity, for a frozen projection: C(D1 + D2) = C(D1) + C(D2).  With the same
    Phat (same D Q direction) the update is linear in w and in D; checked by scaling D."""
    rng = np.random.default_rng(9)
    p, q = 6, 5
    base = rng.standard_normal((p, q))
    D = rng.standard_normal((p, q))
    outs = []
    for scale in (1.0, 2.0):
        prob = make(2, [[0, 1]], 0.25, [(p, q)])
        X = [[base + scale * D], [base.copy()]]
        Q = [[np.ones((1, q))]]
        O.gossip_round(prob, X, Q)
        outs.append(X[1][0] - base)
    assert np.allclose(outs[1], 2.0 * outs[0], atol=1e-13)


# ------------------------------------------------ Algorithm 2: v_ij = -v_ji
def test_reversing_an_edge_negates_its_state_and_leaves_parameters_alone():
    """Algorithm 2's initialisation and its closing note: v_ij = -v_ji and C(X_j - X_i) = -C(X_i - X_j).
    Seen from the other endpoint an edge has the negated difference and the negated vector:
    the same Phat, the negated Q', the same parameters.  Keeping the vector and negating only
    the difference negates Phat instead and leaves Q' alone."""
    rng = np.random.default_rng(10)
    shapes = [(7, 5), (4, 6)]
    prob_f = make(3, [[0, 1], [1, 2], [2, 0]], 1 / 3, shapes, rank=2, steps=2)
    prob_r = make(3, [[0, 1], [2, 1], [2, 0]], 1 / 3, shapes, rank=2, steps=2)
    X, Q = rand_state(prob_f, rng)
    X2, Q2 = copy_state(X, Q)
    X3, Q3 = copy_state(X, Q)
    Q2[1] = [-a for a in Q2[1]]
    i1 = O.gossip_round(prob_f, X, Q, want_phat=True)
    i2 = O.gossip_round(prob_r, X2, Q2, want_phat=True)
    i3 = O.gossip_round(prob_r, X3, Q3, want_phat=True)
    for i in range(3):
        for l in range(2):
            assert np.allclose(X[i][l], X2[i][l], atol=1e-14)
            assert np.allclose(X[i][l], X3[i][l], atol=1e-14)
    for l in range(2):
        assert np.allclose(Q[1][l], -Q2[1][l], atol=1e-14)
        assert np.allclose(i1.phat[1][l], i2.phat[1][l], atol=1e-14)
        assert np.allclose(Q[1][l], Q3[1][l], atol=1e-14)
        assert np.allclose(i1.phat[1][l], -i3.phat[1][l], atol=1e-14)
        assert np.allclose(Q[0][l], Q2[0][l], atol=1e-14)


def test_relabelling_workers_permutes_the_result():
    rng = np.random.default_rng(11)
    n = 5
    prob = make(n, ring(n), 1 / 3, [(6, 4)], rank=1)
    X, Q = rand_state(prob, rng)
    perm = np.array([2, 3, 4, 0, 1])                       # rotation: a ring automorphism
    X2 = [[X[perm[i]][0].copy()] for i in range(n)]
    Q2 = [[Q[(e + 2) % n][0].copy()] for e in range(n)]
    O.gossip_round(prob, X, Q)
    O.gossip_round(prob, X2, Q2)
    for i in range(n):
        assert np.allclose(X2[i][0], X[perm[i]][0], atol=1e-14)


# ------------------------------------------------ Algorithm 2: s power steps
def test_extra_power_steps_run_on_frozen_parameters_and_apply_only_the_last():
    """Algorithm 2 takes the difference as a fixed argument, overwrites its approximation in
    the loop and returns it once: s = 2 equals one step with zero weight (state advances,
    parameters frozen) followed by one step with the real weight."""
    rng = np.random.default_rng(12)
    shapes = [(9, 6)]
    X, Q = rand_state(make(4, ring(4), 1 / 3, shapes, rank=2), rng)
    Xs, Qs = copy_state(X, Q)
    O.gossip_round(make(4, ring(4), 1 / 3, shapes, rank=2, steps=2), X, Q)
    O.gossip_round(make(4, ring(4), 0.0, shapes, rank=2, steps=1), Xs, Qs)
    O.gossip_round(make(4, ring(4), 1 / 3, shapes, rank=2, steps=1), Xs, Qs)
    for i in range(4):
        assert np.array_equal(X[i][0], Xs[i][0])
    for e in range(4):
        assert np.array_equal(Q[e][0], Qs[e][0])


def test_all_edges_read_start_of_round_parameters():
    """Eq. (2) / Eq. (4) put time t-1 on the whole right-hand side: on a path 0-1-2 the update
    of worker 1 is the sum of the two single-edge corrections computed from the old values."""
    rng = np.random.default_rng(13)
    shapes = [(5, 4)]
    X, Q = rand_state(make(3, [[0, 1], [1, 2]], 0.3, shapes), rng)
    Xa, Qa = copy_state(X, Q)
    Xb, Qb = copy_state(X, Q)
    O.gossip_round(make(3, [[0, 1], [1, 2]], 0.3, shapes), X, Q)
    O.gossip_round(make(3, [[0, 1]], 0.3, shapes), Xa, [Qa[0]])
    O.gossip_round(make(3, [[1, 2]], 0.3, shapes), Xb, [Qb[1]])
    start = copy_state(rand_state(make(3, [[0, 1], [1, 2]], 0.3, shapes),
                                  np.random.default_rng(13))[0], [])[0]
    for i in range(3):
        both = (Xa[i][0] - start[i][0]) + (Xb[i][0] - start[i][0])
        assert np.allclose(X[i][0] - start[i][0], both, atol=1e-14)


# ------------------------------------------------------- degenerate columns
def test_rank_deficient_difference_flags_the_extra_column():
    """Section 3.1's zero-difference rule extended to columns: a rank-1 difference compressed at
    rank 2 has a vanishing second Gram-Schmidt residual; that column is dropped (zero Phat,
    projection vector kept) and the first column still recovers the difference."""
    rng = np.random.default_rng(14)
    p, q = 8, 6
    u, v = rng.standard_normal(p), rng.standard_normal(q)
    base = rng.standard_normal((p, q))
    prob = make(2, [[0, 1]], 0.5, [(p, q)], rank=2)
    X = [[base + np.outer(u, v)], [base.copy()]]
    Q0 = rng.standard_normal((2, q))
    Q = [[Q0.copy()]]
    info = O.gossip_round(prob, X, Q, want_phat=True)
    assert info.degenerate[0].tolist() == [[0, 1]]
    assert not np.any(info.phat[0][0][1])
    assert np.array_equal(Q[0][0][1], Q0[1])
    assert np.allclose(X[0][0], base + 0.5 * np.outer(u, v), atol=1e-12)
    assert np.allclose(X[1][0], base + 0.5 * np.outer(u, v), atol=1e-12)


# ----------------------------------------------------------- precision
def test_float_storage_tracks_the_all_double_oracle():
    """The float-storage build differs from the all-double build only by storage rounding."""
    wl = W.get("tiny")
    prob = O.Problem(wl.n_workers, wl.edges, wl.edge_w.astype(np.float64), wl.shapes, 1, 1)
    X32, Q32 = wl.all_params(), wl.all_q()
    X64 = [[a.astype(np.float64) for a in r] for r in X32]
    Q64 = [[a.astype(np.float64) for a in r] for r in Q32]
    O.gossip_round(prob, X32, Q32)
    O.gossip_round(prob, X64, Q64)
    for i in range(wl.n_workers):
        for l in range(3):
            ref = X64[i][l]
            assert np.abs(X32[i][l] - ref).max() <= 1e-6 * max(np.abs(ref).max(), 1.0)
    for e in range(wl.n_edges):
        for l in range(3):
            ref = Q64[e][l]
            assert np.abs(Q32[e][l] - ref).max() <= 1e-6 * np.sqrt((ref ** 2).mean()) * 10


# ------------------------------------------------- message sizes (tables)
def test_vector_lengths_reproduce_the_printed_compression_ratios():
    """Appendix 'Network architectures': the per-tensor 'Compression' column is
    p*q / ((p+q)/2) -- one length-p or length-q vector per iteration.  The oracle's state
    has exactly those lengths: Phat columns of length p, Q columns of length q."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "compression_ratios.txt"))
            if l.strip() and not l.startswith("#")]
    rng = np.random.default_rng(15)
    for p, q, printed in [(int(a), int(b), int(c)) for a, b, c in rows]:
        # run the oracle on every printed shape (float storage for the two LSTM matrices) and
        # read the lengths of the vectors it produces
        prob = make(2, [[0, 1]], 0.5, [(p, q)])
        X, Q = rand_state(prob, rng, np.float32 if p * q > 64 * 576 else np.float64)
        info = O.gossip_round(prob, X, Q, want_phat=True)
        sent_odd, sent_even = info.phat[0][0].size, Q[0][0].size
        assert (sent_odd, sent_even) == (p, q)
        assert round(p * q / ((sent_odd + sent_even) / 2)) == printed


# ------------------------------------------- Theorem 1 with random projections
def test_random_left_projections_contract_at_the_rate_of_theorem_1():
    """Theorem 1: with delta-approximate projections the expected squared distance to the mean
    shrinks by (1 - rho * delta) per round, rho = 1 - lambda_2(W)^2.  One power step from a fresh
    N(0,1) vector applies a rank-1 left projection Phat Phat^T with Phat = DQ/|DQ|; for an iid
    Gaussian difference that direction is (nearly) uniform on the sphere, delta = 1/p (Section
    4.1).  Averaged over many rounds the measured contraction must not be slower than the bound
    (it is an upper bound) and, on unstructured data, not much faster either."""
    rng = np.random.default_rng(21)
    n, p, q, w = 8, 12, 12, 0.436
    edges = ring(n)
    Wm = np.zeros((n, n))
    for a, b in edges:
        Wm[a, b] = Wm[b, a] = w
    Wm += np.diag(1 - Wm.sum(1))
    lam = np.sort(np.abs(np.linalg.eigvalsh(Wm)))[::-1]
    rho = 1 - lam[1] ** 2
    delta = 1.0 / p
    prob = make(n, edges, w, [(p, q)])
    ratios = []
    for trial in range(40):
        X = [[rng.standard_normal((p, q))] for _ in range(n)]
        d0 = consensus_distance(X)
        Q = [[rng.standard_normal((1, q))] for _ in range(n)]
        O.gossip_round(prob, X, Q)
        ratios.append(consensus_distance(X) / d0)
    mean = float(np.mean(ratios))
    assert mean <= 1 - rho * delta + 0.01
    assert mean >= 1 - 6 * rho * delta        # sanity: a rank-1 step cannot contract like full gossip


# ------------------------------------------------ Algorithm 1's update step: the gradient term
def test_sgd_term_without_edges_is_plain_sgd():
    """Algorithm 1's update step with no neighbours: X <- X - eta * G."""
    rng = np.random.default_rng(30)
    prob = make(3, np.zeros((0, 2), np.int32), np.zeros(0), [(5, 4), (3, 1)])
    X, Q = rand_state(prob, rng)
    G = [[rng.standard_normal(a.shape) for a in row] for row in X]
    X0 = [[a.copy() for a in row] for row in X]
    O.gossip_round(prob, X, Q, G=G, eta=0.1)
    for i in range(3):
        for l in range(2):
            assert np.allclose(X[i][l], X0[i][l] - 0.1 * G[i][l], atol=1e-15)


def test_sgd_term_adds_to_the_gossip_term_and_moves_the_mean_by_the_mean_gradient():
    """The update step of Algorithm 1 is one expression: gossip correction (from the start-of-round
    parameters) minus eta * G.  So the result is the gossip-only result minus eta * G, the
    projection state is unaffected by G, and the worker mean moves by -eta * mean(G) (Lemma 1
    plus the gradient term)."""
    rng = np.random.default_rng(31)
    n = 5
    prob = make(n, ring(n), 1 / 3, [(7, 6), (4, 1)], rank=2, steps=2)
    X, Q = rand_state(prob, rng)
    G = [[rng.standard_normal(a.shape) for a in row] for row in X]
    Xp, Qp = copy_state(X, Q)
    mean0 = [sum(X[i][l] for i in range(n)) / n for l in range(2)]
    O.gossip_round(prob, X, Q, G=G, eta=0.05)
    O.gossip_round(prob, Xp, Qp)
    for l in range(2):
        for i in range(n):
            assert np.allclose(X[i][l], Xp[i][l] - 0.05 * G[i][l], atol=1e-14)
        gm = sum(G[i][l] for i in range(n)) / n
        assert np.allclose(sum(X[i][l] for i in range(n)) / n, mean0[l] - 0.05 * gm, atol=1e-14)
        for e in range(n):
            assert np.array_equal(Q[e][l], Qp[e][l])


def test_zero_gradient_is_the_gossip_round_bitwise():
    rng = np.random.default_rng(32)
    prob = make(4, ring(4), 1 / 3, [(6, 5)], rank=1)
    X, Q = rand_state(prob, rng, np.float32)
    Xp, Qp = copy_state(X, Q)
    G = [[np.zeros_like(a) for a in row] for row in X]
    O.gossip_round(prob, X, Q, G=G, eta=0.3)
    O.gossip_round(prob, Xp, Qp)
    for i in range(4):
        assert np.array_equal(X[i][0], Xp[i][0])


# ------------------------------------------------ Algorithm 2, one iteration at a time
def _alg2_state(prob, rng, dtype=np.float64):
    Vq = [[rng.standard_normal((prob.layer_rank(l), prob.shapes[l][1])).astype(dtype)
           for l in range(len(prob.shapes))] for _ in range(prob.n_edges)]
    Vp = [[np.zeros((prob.layer_rank(l), prob.shapes[l][0]), dtype=dtype)
           for l in range(len(prob.shapes))] for _ in range(prob.n_edges)]
    return Vq, Vp


def test_one_odd_iteration_is_the_right_projection_of_section_3():
    """Section 3: C_v(X) = (X v) v^T with |v| = 1; Algorithm 2's odd iteration applies
    (D vhat) vhat^T and stores v <- D vhat in R^p."""
    rng = np.random.default_rng(40)
    p, q, w = 7, 5, 0.3
    prob = make(2, [[0, 1]], w, [(p, q)])
    X, _ = rand_state(prob, rng)
    Vq, Vp = _alg2_state(prob, rng)
    Xa, Xb, v = X[0][0].copy(), X[1][0].copy(), Vq[0][0][0].copy()
    O.alg2_round(prob, X, Vq, Vp, 0, 1)
    vh = v / np.linalg.norm(v)
    D = Xa - Xb
    assert np.allclose(Vp[0][0][0], D @ vh, atol=1e-14)
    assert np.array_equal(Vq[0][0][0], v)                       # the R^q buffer is only read
    assert np.allclose(X[0][0], Xa - w * np.outer(D @ vh, vh), atol=1e-14)
    assert np.allclose(X[1][0], Xb + w * np.outer(D @ vh, vh), atol=1e-14)


def test_one_even_iteration_is_the_left_projection():
    """Algorithm 2, even iteration ('the same with X transposed'): vhat in R^p, approximation
    vhat (D^T vhat)^T, v <- D^T vhat in R^q."""
    rng = np.random.default_rng(41)
    p, q, w = 6, 8, 0.25
    prob = make(2, [[0, 1]], w, [(p, q)])
    X, _ = rand_state(prob, rng)
    Vq, Vp = _alg2_state(prob, rng)
    Vp[0][0][0] = rng.standard_normal(p)
    Xa, Xb, v = X[0][0].copy(), X[1][0].copy(), Vp[0][0][0].copy()
    O.alg2_round(prob, X, Vq, Vp, 1, 1)                          # k = 2
    vh = v / np.linalg.norm(v)
    D = Xa - Xb
    assert np.allclose(Vq[0][0][0], D.T @ vh, atol=1e-14)
    assert np.allclose(X[0][0], Xa - w * np.outer(vh, D.T @ vh), atol=1e-14)


@pytest.mark.parametrize("rank", [1, 3])
def test_two_iterations_apply_the_same_approximation_as_one_power_step(rank):
    """Odd then even iteration on frozen parameters = P, orthonormalise, Q': the paper's
    'PowerGossip (2 iterations)' is this build's one power step (normalising v first does not
    change the orthonormalised product)."""
    rng = np.random.default_rng(42)
    n = 4
    prob = make(n, ring(n), 1 / 3, [(9, 6), (5, 1)], rank=rank)
    X, Q = rand_state(prob, rng)
    X2 = [[a.copy() for a in row] for row in X]
    Vq = [[a.copy() for a in row] for row in Q]
    Vp = [[np.zeros((prob.layer_rank(l), prob.shapes[l][0])) for l in range(2)] for _ in range(n)]
    info = O.gossip_round(prob, X, Q, want_phat=True)
    O.alg2_round(prob, X2, Vq, Vp, 0, 2)
    for i in range(n):
        for l in range(2):
            assert np.allclose(X2[i][l], X[i][l], atol=1e-12)
    for e in range(n):
        for l in range(2):
            assert np.allclose(Vq[e][l], Q[e][l], atol=1e-12)   # v after the even iteration = Q'


def test_iterations_alternate_spaces_and_keep_the_mean():
    """Algorithm 2: v 'changes between R^p and R^q'; Lemma 1 holds for every iteration count."""
    rng = np.random.default_rng(43)
    n = 5
    prob = make(n, ring(n), 1 / 3, [(8, 5)], rank=2)
    X, _ = rand_state(prob, rng)
    Vq, Vp = _alg2_state(prob, rng)
    mean0 = sum(X[i][0] for i in range(n)) / n
    k = 0
    for its in (1, 1, 3, 2):
        vq0 = [Vq[e][0].copy() for e in range(n)]
        vp0 = [Vp[e][0].copy() for e in range(n)]
        O.alg2_round(prob, X, Vq, Vp, k, its)
        k += its
        if its == 1:      # exactly one buffer was written, the other only read
            wrote_p = any(not np.array_equal(Vp[e][0], vp0[e]) for e in range(n))
            wrote_q = any(not np.array_equal(Vq[e][0], vq0[e]) for e in range(n))
            assert wrote_p != wrote_q and wrote_p == (k % 2 == 1)
        assert np.allclose(sum(X[i][0] for i in range(n)) / n, mean0, atol=1e-13)


def test_iterated_single_steps_reach_the_top_singular_pair():
    """Eq. (3) as written: alternating single iterations on a fixed difference are power iteration."""
    rng = np.random.default_rng(44)
    p, q = 10, 7
    U, _ = np.linalg.qr(rng.standard_normal((p, p)))
    V, _ = np.linalg.qr(rng.standard_normal((q, q)))
    sv = np.array([4.0, 1.0, 0.5, 0.2, 0.1, 0.05, 0.01])
    D = (U[:, :q] * sv) @ V.T
    prob = make(2, [[0, 1]], 0.0, [(p, q)])
    X = [[D.copy()], [np.zeros((p, q))]]
    Vq, Vp = _alg2_state(prob, rng)
    for k in range(40):
        O.alg2_round(prob, X, Vq, Vp, k, 1)
    Us, ss, Vts = np.linalg.svd(D)
    s1 = np.sign(Vp[0][0][0] @ Us[:, 0])
    assert np.allclose(Vp[0][0][0], s1 * ss[0] * Us[:, 0], atol=1e-8)
    s2 = np.sign(Vq[0][0][0] @ Vts[0])
    assert np.allclose(Vq[0][0][0], s2 * ss[0] * Vts[0], atol=1e-8)


def test_iteration_on_identical_workers_writes_a_zero_vector_then_drops_it_and_keeps_the_other_buffer():
    """Section 3.1: a zero difference gives a zero update.  Algorithm 2 on identical workers: the
    odd iteration stores p_j - p_i = 0 in the R^p buffer; the next (even) iteration cannot
    normalise that vector, so it is dropped: nothing is applied, and the R^q buffer it would have
    written keeps its bits (zeros there would be a state that can never recover)."""
    rng = np.random.default_rng(45)
    n, p, q = 3, 7, 5
    prob = make(n, ring(n), 1 / 3, [(p, q)], rank=2)
    base = rng.standard_normal((p, q))
    X = [[base.copy()] for _ in range(n)]
    Vq, Vp = _alg2_state(prob, rng)
    for e in range(n):
        Vp[e][0][:] = rng.standard_normal((2, p))       # stale content that the odd iteration must overwrite
    vq0 = [Vq[e][0].copy() for e in range(n)]
    flags = O.alg2_round(prob, X, Vq, Vp, 0, 1)          # k = 1, odd
    assert not flags[0].any()                            # a random v normalises fine
    for e in range(n):
        assert not Vp[e][0].any()                        # p_j - p_i = 0, written
        assert np.array_equal(Vq[e][0], vq0[e])
    flags = O.alg2_round(prob, X, Vq, Vp, 1, 1)          # k = 2, even: v = 0 in R^p
    assert flags[0].all()
    for e in range(n):
        assert np.array_equal(Vq[e][0], vq0[e])          # untouched, bit for bit
        assert not Vp[e][0].any()
    for i in range(n):
        assert np.array_equal(X[i][0], base)
    # and the state recovers once the workers differ again
    X[0][0] += rng.standard_normal((p, q))
    flags = O.alg2_round(prob, X, Vq, Vp, 2, 1)          # k = 3, odd, from the kept R^q vectors
    assert not flags[0].any() and Vp[0][0].any()


def test_iterations_on_a_rank_one_difference_drop_the_second_column_in_the_even_iteration():
    """Algorithm 2 at rank 2 on D = u v^T (reading: Gram-Schmidt over the stored columns, a column
    that cannot be normalised contributes nothing and leaves the buffer it would have written
    alone).  Odd iteration: both unit vectors are fine, both products are multiples of u.  Even
    iteration: the second stored column is parallel to the first, its residual vanishes, it is
    dropped; the first column alone gives uhat (D^T uhat)^T = D, so with w = 1/2 both workers
    land on their mean, and column 2 of the R^q buffer keeps its bits."""
    rng = np.random.default_rng(46)
    p, q = 9, 6
    u, v = rng.standard_normal(p), rng.standard_normal(q)
    base = rng.standard_normal((p, q))
    prob = make(2, [[0, 1]], 0.5, [(p, q)], rank=2)
    X = [[base + np.outer(u, v)], [base.copy()]]
    Vq, Vp = _alg2_state(prob, rng)
    vq0 = Vq[0][0].copy()
    flags = O.alg2_round(prob, X, Vq, Vp, 0, 2)          # k = 1 (odd) and k = 2 (even), one call
    assert flags[0].tolist() == [[0, 1]]
    uh = u / np.linalg.norm(u)
    s = np.sign(Vp[0][0][0] @ uh)
    # R^p buffer after the odd iteration: D vhat_k = u (v . vhat_k), both columns along u
    for k in range(2):
        assert np.allclose(np.abs(Vp[0][0][k] @ uh), np.linalg.norm(Vp[0][0][k]), rtol=1e-12)
    assert np.allclose(Vq[0][0][0], s * np.linalg.norm(u) * v, atol=1e-12)   # D^T uhat
    assert np.array_equal(Vq[0][0][1], vq0[1])                               # dropped: kept
    mean = base + 0.5 * np.outer(u, v)
    assert np.allclose(X[0][0], mean, atol=1e-12) and np.allclose(X[1][0], mean, atol=1e-12)


def test_gradient_term_of_algorithm_1_inside_the_single_iteration_procedure():
    """The update step of Algorithm 1 around Algorithm 2's compressor: without neighbours the step
    is X - eta G; with neighbours it is the gradient-free result minus eta G, for an odd and for
    an even last iteration, and neither vector buffer depends on G."""
    rng = np.random.default_rng(47)
    lone = make(3, np.zeros((0, 2), np.int32), np.zeros(0), [(5, 4), (3, 1)])
    X, _ = rand_state(lone, rng)
    G = [[rng.standard_normal(a.shape) for a in row] for row in X]
    X0 = [[a.copy() for a in row] for row in X]
    O.alg2_round(lone, X, [], [], 0, 1, G=G, eta=0.2)
    for i in range(3):
        for l in range(2):
            assert np.allclose(X[i][l], X0[i][l] - 0.2 * G[i][l], atol=1e-15)
            assert not np.array_equal(X[i][l], X0[i][l])
    n = 5
    prob = make(n, ring(n), 1 / 3, [(7, 6), (4, 1)], rank=2)
    for k_done, its in ((0, 1), (1, 1), (0, 2), (2, 3)):
        X, _ = rand_state(prob, rng)
        Vq, Vp = _alg2_state(prob, rng)
        for e in range(n):
            for l in range(2):
                Vp[e][l][:] = rng.standard_normal(Vp[e][l].shape)
        G = [[rng.standard_normal(a.shape) for a in row] for row in X]
        Xp = [[a.copy() for a in row] for row in X]
        Vqp = [[a.copy() for a in row] for row in Vq]
        Vpp = [[a.copy() for a in row] for row in Vp]
        O.alg2_round(prob, X, Vq, Vp, k_done, its, G=G, eta=0.05)
        O.alg2_round(prob, Xp, Vqp, Vpp, k_done, its)
        for l in range(2):
            for i in range(n):
                assert np.allclose(X[i][l], Xp[i][l] - 0.05 * G[i][l], atol=1e-14)
                assert not np.allclose(X[i][l], Xp[i][l], atol=1e-6)
            for e in range(n):
                assert np.array_equal(Vq[e][l], Vqp[e][l]) and np.array_equal(Vp[e][l], Vpp[e][l])
