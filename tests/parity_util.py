"""Shared helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same
seeded inputs and compare element by element."""
import contextlib
import copy
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import pg_oracle as O

TOL_1 = 1e-5     # relative error per element after one round
TOL_10 = 1e-4    # after ten rounds


@contextlib.contextmanager
def env_setting(name, value):
    """Set an environment variable the library reads in pg_init for the duration of the block."""
    old = os.environ.get(name)
    os.environ[name] = str(value)
    try:
        yield
    finally:
        if old is None:
            os.environ.pop(name, None)
        else:
            os.environ[name] = old


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max(|ref|, rms(ref)): per-element relative error, with the matrix's
    RMS as the floor so that entries that happen to be ~0 do not dominate."""
    ref64 = ref.astype(np.float64)
    rms = float(np.sqrt(np.mean(ref64 ** 2))) if ref.size else 0.0
    den = np.maximum(np.abs(ref64), rms)
    den[den == 0] = 1.0
    return float(np.max(np.abs(got.astype(np.float64) - ref64) / den)) if ref.size else 0.0


def oracle_problem(wl):
    return O.Problem(wl.n_workers, wl.edges, wl.edge_w.astype(np.float64), wl.shapes,
                     wl.rank, wl.power_steps)


def compare_state(gb, X, Q, layers, tol, what="", phat=None, check_q=True, flags=None):
    """gb: GossipBuffers after its rounds; X[i][j], Q[e][j]: oracle state for layers[j];
    phat[e][j] / flags[j] (E, r_l): the oracle's last orthonormal columns and dropped flags."""
    worst = dict(x=0.0, q=0.0, ph=0.0)
    for j, l in enumerate(layers):
        for i in range(gb.n):
            e_ = rel_err(gb.get_layer(i, l), X[i][j])
            worst["x"] = max(worst["x"], e_)
            assert e_ <= tol, f"{what}: X worker {i} layer {l}: rel err {e_:.3e} > {tol}"
        if check_q:
            for e in range(gb.n_edges):
                e_ = rel_err(gb.get_q(e, l), Q[e][j])
                worst["q"] = max(worst["q"], e_)
                assert e_ <= tol, f"{what}: Q edge {e} layer {l}: rel err {e_:.3e} > {tol}"
        if phat is not None:
            for e in range(gb.n_edges):
                e_ = rel_err(gb.get_phat(e, l), phat[e][j])
                worst["ph"] = max(worst["ph"], e_)
                assert e_ <= tol, f"{what}: Phat edge {e} layer {l}: rel err {e_:.3e} > {tol}"
        if flags is not None:
            for e in range(gb.n_edges):
                assert np.array_equal(gb.get_flags(e, l), flags[j][e]), f"{what}: flags edge {e} layer {l}"
    return worst


class Snapshot:
    """Oracle state after some round: X[i][j], Q[e][j], phat[e][j], degenerate[j] (E, r_l)."""

    def __init__(self, X, Q, phat, degenerate):
        self.X, self.Q, self.phat, self.degenerate = X, Q, phat, degenerate


def oracle_rounds(wl, X, Q, rounds, layers, snap_at=()):
    """Run `rounds` oracle rounds in place on X[i][j] / Q[e][j] holding only `layers`.

    The oracle itself is single-threaded and handles one matrix per call; matrices are
    independent (Section 2), so the loop over layers is spread over host threads here (the C
    calls release the interpreter lock): every layer sees exactly the calls it would see in a
    serial loop, so the results are bit-identical to one thread.  Returns the RoundInfo of the
    last round; with `snap_at` (round numbers) also {round: Snapshot} of deep copies."""
    prob = oracle_problem(wl)
    sub = O.Problem(prob.n_workers, prob.edges, prob.edge_w, [prob.shapes[l] for l in layers],
                    prob.rank, prob.power_steps)
    nL, E, n = len(layers), sub.n_edges, sub.n_workers
    snaps = {t: [None] * nL for t in snap_at}
    last = [None] * nL
    O._lib("f32" if X[0][0].dtype == np.float32 else "f64")   # built and loaded before the threads start

    def one_layer(j):
        X_l = [X[i][j] for i in range(n)]
        Q_l = [Q[e][j] for e in range(E)]
        for t in range(1, rounds + 1):
            ph, deg = O.round_layer(sub, j, X_l, Q_l, want_phat=True)
            if t in snaps:
                snaps[t][j] = ([a.copy() for a in X_l], [a.copy() for a in Q_l], copy.deepcopy(ph), deg.copy())
            last[j] = (ph, deg)
            if sub.shapes[j][0] * sub.shapes[j][1] >= 10_000_000:   # a long serial call: say where it is
                print(f"   oracle: layer {layers[j]} {sub.shapes[j]} round {t} of {rounds}", flush=True)

    order = sorted(range(nL), key=lambda j: -sub.shapes[j][0] * sub.shapes[j][1])
    nthreads = max(1, min(16, os.cpu_count() or 1, nL))
    with ThreadPoolExecutor(nthreads) as pool:
        list(pool.map(one_layer, order))
    info = O.RoundInfo()
    info.phat = [[last[j][0][e] for j in range(nL)] for e in range(E)]
    info.degenerate = [last[j][1] for j in range(nL)]
    if not snap_at:
        return info
    out = {}
    for t, per in snaps.items():
        out[t] = Snapshot([[per[j][0][i] for j in range(nL)] for i in range(n)],
                          [[per[j][1][e] for j in range(nL)] for e in range(E)],
                          [[per[j][2][e] for j in range(nL)] for e in range(E)],
                          [per[j][3] for j in range(nL)])
    return info, out
