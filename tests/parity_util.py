"""Shared helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same
seeded inputs and compare element by element."""
import numpy as np

from oracle import pg_oracle as O

TOL_1 = 1e-5     # relative error per element after one round
TOL_10 = 1e-4    # after ten rounds


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


def compare_state(gb, X, Q, layers, tol, what="", phat=None, check_q=True):
    """gb: GossipBuffers after its rounds; X[i][j], Q[e][j]: oracle state for layers[j]."""
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
    return worst


def oracle_rounds(wl, X, Q, rounds, layers):
    """Run `rounds` oracle rounds in place on X[i][j] / Q[e][j] holding only `layers`."""
    prob = oracle_problem(wl)
    sub = O.Problem(prob.n_workers, prob.edges, prob.edge_w, [prob.shapes[l] for l in layers],
                    prob.rank, prob.power_steps)
    info = None
    for _ in range(rounds):
        info = O.gossip_round(sub, X, Q, want_phat=True)
    return info
