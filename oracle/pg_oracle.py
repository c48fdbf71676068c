"""ctypes front end of the PowerGossip CPU oracle (``pg_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the CPU-baseline leg of ``bench.py``; never by the product package.

The C file states one gossip round for one parameter matrix; this module adds
the loop over layers (the paper treats every weight and bias separately,
Section 2) and the two storage precisions (float storage / all double).

Data model used here (deliberately simple, not the GPU library's layout):
  X[i][l]  numpy array (p_l, q_l), C-contiguous, worker i, layer l
  Q[e][l]  numpy array (r_l, q_l): row k is the k-th projection vector of
           edge e for layer l (Algorithm 2's v_ij, one per rank column)
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pg_oracle.c")
_LIBS = {"f32": os.path.join(_HERE, "libpg_oracle_f32.so"),
         "f64": os.path.join(_HERE, "libpg_oracle_f64.so")}
_loaded = {}


def build(force: bool = False) -> None:
    """Compile both precisions of the oracle with gcc (no fast-math, no contraction)."""
    for kind, out in _LIBS.items():
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra"]
        if kind == "f64":
            cmd.append("-DPGO_ALL_DOUBLE")
        cmd += [_SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


def _lib(kind: str):
    if kind not in _loaded:
        build()
        lib = ctypes.CDLL(_LIBS[kind])
        lib.pgo_real_bytes.restype = ctypes.c_int
        lib.pgo_round_layer.restype = ctypes.c_int
        lib.pgo_round_layer.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.pgo_round_layer_sgd.restype = ctypes.c_int
        lib.pgo_round_layer_sgd.argtypes = lib.pgo_round_layer.argtypes + [ctypes.c_void_p, ctypes.c_double]
        lib.pgo_alg2_layer.restype = ctypes.c_int
        lib.pgo_alg2_layer.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_longlong, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_double]
        assert lib.pgo_real_bytes() == (4 if kind == "f32" else 8)
        _loaded[kind] = lib
    return _loaded[kind]


@dataclass
class Problem:
    """Topology, layer shapes and compressor settings of a PowerGossip run."""
    n_workers: int
    edges: np.ndarray                    # (E, 2) int32, (a, b) pairs
    edge_w: np.ndarray                   # (E,) float64, W_ab
    shapes: List[Tuple[int, int]]        # [(p_l, q_l)]
    rank: int = 1
    power_steps: int = 1

    def __post_init__(self):
        self.edges = np.ascontiguousarray(self.edges, dtype=np.int32).reshape(-1, 2)
        self.edge_w = np.ascontiguousarray(self.edge_w, dtype=np.float64).reshape(-1)
        assert self.edge_w.shape[0] == self.edges.shape[0]

    @property
    def n_edges(self) -> int:
        return int(self.edges.shape[0])

    def layer_rank(self, l: int) -> int:
        p, q = self.shapes[l]
        return min(self.rank, p, q)


@dataclass
class RoundInfo:
    """Side results of the last power step of a round, per layer."""
    phat: List[List[np.ndarray]] = field(default_factory=list)   # [e][l] -> (r_l, p_l)
    degenerate: List[np.ndarray] = field(default_factory=list)   # [l] -> (E, r_l) int32


def _ptr_array(arrs: Sequence[Optional[np.ndarray]]):
    out = (ctypes.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        out[i] = None if a is None else a.ctypes.data
    return out


def round_layer(prob: Problem, l: int, X_l: Sequence[np.ndarray], Q_l: Sequence[np.ndarray],
                want_phat: bool = True, G_l: Optional[Sequence[np.ndarray]] = None, eta: float = 0.0):
    """One round on layer ``l``: X_l[i] (p, q) and Q_l[e] (r_l, q) are updated in place.
    With G_l (one gradient per worker) the step is Algorithm 1's: gossip term minus eta * G.

    Returns (phat, degenerate): phat[e] is (r_l, p) or None; degenerate is (E, r_l) int32.
    """
    p, q = prob.shapes[l]
    r = prob.layer_rank(l)
    dt = X_l[0].dtype
    kind = {np.dtype(np.float32): "f32", np.dtype(np.float64): "f64"}[np.dtype(dt)]
    for a in X_l:
        assert a.dtype == dt and a.shape == (p, q) and a.flags.c_contiguous
    for a in Q_l:
        assert a.dtype == dt and a.shape == (r, q) and a.flags.c_contiguous
    assert len(X_l) == prob.n_workers and len(Q_l) == prob.n_edges
    phat = [np.zeros((r, p), dtype=dt) for _ in range(prob.n_edges)] if want_phat else None
    deg = np.zeros((prob.n_edges, r), dtype=np.int32)
    if G_l is not None:
        for a in G_l:
            assert a.dtype == dt and a.shape == (p, q) and a.flags.c_contiguous
        assert len(G_l) == prob.n_workers
    rc = _lib(kind).pgo_round_layer_sgd(
        prob.n_workers, prob.n_edges, prob.edges.ctypes.data, prob.edge_w.ctypes.data,
        p, q, prob.rank, prob.power_steps,
        ctypes.cast(_ptr_array(X_l), ctypes.c_void_p),
        ctypes.cast(_ptr_array(Q_l), ctypes.c_void_p),
        ctypes.cast(_ptr_array(phat), ctypes.c_void_p) if want_phat else None,
        deg.ctypes.data,
        ctypes.cast(_ptr_array(G_l), ctypes.c_void_p) if G_l is not None else None,
        float(eta))
    if rc != 0:
        raise ValueError(f"pgo_round_layer failed with code {rc}")
    return phat, deg


def gossip_round(prob: Problem, X, Q, layers: Optional[Sequence[int]] = None,
                 want_phat: bool = False, G=None, eta: float = 0.0) -> RoundInfo:
    """One PowerGossip round over the chosen layers (default: all), in place.  With G[i][l]
    (gradients laid out like X) it is one step of Algorithm 1 with learning rate eta."""
    info = RoundInfo()
    ls = range(len(prob.shapes)) if layers is None else layers
    per_layer_phat = []
    for l in ls:
        ph, deg = round_layer(prob, l, [X[i][l] for i in range(prob.n_workers)],
                              [Q[e][l] for e in range(prob.n_edges)], want_phat=want_phat,
                              G_l=None if G is None else [G[i][l] for i in range(prob.n_workers)],
                              eta=eta)
        per_layer_phat.append(ph)
        info.degenerate.append(deg)
    if want_phat:
        info.phat = [[per_layer_phat[j][e] for j in range(len(per_layer_phat))]
                     for e in range(prob.n_edges)]
    return info


def alg2_round(prob: Problem, X, Vq, Vp, k_done: int, iterations: int,
               layers: Optional[Sequence[int]] = None, G=None, eta: float = 0.0):
    """Algorithm 2 taken literally: `iterations` single mat-vec iterations (numbered from
    k_done + 1) on frozen parameters, the last approximation applied.  Vq[e][l] is (r_l, q_l),
    Vp[e][l] is (r_l, p_l); both are updated in place.  Returns the dropped flags per layer."""
    ls = range(len(prob.shapes)) if layers is None else layers
    out = []
    for l in ls:
        p, q = prob.shapes[l]
        r = prob.layer_rank(l)
        X_l = [X[i][l] for i in range(prob.n_workers)]
        dt = X_l[0].dtype
        kind = {np.dtype(np.float32): "f32", np.dtype(np.float64): "f64"}[np.dtype(dt)]
        vq = [Vq[e][l] for e in range(prob.n_edges)]
        vp = [Vp[e][l] for e in range(prob.n_edges)]
        for a in X_l:
            assert a.dtype == dt and a.shape == (p, q) and a.flags.c_contiguous
        for a in vq:
            assert a.dtype == dt and a.shape == (r, q) and a.flags.c_contiguous
        for a in vp:
            assert a.dtype == dt and a.shape == (r, p) and a.flags.c_contiguous
        G_l = None if G is None else [G[i][l] for i in range(prob.n_workers)]
        drop = np.zeros((prob.n_edges, r), dtype=np.int32)
        rc = _lib(kind).pgo_alg2_layer(
            prob.n_workers, prob.n_edges, prob.edges.ctypes.data, prob.edge_w.ctypes.data,
            p, q, prob.rank, int(k_done), int(iterations),
            ctypes.cast(_ptr_array(X_l), ctypes.c_void_p), ctypes.cast(_ptr_array(vq), ctypes.c_void_p),
            ctypes.cast(_ptr_array(vp), ctypes.c_void_p), drop.ctypes.data,
            ctypes.cast(_ptr_array(G_l), ctypes.c_void_p) if G_l is not None else None, float(eta))
        if rc != 0:
            raise ValueError(f"pgo_alg2_layer failed with code {rc}")
        out.append(drop)
    return out
