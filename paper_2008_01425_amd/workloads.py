"""Seeded synthetic PowerGossip workloads (inputs only -- none of the method's arithmetic).

Both the GPU library's callers and the CPU oracle's callers draw their inputs
from here, so that they start from identical bits.  Shapes follow the models
the paper trains (its ResNet-20 and LSTM parameter tables in the appendix
"Network architectures") and the other model shapes this build is measured on;
values follow the paper's setting of workers that start from a common point
and drift apart: X_i = B + sigma * N(0, 1) with a shared base B ~ N(0, 1), and
projection vectors initialised entry-wise N(0, 1) (initialisation of Algorithm 2).

Every (worker, layer), (layer) and (edge, layer) block has its own counter-based
stream (numpy Philox keyed by (seed, tag, indices)), so any single block can be
regenerated without generating the rest.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


def ring_edges(n: int) -> np.ndarray:
    """Ring 0-1-...-(n-1)-0 as (i, i+1 mod n); n = 2 gives the single edge (0, 1)."""
    if n < 2:
        return np.zeros((0, 2), dtype=np.int32)
    if n == 2:
        return np.array([[0, 1]], dtype=np.int32)
    return np.array([[i, (i + 1) % n] for i in range(n)], dtype=np.int32)


def torus_edges(rows: int, cols: int) -> np.ndarray:
    """rows x cols torus, row-major worker ids: (v, right(v)) then (v, down(v)) for every v."""
    out = []
    for r in range(rows):
        for c in range(cols):
            v = r * cols + c
            out.append((v, r * cols + (c + 1) % cols))
            out.append((v, ((r + 1) % rows) * cols + c))
    return np.array(out, dtype=np.int32)


def resnet20_shapes() -> List[Tuple[int, int]]:
    """Conv weights as out x (in*k*k), each followed by two length-out vectors; fc and its bias."""
    shapes: List[Tuple[int, int]] = []

    def conv(out, inp, k=3):
        shapes.extend([(out, inp * k * k), (out, 1), (out, 1)])

    conv(16, 3)
    inp = 16
    for planes in (16, 32, 64):
        for _ in range(3):
            conv(planes, inp)
            conv(planes, planes)
            inp = planes
    shapes.extend([(10, 64), (10, 1)])
    return shapes


def vgg16_shapes() -> List[Tuple[int, int]]:
    chans = [64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512]
    shapes, inp = [], 3
    for out in chans:
        shapes.append((out, inp * 9))
        inp = out
    shapes.append((10, 512))
    return shapes


def lstm_shapes() -> List[Tuple[int, int]]:
    return [(33278, 650)] + [(2600, 650)] * 4


def resnet50_shapes() -> List[Tuple[int, int]]:
    shapes: List[Tuple[int, int]] = []

    def conv(out, inp, k):
        shapes.extend([(out, inp * k * k), (out, 1), (out, 1)])

    conv(64, 3, 7)
    inp = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            conv(planes, inp, 1)
            conv(planes, planes, 3)
            conv(4 * planes, planes, 1)
            if b == 0:
                conv(4 * planes, inp, 1)
            inp = 4 * planes
    shapes.extend([(1000, 2048), (1000, 1)])
    return shapes


@dataclass
class Workload:
    name: str
    n_workers: int
    edges: np.ndarray          # (E, 2) int32
    edge_w: np.ndarray         # (E,) float32
    shapes: List[Tuple[int, int]]
    rank: int
    power_steps: int
    sigma: float               # std of the per-worker deviation from the base
    rounds: int                # rounds the configuration asks for in long parity runs
    seed: int = 0
    # Optional planted spectrum (sigma_1, sigma_2, ...): every layer gets shared orthonormal
    # directions u_k, v_k and worker i adds (i + 1) * sum_k sigma_k u_k v_k^T, so the difference
    # of workers a and b is (a - b) * sum_k sigma_k u_k v_k^T + noise: singular values in the
    # planted ratios on every edge (the paper's premise: differences with a fast-decaying
    # spectrum, Section 3.1 and the appendix on power spectra), above a flat noise floor.
    spectrum: Tuple[float, ...] = ()

    @property
    def n_edges(self) -> int:
        return int(self.edges.shape[0])

    @property
    def params_per_worker(self) -> int:
        return int(sum(p * q for p, q in self.shapes))

    def layer_rank(self, l: int) -> int:
        p, q = self.shapes[l]
        return min(self.rank, p, q)

    # ---- seeded blocks -------------------------------------------------
    def _rng(self, tag: int, *idx: int) -> np.random.Generator:
        key = np.random.SeedSequence([self.seed, tag, *idx])
        return np.random.Generator(np.random.Philox(key))

    def base(self, l: int) -> np.ndarray:
        p, q = self.shapes[l]
        return self._rng(1, l).standard_normal((p, q), dtype=np.float32)

    def worker_layer(self, i: int, l: int, base: np.ndarray | None = None) -> np.ndarray:
        """X_i^l = B^l + sigma * N(0,1), float32, shape (p_l, q_l)."""
        p, q = self.shapes[l]
        b = self.base(l) if base is None else base
        noise = self._rng(2, i, l).standard_normal((p, q), dtype=np.float32)
        x = b + np.float32(self.sigma) * noise
        if self.spectrum:
            x = x.astype(np.float64) + (i + 1) * self.planted(l)
        return x.astype(np.float32)

    def planted(self, l: int) -> np.ndarray:
        """sum_k sigma_k u_k v_k^T (float64) with random orthonormal u_k in R^p, v_k in R^q."""
        p, q = self.shapes[l]
        k = min(len(self.spectrum), p, q)
        rng = self._rng(4, l)
        u, _ = np.linalg.qr(rng.standard_normal((p, k)))
        v, _ = np.linalg.qr(rng.standard_normal((q, k)))
        return (u * np.asarray(self.spectrum[:k], dtype=np.float64)) @ v.T

    def q_init(self, e: int, l: int) -> np.ndarray:
        """Initial projection vectors of edge e, layer l: (r_l, q_l) float32, entry-wise N(0,1)."""
        _, q = self.shapes[l]
        return self._rng(3, e, l).standard_normal((self.layer_rank(l), q), dtype=np.float32)

    def all_params(self, layers=None):
        """X[i][l] for every worker and the chosen layers (default all)."""
        ls = list(range(len(self.shapes))) if layers is None else list(layers)
        bases = {l: self.base(l) for l in ls}
        return [[self.worker_layer(i, l, bases[l]) for l in ls] for i in range(self.n_workers)]

    def all_q(self, layers=None):
        ls = list(range(len(self.shapes))) if layers is None else list(layers)
        return [[self.q_init(e, l) for l in ls] for e in range(self.n_edges)]


def _mk(name, n, edges, w, shapes, rank, steps, sigma, rounds):
    ew = np.full((edges.shape[0],), w, dtype=np.float32)
    return Workload(name, n, edges, ew, shapes, rank, steps, sigma, rounds)


def get(name: str) -> Workload:
    """The named configurations this build is tested and measured on."""
    if name == "tiny":
        return _mk(name, 4, ring_edges(4), 1 / 3, [(64, 32), (32, 16), (16, 1)], 1, 1, 0.1, 10)
    if name == "resnet20":
        return _mk(name, 8, ring_edges(8), 1 / 3, resnet20_shapes(), 1, 1, 0.01, 10)
    if name in ("vgg16", "vgg16_r1"):
        return _mk("vgg16_r1", 16, ring_edges(16), 1 / 3, vgg16_shapes(), 1, 1, 0.01, 10)
    if name == "vgg16_r2":
        return _mk(name, 16, ring_edges(16), 1 / 3, vgg16_shapes(), 2, 1, 0.01, 10)
    if name == "lstm":
        return _mk(name, 16, torus_edges(4, 4), 1 / 5, lstm_shapes(), 4, 2, 0.01, 10)
    if name == "resnet50":
        return _mk(name, 64, torus_edges(8, 8), 1 / 5, resnet50_shapes(), 2, 2, 0.01, 100)
    raise KeyError(name)


NAMES = ("tiny", "resnet20", "vgg16_r1", "vgg16_r2", "lstm", "resnet50")
