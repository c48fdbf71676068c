#!/usr/bin/env python3
"""The unstructured half of the paper's consensus experiment (Section 5, Figure 1, settings in
the appendix "Experimental settings": 8 workers on a ring, W_ij = 0.436 between neighbours,
each worker starts from a 100 x 100 standard-normal matrix), run on the GPU library:

    python -m paper_2008_01425_amd.consensus_experiment [--rounds 300] [--rank 1]

Prints the consensus error (1/n) sum_i |X_i - mean|_F^2 against bits sent per worker for
  * PowerGossip with the warm-started power iteration (pg_round, one power step = 2 iterations),
  * the same compressor with a fresh N(0,1) projection every round (random projections),
  * the literal one-iteration-per-round schedule (pg_iterate).
Every step of every variant runs in the library's kernels; this module only draws the seeded
inputs (`initial_matrices`, `projection_stream`) and reads the error back.  Uncompressed gossip
(a full-rank projector, rank 100 here) is beyond the library's 16 columns per edge and is not
part of this program; the Faces half of the figure needs a dataset and is not reproduced.
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import workloads as W
from .device import GossipBuffers


def consensus_error(gb: GossipBuffers) -> float:
    x = torch.stack([t.double() for t in gb.x])
    return float(((x - x.mean(0, keepdim=True)) ** 2).sum() / gb.n)


def initial_matrices(n: int, p: int, q: int, seed: int):
    """X_i ~ N(0, 1) entry-wise, one (p, q) float32 matrix per worker."""
    rng = np.random.default_rng([seed, 1])
    return [rng.standard_normal((p, q)).astype(np.float32) for _ in range(n)]


def projection_stream(n_edges: int, rank: int, q: int, seed: int):
    """Generator of projection states: every item is a list of n_edges (rank, q) float32 arrays,
    entry-wise N(0, 1) (the initialisation of Algorithm 2; drawn afresh for random projections)."""
    rng = np.random.default_rng([seed, 2])
    while True:
        yield [rng.standard_normal((rank, q)).astype(np.float32) for _ in range(n_edges)]


VARIANTS = ("power_iteration", "random_projection", "one_iteration")


def run(rounds: int = 300, rank: int = 1, n: int = 8, p: int = 100, q: int = 100, w: float = 0.436,
        seed: int = 0, every: int = 25):
    """{variant: [(round, bits sent per worker so far, consensus error)]}."""
    edges = W.ring_edges(n)
    ew = np.full((n,), w, dtype=np.float32)
    X0 = initial_matrices(n, p, q, seed)
    deg = 2
    out = {}
    for name in VARIANTS:
        gb = GossipBuffers(n, edges, ew, [(p, q)], rank, 1)
        r = gb.ranks[0]
        for i in range(n):
            gb.set_layer(i, 0, X0[i])
        states = projection_stream(n, r, q, seed)
        for e, a in enumerate(next(states)):
            gb.set_q(e, 0, a)
        if name == "one_iteration":
            gb.alloc_pstate()
        curve = []
        bits = 0
        for t in range(rounds + 1):
            if t % every == 0:
                curve.append((t, bits, consensus_error(gb)))
            if name == "power_iteration":
                gb.round()
                bits += deg * r * (p + q) * 32
            elif name == "random_projection":
                for e, a in enumerate(next(states)):
                    gb.set_q(e, 0, a)
                gb.round()
                bits += deg * r * (p + q) * 32
            else:
                gb.iterate(t, 1)
                bits += deg * r * (p if t % 2 == 0 else q) * 32
        gb.close()
        out[name] = curve
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rounds", type=int, default=300)
    ap.add_argument("--rank", type=int, default=1)
    args = ap.parse_args()
    res = run(args.rounds, args.rank)
    for name, curve in res.items():
        print(name)
        for t, bits, err in curve:
            print(f"  round {t:5d}  bits/worker {bits:12d}  consensus error {err:.6e}")


if __name__ == "__main__":
    main()
