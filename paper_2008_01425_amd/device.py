"""Device-memory plumbing around the binding: PyTorch is used only to allocate HBM buffers,
to copy layered numpy data in and out of the library's flat layouts, and for streams."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from .workloads import Workload


class GossipBuffers:
    """Context + the caller-owned device buffers of one PowerGossip problem."""

    def __init__(self, n_workers, edges, edge_w, shapes, rank, power_steps, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("GossipBuffers needs a GPU: the PowerGossip path has no CPU fallback")
        self.shapes = [(int(p), int(q)) for p, q in shapes]
        self.n, self.n_edges, self.L = int(n_workers), int(np.asarray(edge_w).size), len(self.shapes)
        self.ctx = B.pg_init(n_workers, edges, edge_w, [s[0] for s in self.shapes],
                             [s[1] for s in self.shapes], rank, power_steps)
        self.device = torch.device(device)
        self.N = B.pg_param_floats(self.ctx)
        self.x = [torch.zeros(self.N, dtype=torch.float32, device=self.device) for _ in range(self.n)]
        self.q = torch.zeros(max(1, B.pg_qstate_floats(self.ctx)), dtype=torch.float32, device=self.device)
        self.ws = torch.zeros(B.pg_workspace_bytes(self.ctx), dtype=torch.uint8, device=self.device)
        assert self.ws.data_ptr() % 256 == 0
        self.ptrs = [t.data_ptr() for t in self.x]
        self.ranks = [B.pg_layer_rank(self.ctx, l) for l in range(self.L)]
        B.pg_upload(self.ctx)

    @classmethod
    def from_workload(cls, wl: Workload, device="cuda:0", fill=True):
        gb = cls(wl.n_workers, wl.edges, wl.edge_w, wl.shapes, wl.rank, wl.power_steps, device)
        if fill:
            gb.fill_from_workload(wl)
        return gb

    def close(self):
        if self.ctx:
            torch.cuda.synchronize()
            B.pg_destroy(self.ctx)
            self.ctx = None

    # ---- host <-> device, layer by layer --------------------------------
    def _layer_view(self, buf: torch.Tensor, l: int) -> torch.Tensor:
        """The p x q matrix of layer l inside a worker buffer (rows pg_layer_stride floats apart)."""
        p, q = self.shapes[l]
        off, ld = B.pg_layer_offset(self.ctx, l), B.pg_layer_stride(self.ctx, l)
        return buf[off:off + p * ld].view(p, ld)[:, :q]

    def set_layer(self, i: int, l: int, a: np.ndarray):
        p, q = self.shapes[l]
        self._layer_view(self.x[i], l).copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).reshape(p, q)))

    def get_layer(self, i: int, l: int) -> np.ndarray:
        return self._layer_view(self.x[i], l).cpu().numpy()

    def set_q(self, e: int, l: int, a: np.ndarray):
        r, q = self.ranks[l], self.shapes[l][1]
        off = B.pg_q_offset(self.ctx, e, l)
        self.q[off:off + r * q].copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).reshape(-1)))

    def get_q(self, e: int, l: int) -> np.ndarray:
        r, q = self.ranks[l], self.shapes[l][1]
        off = B.pg_q_offset(self.ctx, e, l)
        return self.q[off:off + r * q].cpu().numpy().reshape(r, q)

    def get_phat(self, e: int, l: int) -> np.ndarray:
        r, p = self.ranks[l], self.shapes[l][0]
        off = B.pg_ws_phat_offset(self.ctx, e, l)
        return self.ws[off:off + 4 * r * p].view(torch.float32).cpu().numpy().reshape(r, p)

    def get_flags(self, e: int, l: int) -> np.ndarray:
        off = B.pg_ws_flag_offset(self.ctx, e, l)
        return self.ws[off:off + 4 * self.ranks[l]].view(torch.int32).cpu().numpy()

    def fill_from_workload(self, wl: Workload, layers: Optional[Sequence[int]] = None):
        """Fill every worker's parameters and every edge's projection state from the seeded
        generator (all layers, or only the listed ones; the others stay zero)."""
        ls = range(self.L) if layers is None else layers
        for l in ls:
            base = wl.base(l)
            for i in range(self.n):
                self.set_layer(i, l, wl.worker_layer(i, l, base))
            for e in range(self.n_edges):
                self.set_q(e, l, wl.q_init(e, l))

    def fill_from_arrays(self, X, Q, layers: Optional[Sequence[int]] = None):
        """Fill from host arrays X[i][j] (p, q) and Q[e][j] (r, q) holding the listed layers
        (default: all, in order)."""
        ls = list(range(self.L)) if layers is None else list(layers)
        for j, l in enumerate(ls):
            for i in range(self.n):
                self.set_layer(i, l, X[i][j])
            for e in range(self.n_edges):
                self.set_q(e, l, Q[e][j])

    # ---- the two entry points -------------------------------------------
    def round(self, stream: Optional[torch.cuda.Stream] = None):
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        B.pg_round(self.ctx, self.ptrs, self.q.data_ptr(), self.ws.data_ptr(), s.cuda_stream)

    def round_static(self, stream: Optional[torch.cuda.Stream] = None):
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        B.pg_round_static(self.ctx, self.ptrs, self.q.data_ptr(), s.cuda_stream)

    def alloc_grads(self):
        """Gradient buffers laid out like the parameter buffers (zero-filled)."""
        self.g = [torch.zeros(self.N, dtype=torch.float32, device=self.device) for _ in range(self.n)]
        self.gptrs = [t.data_ptr() for t in self.g]

    def set_grad_layer(self, i: int, l: int, a: np.ndarray):
        p, q = self.shapes[l]
        self._layer_view(self.g[i], l).copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).reshape(p, q)))

    def round_sgd(self, eta: float, stream: Optional[torch.cuda.Stream] = None):
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        B.pg_round_sgd(self.ctx, self.ptrs, self.gptrs, eta, self.q.data_ptr(), self.ws.data_ptr(), s.cuda_stream)

    def alloc_pstate(self):
        """The R^p half of Algorithm 2's alternating vector (zero-filled)."""
        self.pstate = torch.zeros(max(1, B.pg_pstate_floats(self.ctx)), dtype=torch.float32, device=self.device)

    def set_p(self, e: int, l: int, a: np.ndarray):
        r, p = self.ranks[l], self.shapes[l][0]
        off = B.pg_p_offset(self.ctx, e, l)
        self.pstate[off:off + r * p].copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).reshape(-1)))

    def get_p(self, e: int, l: int) -> np.ndarray:
        r, p = self.ranks[l], self.shapes[l][0]
        off = B.pg_p_offset(self.ctx, e, l)
        return self.pstate[off:off + r * p].cpu().numpy().reshape(r, p)

    def iterate(self, k_done: int, iterations: int, eta: Optional[float] = None,
                stream: Optional[torch.cuda.Stream] = None):
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        B.pg_iterate(self.ctx, self.ptrs, self.q.data_ptr(), self.pstate.data_ptr(), k_done, iterations,
                     None if eta is None else self.gptrs, 0.0 if eta is None else eta,
                     self.ws.data_ptr(), s.cuda_stream)

    def run(self, rounds: int, stream: Optional[torch.cuda.Stream] = None):
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        B.pg_run(self.ctx, self.ptrs, self.q.data_ptr(), self.ws.data_ptr(), s.cuda_stream, rounds)
