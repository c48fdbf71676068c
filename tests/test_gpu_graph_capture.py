"""The calls that launch kernels only -- pg_run, pg_round and pg_round_static on a context that is
already uploaded and has seen its buffers -- recorded into a HIP graph and replayed: every replay
must give bit for bit what the same calls give when launched directly, also with other work of the
same context between the replays."""
import numpy as np
import pytest

from paper_2008_01425_amd import workloads as W

pytestmark = pytest.mark.gpu


def _workload():
    shapes = [(64, 144), (32, 288), (10, 64), (64, 1), (33, 50)]
    edges = W.ring_edges(6)
    return W.Workload("ring6_graph", 6, edges, np.full((len(edges),), 1 / 3, np.float32), shapes, 2, 1, 0.05, 10, 7)


def _state(gb):
    import torch
    torch.cuda.synchronize()
    return [x.clone() for x in gb.x], gb.q.clone()


def _restore(gb, state):
    for a, b in zip(gb.x, state[0]):
        a.copy_(b)
    gb.q.copy_(state[1])


def _same(gb, state):
    import torch
    torch.cuda.synchronize()
    return all(torch.equal(a, b) for a, b in zip(gb.x, state[0])) and torch.equal(gb.q, state[1])


@pytest.mark.parametrize("call", ["run", "round", "round_static"])
def test_replays_of_a_captured_call_equal_the_direct_call(call):
    import torch
    from paper_2008_01425_amd.device import GossipBuffers
    wl = _workload()
    gb = GossipBuffers.from_workload(wl)
    issue = {"run": lambda: gb.run(3), "round": gb.round, "round_static": gb.round_static}[call]
    start = _state(gb)
    issue()  # uploads the tables and caches the buffer addresses: nothing but launches from here on
    direct = _state(gb)
    assert not _same(gb, start)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    _restore(gb, start)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        issue()
    for replay in range(3):
        _restore(gb, start)
        graph.replay()
        assert _same(gb, direct), f"replay {replay} of pg_{call} differs from the direct call"
        # other work of the same context between the replays, and a synchronisation
        gb.round()
        gb.run(2)
        torch.cuda.synchronize()
    gb.close()
