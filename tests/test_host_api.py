"""Host-side logic of the C-ABI library, without a GPU: the library loads, exports every
symbol the header declares, validates its inputs and reports consistent layouts."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2008_01425_amd import binding as B
from paper_2008_01425_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _init(n, edges, w, shapes, rank=1, steps=1):
    edges = np.asarray(edges, dtype=np.int32).reshape(-1, 2)
    ew = np.full((len(edges),), w, dtype=np.float32) if np.isscalar(w) else np.asarray(w, np.float32)
    return B.pg_init(n, edges, ew, [s[0] for s in shapes], [s[1] for s in shapes], rank, steps)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "powergossip.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pg_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    raw = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name


def test_strerror_covers_all_codes():
    texts = {B.pg_strerror(c) for c in (0, -1, -2, -3, -4, -5, -6)}
    assert len(texts) == 7 and all(texts)
    assert "unknown" in B.pg_strerror(-99)


@pytest.mark.parametrize("edges,code", [
    ([[0, 0]], B.PG_ERR_TOPOLOGY),            # self-loop
    ([[0, 3]], B.PG_ERR_TOPOLOGY),            # out of range
    ([[-1, 1]], B.PG_ERR_TOPOLOGY),
    ([[0, 1], [1, 0]], B.PG_ERR_TOPOLOGY),    # duplicate, reversed
    ([[0, 1], [0, 1]], B.PG_ERR_TOPOLOGY),
])
def test_bad_topologies_are_rejected(edges, code):
    with pytest.raises(B.PGError) as e:
        _init(3, edges, 0.2, [(4, 4)])
    assert e.value.status == code


def test_bad_arguments_are_rejected():
    ok_edges = [[0, 1], [1, 2]]
    cases = [
        (lambda: _init(3, ok_edges, 0.2, [(0, 4)]), B.PG_ERR_SHAPE),
        (lambda: _init(3, ok_edges, 0.2, [(4, -1)]), B.PG_ERR_SHAPE),
        (lambda: _init(3, ok_edges, 0.2, [(4, 4)], rank=0), B.PG_ERR_ARG),
        (lambda: _init(3, ok_edges, 0.2, [(4, 4)], steps=0), B.PG_ERR_ARG),
        (lambda: _init(0, [], 0.2, [(4, 4)]), B.PG_ERR_ARG),
        (lambda: _init(3, ok_edges, -0.1, [(4, 4)]), B.PG_ERR_ARG),
        (lambda: _init(3, ok_edges, float("nan"), [(4, 4)]), B.PG_ERR_ARG),
        (lambda: _init(3, ok_edges, 0.6, [(4, 4)]), B.PG_ERR_ARG),      # worker 1: 1.2 > 1
        (lambda: _init(3, ok_edges, 0.2, [(64, 64)], rank=17), B.PG_ERR_ARG),  # one edge's columns exceed a pass
    ]
    for fn, code in cases:
        with pytest.raises(B.PGError) as e:
            fn()
        assert e.value.status == code
    assert B.lib.pg_init(None, 1, 0, None, None, 1, None, None, 1, 1) == B.PG_ERR_ARG
    assert B.lib.pg_destroy(None) == B.PG_ERR_ARG
    assert B.lib.pg_round(None, None, None, None, None) == B.PG_ERR_ARG
    assert B.lib.pg_round_static(None, None, None, None) == B.PG_ERR_ARG
    # the static-workspace round never uploads (that allocates): a context that has not been
    # through pg_upload is refused before any HIP call
    ctx = _init(3, ok_edges, 0.2, [(4, 4)])
    assert B.lib.pg_round_static(ctx, None, None, None) == B.PG_ERR_ARG
    B.pg_destroy(ctx)


def test_layouts_are_aligned_disjoint_and_complete():
    wl = W.get("resnet20")
    ctx = _init(wl.n_workers, wl.edges, wl.edge_w, wl.shapes, rank=2, steps=1)
    L, E = len(wl.shapes), wl.n_edges
    spans = []
    for l, (p, q) in enumerate(wl.shapes):
        off, ld = B.pg_layer_offset(ctx, l), B.pg_layer_stride(ctx, l)
        assert off % 32 == 0 and ld == q          # a ring at rank 2: 4 stacked columns, no row padding
        assert B.pg_layer_rank(ctx, l) == min(2, p, q)
        spans.append((off, off + p * ld))
    spans.sort()
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
    assert spans[-1][1] <= B.pg_param_floats(ctx) < spans[-1][1] + 32
    qsp = []
    for e in range(E):
        for l, (p, q) in enumerate(wl.shapes):
            off = B.pg_q_offset(ctx, e, l)
            assert off % 4 == 0
            qsp.append((off, off + q * min(2, p, q)))
    qsp.sort()
    assert all(a[1] <= b[0] for a, b in zip(qsp, qsp[1:]))
    assert qsp[-1][1] <= B.pg_qstate_floats(ctx)
    ws = B.pg_workspace_bytes(ctx)
    assert ws % 256 == 0 and ws > 0
    seen = []
    for e in range(E):
        for l, (p, q) in enumerate(wl.shapes):
            r = min(2, p, q)
            po, fo = B.pg_ws_phat_offset(ctx, e, l), B.pg_ws_flag_offset(ctx, e, l)
            assert po % 4 == 0 and po + 4 * r * p <= ws and fo + 4 * r <= ws
            seen.append((po, po + 4 * r * p))
            seen.append((fo, fo + 4 * r))
    seen.sort()
    assert all(a[1] <= b[0] for a, b in zip(seen, seen[1:]))
    # out-of-range queries
    assert B.pg_layer_offset(ctx, L) == ctypes.c_size_t(-1).value
    assert B.pg_q_offset(ctx, E, 0) == ctypes.c_size_t(-1).value
    assert B.pg_layer_rank(ctx, -1) == -1
    B.pg_destroy(ctx)


@pytest.mark.parametrize("name,N,mats", [("tiny", 2576, 2), ("resnet20", 269722, 20),
                                         ("vgg16_r1", 14715584, 14), ("lstm", 28390700, 5),
                                         ("resnet50", 25557032, 54)])
def test_workload_shapes_and_byte_accounting(name, N, mats):
    wl = W.get(name)
    assert wl.params_per_worker == N
    assert sum(1 for p, q in wl.shapes if q > 1) == mats
    ctx = _init(wl.n_workers, wl.edges, wl.edge_w, wl.shapes, wl.rank, wl.power_steps)
    s = wl.power_steps
    assert B.pg_round_bytes(ctx, False) == 4.0 * wl.n_workers * N * (2 * s + 2)
    assert B.pg_round_bytes(ctx, True) == 4.0 * wl.n_workers * N * (2 * s + 1)
    assert B.pg_message_floats(ctx) == sum(min(wl.rank, p, q) * (p + q) for p, q in wl.shapes)
    B.pg_destroy(ctx)


def test_rows_are_padded_to_whole_lines_only_where_wavefronts_share_rows():
    """8 or more stacked columns (here: 4 x 4 torus at rank 4, and at rank 2): rows of layers with
    at least 64 columns start on 128-byte boundaries; elsewhere the stride is the row length."""
    wl = W.get("lstm")
    ctx = _init(wl.n_workers, wl.edges, wl.edge_w, [(33278, 650), (2600, 650), (40, 63), (100, 64), (7, 1)], 4, 2)
    assert [B.pg_layer_stride(ctx, l) for l in range(5)] == [672, 672, 63, 64, 1]
    end = 0
    for l, (p, q) in enumerate([(33278, 650), (2600, 650), (40, 63), (100, 64), (7, 1)]):
        off = B.pg_layer_offset(ctx, l)
        assert off % 32 == 0 and off >= end
        end = off + p * B.pg_layer_stride(ctx, l)
    assert end <= B.pg_param_floats(ctx)
    assert B.pg_layer_stride(ctx, 5) == ctypes.c_size_t(-1).value
    B.pg_destroy(ctx)
    ctx = _init(5, W.ring_edges(5), 1 / 3, [(2600, 650)], 4, 1)     # 8 stacked columns
    assert B.pg_layer_stride(ctx, 0) == 672
    B.pg_destroy(ctx)
    ctx = _init(5, W.ring_edges(5), 1 / 3, [(2600, 650)], 2, 1)     # 4 stacked columns: one wavefront per row group
    assert B.pg_layer_stride(ctx, 0) == 650
    B.pg_destroy(ctx)


def test_message_floats_reproduce_the_papers_compression_column():
    """One power step sends a length-p and a length-q vector per matrix (two of the paper's
    iterations): p*q / (message/2) is the printed per-tensor ratio."""
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "compression_ratios.txt"))
            if l.strip() and not l.startswith("#")]
    for p, q, printed in [(int(a), int(b), int(c)) for a, b, c in rows]:
        ctx = _init(2, [[0, 1]], 0.5, [(p, q)])
        assert round(p * q / (B.pg_message_floats(ctx) / 2)) == printed
        B.pg_destroy(ctx)


def test_topology_builders():
    assert W.ring_edges(4).tolist() == [[0, 1], [1, 2], [2, 3], [3, 0]]
    t = W.torus_edges(4, 4)
    assert t.shape == (32, 2)
    deg = np.bincount(t.reshape(-1), minlength=16)
    assert (deg == 4).all()
    assert len({tuple(sorted(e)) for e in t.tolist()}) == 32


def test_seeded_blocks_are_reproducible_and_independent():
    wl = W.get("tiny")
    a = wl.worker_layer(2, 1)
    assert np.array_equal(a, W.get("tiny").worker_layer(2, 1))
    assert not np.array_equal(a, wl.worker_layer(3, 1))
    d = (wl.worker_layer(0, 0).astype(np.float64) - wl.base(0))
    assert abs(d.std() - 0.1) < 0.01
    q = wl.q_init(1, 0)
    assert q.shape == (1, 32) and abs(q.std() - 1.0) < 0.3


def test_planted_spectrum_gives_every_edge_the_prescribed_singular_values():
    """Workload.spectrum: worker i adds (i + 1) * sum_k sigma_k u_k v_k^T with shared orthonormal
    directions, so the difference of workers a and b has singular values |a - b| * sigma_k above
    the noise floor, in the planted ratios on every edge."""
    spectrum = (200.0, 2.0, 1.0, 0.5)
    wl = W.Workload("planted", 5, W.ring_edges(5), np.full((5,), 0.05, np.float32), [(60, 80), (33, 1)],
                    4, 1, 1e-6, 10, 11, spectrum)
    X = wl.all_params()
    for a, b in ((0, 1), (3, 4), (4, 0)):
        sv = np.linalg.svd(X[a][0].astype(np.float64) - X[b][0].astype(np.float64), compute_uv=False)
        assert np.allclose(sv[:4], abs(a - b) * np.array(spectrum), rtol=1e-3)
        assert sv[4] < 1e-3 * sv[3]
    assert X[0][1].shape == (33, 1) and np.array_equal(X[0][0], wl.worker_layer(0, 0))


def test_one_hip_runtime_whichever_of_library_and_torch_loads_first():
    """The library must share torch's HIP runtime also when it is loaded before torch (host-only
    tests collected ahead of GPU tests do exactly that); two runtimes in one process leave the
    second without a device."""
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2008_01425_amd import binding\n"
            "import torch\n"
            "paths = {l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l}\n"
            "print(len(paths))\n" % ROOT)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr[-2000:]
    assert out.stdout.strip().splitlines()[-1] == "1"


def test_plan_with_mixed_degrees_in_one_layer():
    """Workers of degree 3, 2, 1 and 0 at rank 4: one layer then holds workers with 12, 8 and 4
    stacked columns (different kernel families share the layer's segment geometry) and one
    without any."""
    edges = [[0, 1], [2, 0], [0, 3], [3, 1]]
    shapes = [(48, 36), (17, 1), (20, 64), (300, 650)]
    ctx = _init(5, edges, [0.3, 0.2, 0.25, 0.4], shapes, rank=4, steps=2)
    assert B.pg_message_floats(ctx) == sum(min(4, p, q) * (p + q) for p, q in shapes)
    assert B.pg_workspace_bytes(ctx) > 0
    B.pg_destroy(ctx)


def test_planner_tiles_cover_every_matrix_exactly_once(tmp_path):
    """tests/plan_cover.cpp links the host planner alone (no HIP) and checks, for the benchmark
    shapes, odd shapes and mixed degrees, in each kernel-family setting: row tiles x segments and
    column tiles x row blocks partition every matrix, tiles respect their kernels' limits, partial
    sums fit the workspace."""
    import subprocess
    exe = str(tmp_path / "plan_cover")
    src = [os.path.join(ROOT, "tests", "plan_cover.cpp"),
           os.path.join(ROOT, "paper_2008_01425_amd", "csrc", "pg_plan.cpp")]
    build = subprocess.run(["g++", "-O1", "-std=c++17", "-o", exe] + src, capture_output=True, text=True, timeout=300)
    assert build.returncode == 0, build.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-3000:]
    assert run.stdout.count("ok ") == 45 and "FAIL" not in run.stdout


SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def _run_sanitized(cmd, exe):
    import subprocess
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)      # the sanitizer runtime must come first in the link order
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-3000:])
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
    return run.stdout


def test_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The host planner (every table the kernels index with) built with ASan + UBSan and run over
    the same problems as the cover check: no out-of-bounds write, overflow or leak."""
    exe = str(tmp_path / "plan_cover_san")
    src = [os.path.join(ROOT, "tests", "plan_cover.cpp"),
           os.path.join(ROOT, "paper_2008_01425_amd", "csrc", "pg_plan.cpp")]
    out = _run_sanitized(["g++", "-O1", "-std=c++17"] + SAN + ["-o", exe] + src, exe)
    assert "FAIL" not in out and out.count("ok ") == 45


@pytest.mark.parametrize("define", [[], ["-DPGO_ALL_DOUBLE"]])
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path, define):
    """Both builds of the CPU oracle, all three entry points, on odd little problems."""
    exe = str(tmp_path / "oracle_san")
    src = os.path.join(ROOT, "tests", "oracle_sanitize.c")
    out = _run_sanitized(["gcc", "-O1", "-std=c11", "-ffp-contract=off"] + SAN + define + ["-o", exe, src, "-lm"], exe)
    assert "oracle sanitize ok" in out


def test_profile_summaries_classify_every_pass_kernel():
    """The rocprofv3 summariser maps kernel names to the kinds pg_profile_collect reports; the
    committed traffic summaries are read back by bench.py under those kinds."""
    from paper_2008_01425_amd.rocprof_summary import kernel_kind
    assert kernel_kind("pg::row_kernel<2, 8, 1, true, true, false>") == "update_sweep_p"
    assert kernel_kind("pg::row_kernel<2, 4, 1, false, true, false>") == "sweep_p"
    assert kernel_kind("pg::row_wide_kernel<4, 8, 4, true, false, false>") == "update"
    assert kernel_kind("pg::mrow_kernel<2, 4, 2, 1, true, false, true>") == "update_sgd"
    assert kernel_kind("pg::vec_row_kernel<4, true, true, false>") == "update_sweep_p"
    assert kernel_kind("pg::vec_row_kernel<4, false, true, false>") == "sweep_p"
    assert kernel_kind("pg::col_kernel<0, 2, 8>") == "sweep_q"
    assert kernel_kind("pg::mcol_kernel<4, 2>") == "sweep_q"
    assert kernel_kind("pg::vec_col_kernel<4>") == "sweep_q"
    assert kernel_kind("pg::comb_kernel") is None
    assert kernel_kind("pg::orth_gram_kernel<256, 2>") is None
    for wl in ("vgg16_r1", "vgg16_r2", "lstm", "resnet50"):
        path = os.path.join(ROOT, "profiles", f"{wl}_traffic_counters.txt")
        kinds = {line.split()[1] for line in open(path) if line.startswith("traffic ")}
        assert kinds == {"sweep_p", "sweep_q", "update", "update_sweep_p"}, (wl, kinds)
