"""Host-side checks of the C-ABI library: it loads without a GPU, exports every function that
include/mixgcn.h declares, and the Python structs match the header's layout."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mixgcn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mixgcn_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_six_calls():
    names = declared_functions()
    for f in ("mixgcn_build_csr", "mixgcn_normalize", "mixgcn_aggregate", "mixgcn_update",
              "mixgcn_layer_fwd", "mixgcn_layer_bwd"):
        assert f in names


def test_library_exports_every_declared_symbol():
    import paper_2501_01951_amd as m

    lib = m.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in mixgcn.h but not exported"
    assert lib.mixgcn_version() == 100
    assert lib.mixgcn_strerror(-1) == b"invalid argument"
    assert lib.mixgcn_strerror(0) == b"ok"


def test_struct_layouts_match_header():
    from paper_2501_01951_amd.binding import LayerDesc, _GraphView

    # mixgcn_layer_desc: 2 x int32, 4 x int64, 4 x int32
    assert ctypes.sizeof(LayerDesc) == 2 * 4 + 4 * 8 + 4 * 4
    assert LayerDesc.ld_h.offset == 8 and LayerDesc.ld_w.offset == 32 and LayerDesc.dtype.offset == 40
    # mixgcn_graph_view: 2 x uint32, int64, 8 pointers
    assert ctypes.sizeof(_GraphView) == 8 + 8 + 8 * 8
    assert _GraphView.rowptr.offset == 16


def test_argument_errors_need_no_gpu():
    """Calls that fail validation before touching the device."""
    import paper_2501_01951_amd as m

    lib = m.load_library()
    out = ctypes.c_void_p()
    assert lib.mixgcn_build_csr(None, None, 0, 0, 3, None, ctypes.byref(out)) == -1  # n_nodes == 0
    assert b"n_nodes" in lib.mixgcn_last_error()
    assert lib.mixgcn_build_csr(None, None, 5, 10, 3, None, ctypes.byref(out)) == -1  # null edges
    assert lib.mixgcn_build_csr(None, None, 0, 10, 1 << 9, None, ctypes.byref(out)) == -1  # flag
    assert lib.mixgcn_normalize(None, 0, None) == -1
    assert lib.mixgcn_graph_reserve_streams(None, 1) == -1
    assert lib.mixgcn_graph_free(None) == 0
    assert lib.mixgcn_update(9, 0, None, 0, None, 0, None, 0, 1, 1, 1, None, 0, 0.0, None) == -1
    assert lib.mixgcn_update(0, 0, None, 4, None, 4, None, 4, 1, 4, 4, None, 0, 0.0, None) == -1
    assert lib.mixgcn_set_update_arith(2) == -1 and b"set_update_arith" in lib.mixgcn_last_error()
    assert lib.mixgcn_set_update_arith(m.ARITH_BF16X3) == 0
    assert lib.mixgcn_set_update_arith(m.ARITH_FP32) == 0


# ---- sizing rule of the aggregation scratch ---------------------------------------------------

@pytest.mark.parametrize("nnz", [1, 255, 4096, 45_056, 1_000_003, 32_450_196, 3_310_441_142])
def test_aggregation_scratch_bound_covers_every_call(nnz):
    """mixgcn_aggregate_scratch_bytes(nnz), the size fixed when a graph is normalised, is at
    least what any call on that graph uses: every column count, both storage types, entry
    ranges of every length and alignment (the span length, and with it the number of row
    pieces per entry, depends on the range)."""
    import numpy as np
    import paper_2501_01951_amd as m

    lib = m.load_library()
    bound = lib.mixgcn_aggregate_scratch_bytes(nnz)
    assert bound > 0
    rng = np.random.default_rng(nnz)
    widths = [1, 3, 4, 8, 16, 17, 32, 47, 64, 100, 128, 129, 172, 255, 256, 257, 300, 512, 1024]
    lengths = {nnz, max(1, nnz // 2), min(nnz, 256), min(nnz, 257), min(nnz, 8192 * 256),
               min(nnz, 8192 * 2048), min(nnz, 8192 * 2048 - 1), min(nnz, 8191 * 4096 + 1)}
    lengths |= {int(x) for x in np.minimum(nnz, rng.integers(1, 1 << 34, size=40) >>
                                           rng.integers(0, 34, size=40)) if x > 0}
    worst = 0
    for dtype in (m.F32, m.BF16):
        for w in widths:
            for ln in sorted(lengths):
                for e0 in {0, nnz - ln, int(rng.integers(0, nnz - ln + 1))}:
                    need = lib.mixgcn_aggregate_scratch_need(dtype, w, e0, e0 + ln)
                    assert 0 <= need <= bound, (dtype, w, e0, ln, need, bound)
                    worst = max(worst, need)
    # and the bound is not wildly generous: at most twice the largest need seen
    assert bound <= 2 * worst + 4096, (bound, worst)
    assert lib.mixgcn_aggregate_scratch_need(7, 4, 0, 1) == -1
    assert lib.mixgcn_aggregate_scratch_need(m.F32, 4, 5, 1) == -1
    assert lib.mixgcn_aggregate_scratch_bytes(-1) == 0


def test_aggregation_scratch_bound_with_whole_row_gathers():
    """The measurement aid that gathers whole rows uses shorter spans (one entry per gather
    instruction at 256 fp32 columns), so a graph normalised with it on gets a larger scratch:
    the bound follows the mode, and still covers every call."""
    import paper_2501_01951_amd as m

    lib = m.load_library()
    nnz = 5_000_000
    plain = lib.mixgcn_aggregate_scratch_bytes(nnz)
    assert lib.mixgcn_set_aggregate_whole_rows(1) == 0
    try:
        bound = lib.mixgcn_aggregate_scratch_bytes(nnz)
        assert bound > plain
        for dtype in (m.F32, m.BF16):
            for w in (1, 16, 47, 100, 128, 256, 300):
                for e0, e1 in ((0, nnz), (12345, 12345 + 70_000), (nnz - 300, nnz), (1000, 1001)):
                    need = lib.mixgcn_aggregate_scratch_need(dtype, w, e0, e1)
                    assert 0 <= need <= bound, (dtype, w, e0, e1, need, bound)
    finally:
        assert lib.mixgcn_set_aggregate_whole_rows(0) == 0
    assert lib.mixgcn_aggregate_scratch_bytes(nnz) == plain


# ---- host arithmetic of the cross-layer pipeline (Sec. 3.2.2) -------------------------------

def _windows(m, n, s, b):
    return [m.pipeline_window(n, s, b, c) for c in range(s)]


@pytest.mark.parametrize("n,s,b", [(1000, 8, 130), (1000, 8, 0), (100, 20, 7), (5000, 3, 4999),
                                   (1 << 20, 5, 549_127), (77, 1, 5), (4096, 32, 1)])
def test_pipeline_window_covers_exactly_the_rows_within_b(n, s, b):
    """The batches tile [0, n) in order; every row within b of a batch lies in a batch of
    [first, last], and first / last are not wider than needed."""
    import numpy as np
    import paper_2501_01951_amd as m

    w = _windows(m, n, s, b)
    assert w[0][0] == 0 and w[-1][1] == n
    for c in range(s - 1):
        assert w[c][1] == w[c + 1][0] and w[c][0] <= w[c][1]
    batch_of = np.empty(n, dtype=np.int64)
    for c, (r0, r1, _, _) in enumerate(w):
        batch_of[r0:r1] = c
    for c, (r0, r1, first, last) in enumerate(w):
        assert first <= c <= last
        if r1 == r0:
            continue
        rows = np.arange(max(0, r0 - b), min(n, r1 + b))
        used = batch_of[rows]
        assert used.min() >= first and used.max() <= last
        if w[first][1] > w[first][0]:
            assert used.min() == first
        if w[last][1] > w[last][0]:
            assert used.max() == last


def test_pipeline_window_on_a_graph_holds_every_neighbor():
    """With b = the graph's bandwidth, every stored neighbor of a row of batch c lies in a batch
    of [first, last] (the rows an aggregation of that batch gathers)."""
    import numpy as np
    import oracle
    import graphgen as gg
    import paper_2501_01951_amd as m

    n = 3000
    s0, d0 = gg.ring_lattice_edges(n, 6)
    perm = np.random.default_rng(1).permutation(n).astype(np.uint32)
    g = oracle.build_csr(perm[s0], perm[d0], n)
    pos = oracle.rcm(g)
    g2 = oracle.build_csr(pos[perm[s0]], pos[perm[d0]], n)
    b = oracle.bandwidth(g2)
    assert b < 20
    s = 9
    w = _windows(m, n, s, b)
    rowptr, col = g2.rowptr, g2.col.astype(np.int64)
    for c, (r0, r1, first, last) in enumerate(w):
        nb = col[rowptr[r0]:rowptr[r1]]
        assert nb.min() >= w[first][0] and nb.max() < w[last][1]
    # and one less than the bandwidth is not enough for some batch
    short = _windows(m, n, s, 0)
    assert any(col[rowptr[r0]:rowptr[r1]].max() >= short[l][1] or
               col[rowptr[r0]:rowptr[r1]].min() < short[f][0] for (r0, r1, f, l) in short)


@pytest.mark.parametrize("n,b", [(128 * 3 * 7 * 40, 1000), (35840, 26880), (10752, 5376),
                                 (128 * 360, 25)])
def test_proposition_3_5_is_the_point_where_the_first_batch_stops_waiting_for_the_last(n, b):
    """With s = ceil(2n / (n - b)) batches of equal size the first batch of an aggregation does
    not read the last batch of its input; with one batch fewer it does (batch sizes chosen so
    that n / s is a whole number of 128-row tiles for both)."""
    import paper_2501_01951_amd as m

    s = m.pipeline_stages(n, b)
    assert s >= 3 and n % (128 * s) == 0 and n % (128 * (s - 1)) == 0
    _, _, _, last = m.pipeline_window(n, s, b, 0)
    assert last <= s - 2
    _, _, _, last = m.pipeline_window(n, s - 1, b, 0)
    assert last == s - 2


def test_pipelined_calls_reject_bad_arguments_without_a_gpu():
    import paper_2501_01951_amd as m

    lib = m.load_library()
    assert lib.mixgcn_pipeline_window(10, 0, 1, 0, None, None, None, None) == -1
    assert lib.mixgcn_pipeline_window(10, 2, 1, 2, None, None, None, None) == -1
    assert lib.mixgcn_pipeline_window(10, 2, -1, 0, None, None, None, None) == -1
    assert lib.mixgcn_forward_pipelined(None, 0, None, None, None, None, None, 0, None) == -1
    assert lib.mixgcn_backward_pipelined(None, 1, None, None, None, None, None, None, None, None, 0,
                                         None) == -1


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus 2 exits with a message (before touching torch)."""
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


# ---- host logic around the library -------------------------------------------------------------

def test_row_pitch_rule_of_the_step_helper():
    """Feature buffers of the step helper: rows longer than a 128-byte line get a pitch of an odd
    number of lines (spreads a column slice over the L2 channels), shorter rows a power-of-two
    pitch (a gathered row never straddles two lines); every pitch is a whole number of 16-byte
    groups, as the ABI asks."""
    import torch
    from paper_2501_01951_amd.model import padded_rows

    for dtype, es in ((torch.float32, 4), (torch.bfloat16, 2)):
        for f in (1, 3, 4, 8, 16, 17, 31, 32, 47, 64, 65, 100, 128, 172, 256, 300, 1024):
            t = padded_rows(5, f, dtype, "cpu")
            assert t.shape == (5, f) and t.stride(1) == 1
            pitch = t.stride(0) * es
            assert pitch % 16 == 0 and pitch >= f * es
            if f * es <= 128:
                assert pitch & (pitch - 1) == 0 and pitch < 2 * max(16, f * es)
            else:
                lines = pitch // 128
                assert pitch % 128 == 0 and lines % 2 == 1 and lines <= (f * es + 127) // 128 + 1


def test_roofline_block_of_the_benchmark_line():
    """bench.py's roofline block: achieved = algorithmic bytes / launch time, frac against the
    published 8 TB/s, the counter traffic labelled with its source file (or null), per launch."""
    import sys

    sys.path.insert(0, ROOT)
    import bench

    kinds = {"agg_g64": {"total_ms": 28.0, "launches": 10, "avg_ms": 2.8},
             "agg_g4": {"total_ms": 3.7, "launches": 10, "avg_ms": 0.37},
             "update_fwd": {"total_ms": 7.0, "launches": 10, "avg_ms": 0.7}}
    nnz, n = 32_450_196, 1 << 20
    r = bench.aggregation_roofline("c2", kinds, nnz, n, 4)
    algo = 8.0 * nnz + 2.0 * n * 256 * 4 + 8.0 * n
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["algorithmic_bytes_per_launch"] - algo) < 1 and abs(r["achieved"] - algo / 2.8e-3 / 1e9) < 1e-6
    assert abs(r["frac"] - r["achieved"] / 8000.0) < 1e-12
    assert r["traffic"] and "profiles/c2_aggregate_pmc.txt" in r["traffic_source"]
    assert abs(r["counter_traffic_frac"] - r["traffic"] / 2.8e-3 / 1e9 / 8000.0) < 1e-12
    assert r["no_reuse_bytes_per_launch"] == nnz * (8.0 + 1024) + n * 1024
    # a configuration without a committed counter summary reports null, never a guess
    r1 = bench.aggregation_roofline("c1", kinds, nnz, n, 4)
    assert r1["traffic"] is None and r1["traffic_source"] is None and "counter_traffic_frac" not in r1
    for cfg, width in bench.TRAFFIC_FILES:
        assert os.path.exists(os.path.join(ROOT, "profiles", bench.TRAFFIC_FILES[(cfg, width)]))
        t, src = bench.measured_traffic(cfg, width)
        assert t and t > 0 and src
