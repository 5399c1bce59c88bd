"""The entry point that allocates nothing (mixgcn_aggregate_static) against mixgcn_aggregate and
the oracle: same kernels, scratch in the library's fixed device array."""
import numpy as np
import pytest

import graphgen as gg
import oracle
from parity import RTOL_BF16, RTOL_F32, assert_close, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _graph(mg, src, dst, n):
    g = mg.build_csr(dev(src.view(np.int32)), dev(dst.view(np.int32)), n,
                     mg.SYMMETRIZE | mg.ADD_SELF_LOOPS)
    mg.normalize(g)
    return g


def test_static_scratch_aggregation_two_calls_in_a_row():
    """Two calls in a row on the shared array, the second on a smaller input (whose row pieces
    land in slots the first call has left full), each bit-identical to mixgcn_aggregate and
    within tolerance of the oracle; then column slices, a row range, the transpose and bf16."""
    import paper_2501_01951_amd as mg

    mg.load_library()
    big = gg.config_graph("c2", scale_override=16)
    small = gg.config_graph("c2", scale_override=12)
    graphs = [(_graph(mg, *c), oracle.transpose(oracle.normalize(oracle.build_csr(*c))))
              for c in (big, small)]
    for (g, og), f in zip(graphs, (256, 100)):
        say(f"aggregate_static n={og.n} nnz={og.nnz} f={f}")
        ld = (f + 3) // 4 * 4
        h = gg.normal(41, f, og.n, f, ld=ld)
        hd = dev(h)
        z_ref = torch.full((og.n, ld), 5.0, device="cuda")
        z = torch.full((og.n, ld), 5.0, device="cuda")
        mg.aggregate(g, hd, z_ref, col_end=f)
        mg.aggregate_static(g, hd, z, col_end=f)
        torch.cuda.synchronize()
        assert torch.equal(z, z_ref)
        assert_close(z.cpu().numpy()[:, :f], oracle.spmm(og, h[:, :f].astype(np.float64)), RTOL_F32,
                     f"static f={f}")
    # back to the larger graph: slices, a ragged row range, the transposed matrix, bf16 storage
    g, og = graphs[0]
    h = gg.normal(42, 1, og.n, 512)
    hd = dev(h)
    z_ref = torch.zeros(og.n, 512, device="cuda")
    z = torch.zeros(og.n, 512, device="cuda")
    for (c0, c1, r0, r1, tr) in [(0, 512, 0, og.n, False), (64, 192, 1000, 50001, False),
                                 (256, 512, 0, og.n, True), (8, 12, og.n - 1, og.n, False)]:
        say(f"aggregate_static cols [{c0},{c1}) rows [{r0},{r1}) transpose={tr}")
        z.fill_(-1.0)
        z_ref.fill_(-1.0)
        mg.aggregate(g, hd, z_ref, c0, c1, r0, r1, transpose=tr)
        mg.aggregate_static(g, hd, z, c0, c1, r0, r1, transpose=tr)
        torch.cuda.synchronize()
        assert torch.equal(z, z_ref)
    ref = oracle.spmm(og, h.astype(np.float64))
    mg.aggregate_static(g, hd, z)
    assert_close(z.cpu().numpy(), ref, RTOL_F32, "static 512 columns")
    hb = hd.to(torch.bfloat16)
    zb_ref = torch.zeros(og.n, 512, device="cuda", dtype=torch.bfloat16)
    zb = torch.zeros(og.n, 512, device="cuda", dtype=torch.bfloat16)
    mg.aggregate(g, hb, zb_ref)
    mg.aggregate_static(g, hb, zb)
    torch.cuda.synchronize()
    assert torch.equal(zb.view(torch.int16), zb_ref.view(torch.int16))
    assert_close(zb.float().cpu().numpy(), oracle.spmm(og, hb.float().cpu().numpy().astype(np.float64)),
                 RTOL_BF16, "static bf16")
    for g, _ in graphs:
        g.free()


def test_static_scratch_rejects_what_does_not_fit():
    """More stored entries than the fixed array serves at 256 columns: refused with a message
    before anything runs (the output is untouched); the same graph at 128 columns, which needs
    half the scratch, goes through and equals mixgcn_aggregate."""
    import paper_2501_01951_amd as mg

    lib = mg.load_library()
    n = 1 << 21
    src, dst = gg.rmat_edges(77, 21, 40_000_000)
    g = _graph(mg, src, dst, n)
    nnz = g.nnz
    say(f"aggregate_static limit: nnz={nnz}")
    limit = 64 << 20
    assert lib.mixgcn_aggregate_scratch_need(mg.F32, 256, 0, nnz) > limit
    assert lib.mixgcn_aggregate_scratch_need(mg.F32, 128, 0, nnz) <= limit
    hd = torch.randn(n, 256, device="cuda")
    z = torch.full((n, 256), 3.0, device="cuda")
    with pytest.raises(mg.MixGCNError, match="scratch"):
        mg.aggregate_static(g, hd, z)
    torch.cuda.synchronize()
    assert bool((z == 3.0).all())
    z_ref = torch.full((n, 256), 3.0, device="cuda")
    mg.aggregate_static(g, hd, z, col_end=128)
    mg.aggregate(g, hd, z_ref, col_end=128)
    torch.cuda.synchronize()
    assert torch.equal(z, z_ref)
    g.free()


def test_static_scratch_degenerate_calls():
    """Empty ranges are no-ops, a one-node graph and an edgeless graph give A_hat = I, and bad
    arguments are refused like mixgcn_aggregate refuses them."""
    import paper_2501_01951_amd as mg

    mg.load_library()
    src, dst, n = gg.config_graph("c2", scale_override=10)
    g = _graph(mg, src, dst, n)
    h = torch.randn(n, 24, device="cuda")
    z = torch.full((n, 24), 4.0, device="cuda")
    mg.aggregate_static(g, h, z, row_begin=7, row_end=7)
    mg.aggregate_static(g, h, z, col_begin=5, col_end=5)
    torch.cuda.synchronize()
    assert bool((z == 4.0).all())
    with pytest.raises(mg.MixGCNError):
        mg.aggregate_static(g, h, h)  # H and Z overlap
    with pytest.raises(mg.MixGCNError):
        mg.aggregate_static(g, h, z, row_end=n + 1)
    g.free()
    for n1, s1, d1 in ((1, np.zeros(0, np.uint32), np.zeros(0, np.uint32)),
                       (9, np.zeros(0, np.uint32), np.zeros(0, np.uint32))):
        g1 = _graph(mg, s1, d1, n1)
        x = torch.randn(n1, 7, device="cuda")
        xp = torch.zeros(n1, 8, device="cuda")
        xp[:, :7] = x
        out = torch.zeros(n1, 8, device="cuda")
        mg.aggregate_static(g1, xp[:, :7], out[:, :7])
        torch.cuda.synchronize()
        assert torch.equal(out[:, :7], x) and bool((out[:, 7] == 0).all())
        g1.free()
