"""Randomised parity sweeps (fixed seeds): many small cases with shapes, leading dimensions, row and
column ranges, graph kinds, aggregation weights and epilogue flags drawn at random, each checked
against the oracle element by element, plus everything outside the addressed block for being
untouched.  The hand-picked cases live in test_gpu_parity.py
these look for the corners nobody
thought of (one found: ReLU with ACCUMULATE on rows without entries)."""
import numpy as np
import pytest
import torch

import graphgen as gg
import oracle
from parity import RTOL_BF16, RTOL_F32, assert_close, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mg():
    import paper_2501_01951_amd as m

    assert torch.cuda.is_available()
    m.load_library()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bf16r(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).to(torch.float32).numpy()


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_aggregations(mg, seed):
    rng = np.random.default_rng(seed)
    ncase = 100
    for case in range(ncase):
        kind = rng.integers(0, 4)
        n = int(rng.choice([1, 2, 63, 64, 65, 300, 1000, 4097, 20000, 70001]))
        if kind == 0:   # sparse random, many empty rows when no loops
            e = int(n * rng.choice([0.2, 1, 4, 20]))
            src, dst = rng.integers(0, n, e), rng.integers(0, n, e)
        elif kind == 1:  # hubs: a few rows own most entries (rows far longer than a span)
            e = int(n * 8) + 10
            hubs = rng.integers(0, n, 3)
            src = np.where(rng.random(e) < 0.7, hubs[rng.integers(0, 3, e)], rng.integers(0, n, e))
            dst = rng.integers(0, n, e)
        elif kind == 2 and n >= 8:
            src, dst = gg.ring_lattice_edges(n, 2 * int(rng.integers(1, min(4, n // 2))))
        else:
            e = 3 * n
            src, dst = rng.integers(0, n, e), rng.integers(0, max(1, n // 50 + 1), e)  # few hot columns
        sym, loops = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        mode = int(rng.integers(0, 3))
        eps = float(rng.choice([0.0, 0.5]))
        flags = (mg.SYMMETRIZE if sym else 0) | (mg.ADD_SELF_LOOPS if loops else 0) | mg.BUILD_TRANSPOSE
        src = np.asarray(src, dtype=np.uint32)
        dst = np.asarray(dst, dtype=np.uint32)
        g = mg.build_csr(dev(src.view(np.int32)), dev(dst.view(np.int32)), n, flags)
        mg.normalize(g, mode, eps=eps)
        og = oracle.build_csr(src, dst, n, sym, loops)
        og = [oracle.normalize, oracle.normalize_mean, lambda q: oracle.normalize_sum(q, eps)][mode](og)
        oracle.transpose(og)
        bf = bool(rng.integers(0, 3) == 0)
        vec = 8 if bf else 4
        f = int(rng.choice([4, 7, 8, 12, 16, 33, 40, 64, 100, 127, 128, 200, 256, 257, 264, 520, 1040]))
        ld = (f + vec - 1) // vec * vec + vec * int(rng.integers(0, 3))
        tr = bool(rng.integers(0, 2))
        relu, acc = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        # column bounds that are multiples of nothing (slice bounds floor(d i / m) of Algorithm 2)
        c0 = int(rng.integers(0, f)) if rng.integers(0, 2) else 0
        c1 = f if rng.integers(0, 2) else int(rng.integers(c0 + 1, f + 1))
        r0 = int(rng.integers(0, n)) if rng.integers(0, 2) else 0
        r1 = n if rng.integers(0, 2) else int(rng.integers(r0, n + 1))
        use_mask = bool(rng.integers(0, 3) == 0) and not (relu or acc)
        h = gg.normal(1000 + case, 1, n, ld)
        z0 = gg.normal(1000 + case, 2, n, ld)
        if bf: h, z0 = bf16r(h), bf16r(z0)
        up = (lambda a: dev(a).to(torch.bfloat16)) if bf else dev
        hd, zd = up(h), up(z0)
        desc = f"case {case}: kind={kind} n={n} nnz={og.nnz} sym={sym} loops={loops} mode={mode} bf16={bf} f={f} ld={ld} tr={tr} relu={relu} acc={acc} mask={use_mask} cols=[{c0},{c1}) rows=[{r0},{r1})"
        say(desc)
        agg = oracle.spmm(og, h[:, :f].astype(np.float64), transposed=tr)
        ref = z0[:, :f].astype(np.float64).copy()
        blk = agg[r0:r1, c0:c1]
        if use_mask:
            bits = oracle.dropout_bitmap(case, n, f, 0.5)
            keep = ((bits[:, np.arange(f) // 32] >> (np.arange(f) % 32).astype(np.uint32)) & 1).astype(bool)
            blk = np.where(keep[r0:r1, c0:c1], blk, 0.0)
            mg.aggregate_masked(g, hd[:, :f], zd[:, :f], dev(bits.view(np.int32)), col_begin=c0, col_end=c1, row_begin=r0, row_end=r1, transpose=tr)
        else:
            if acc: blk = ref[r0:r1, c0:c1] + blk
            if relu: blk = np.maximum(blk, 0)
            mg.aggregate(g, hd[:, :f], zd[:, :f], col_begin=c0, col_end=c1, row_begin=r0, row_end=r1, transpose=tr, relu=relu, accumulate=acc)
        ref[r0:r1, c0:c1] = blk
        got = zd.float().cpu().numpy()
        assert_close(got[:, :f], ref, RTOL_BF16 if bf else RTOL_F32, desc)
        # untouched outside the block (exact)
        outside = np.ones((n, f), bool)
        outside[r0:r1, c0:c1] = False
        assert np.array_equal(got[:, :f][outside], z0[:, :f][outside].astype(np.float32)), "outside touched: " + desc
        assert np.array_equal(got[:, f:], z0[:, f:].astype(np.float32)), "padding touched: " + desc
        g.free()


@pytest.mark.parametrize("seed,arith", [(1, "fp32"), (2, "fp32"), (3, "bf16x3"), (4, "bf16x3")])
def test_random_update_products(mg, seed, arith):
    """arith = bf16x3: the same sweep with the three-term bf16 arithmetic switched on, which the
    wide fp32 products with whole reduction steps then take (the others must not care)."""
    mg.set_update_arith(mg.ARITH_BF16X3 if arith == "bf16x3" else mg.ARITH_FP32)
    try:
        _random_update_products(mg, seed)
    finally:
        mg.set_update_arith(mg.ARITH_FP32)


def _random_update_products(mg, seed):
    rng = np.random.default_rng(seed)
    ncase = 80
    for case in range(ncase):
        bf = bool(rng.integers(0, 3) == 0)
        vec = 8 if bf else 4
        n = int(rng.choice([1, 17, 127, 128, 129, 256, 1000, 1024, 2048, 3333, 5000, 16384 + 48, 40000]))
        k = int(rng.choice([4, 16, 20, 32, 48, 64, 100, 128, 160, 256, 272]))
        m = int(rng.choice([3, 8, 16, 32, 47, 64, 96, 128, 172, 256, 384]))
        padk, padm = vec * int(rng.integers(0, 3)), vec * int(rng.integers(0, 3))
        ldk, ldm = (k + vec - 1) // vec * vec + padk, (m + vec - 1) // vec * vec + padm
        ldw = (m + 3) // 4 * 4 + 4 * int(rng.integers(0, 2))
        z = gg.normal(2000 + case, 1, n, k)
        gr = gg.normal(2000 + case, 3, n, m)
        w = gg.glorot(2000 + case, 2, k, m)
        if bf: z, gr = bf16r(z), bf16r(gr)
        q = oracle.Q_BF16 if bf else oracle.Q_NONE
        rt = RTOL_BF16 if bf else RTOL_F32
        def buf(a, ld):
            t = torch.full((a.shape[0], ld), 7.0, device="cuda")
            t[:, :a.shape[1]] = dev(a)
            return t.to(torch.bfloat16) if bf else t
        zd, gd = buf(z, ldk), buf(gr, ldm)
        wd = torch.zeros(k, ldw, device="cuda")
        wd[:, :m] = dev(w)
        desc = f"case {case}: bf16={bf} n={n} k={k} m={m} ldk={ldk} ldm={ldm} ldw={ldw}"
        say(desc)
        z64, w64, g64 = z.astype(np.float64), w.astype(np.float64), gr.astype(np.float64)
        relu = bool(rng.integers(0, 2))
        out = buf(np.zeros((n, m), np.float32), ldm)
        mg.update(mg.OP_FWD_RELU if relu else mg.OP_FWD, zd[:, :k], wd[:, :m], out[:, :m], n, k, m)
        href = oracle.update_fwd(z64, w64, relu, q=q)
        o = out.float().cpu().numpy()
        assert_close(o[:, :m], href, rt, desc + " fwd")
        assert np.all(o[:, (m + vec - 1) // vec * vec:] == 7.0), desc + " fwd padding"
        use_ref = bool(rng.integers(0, 2))
        hr = oracle.update_fwd(z64, w64, True, q=q)
        hd = buf(hr.astype(np.float32), ldm) if use_ref else None
        dp = oracle.relu_grad(g64, hr if use_ref else None)
        dz = buf(np.zeros((n, k), np.float32), ldk)
        mg.update(mg.OP_DGRAD, gd[:, :m], wd[:, :m], dz[:, :k], n, k, m, relu_ref=hd[:, :m] if use_ref else None)
        o = dz.float().cpu().numpy()
        assert_close(o[:, :k], oracle.update_dgrad(dp, w64, q=q), rt, desc + " dgrad")
        assert np.all(o[:, (k + vec - 1) // vec * vec:] == 7.0), desc + " dgrad padding"
        beta = float(rng.integers(0, 2))
        dw = torch.full((k, ldw), 2.0, device="cuda")
        mg.update(mg.OP_WGRAD, zd[:, :k], gd[:, :m], dw[:, :m], n, k, m, relu_ref=hd[:, :m] if use_ref else None, beta=beta)
        o = dw.cpu().numpy()
        assert_close(o[:, :m], oracle.update_wgrad(z64, dp) + 2.0 * beta, 1e-3 if bf else RTOL_F32, desc + f" wgrad beta={beta}")
        assert np.all(o[:, m:] == 2.0), desc + " wgrad padding"
