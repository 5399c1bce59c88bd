"""GPU parity of the opt-in update arithmetic MIXGCN_ARITH_BF16X3 (fp32 operands as three bf16
terms, six bf16 MFMAs per product; forward, data gradient and weight gradient): the same oracle
and the same tolerance as the fp32 MFMA path,
two exactness pins (inputs whose terms and sums are exact must come out bit-exact), a check that
its error is not above the fp32 path's, and the products that must not change with the mode."""
import numpy as np
import pytest

import graphgen as gg
import oracle
from parity import RTOL_F32, assert_close, say
from test_gpu_parity import check_model, dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mg():
    import paper_2501_01951_amd as m

    m.load_library()
    return m


@pytest.fixture()
def split(mg):
    mg.set_update_arith(mg.ARITH_BF16X3)
    try:
        yield mg
    finally:
        mg.set_update_arith(mg.ARITH_FP32)


# (n, k, m): forward needs m > 64 and k a multiple of 16 from 64 up, the data gradient k > 64 and
# the same of m; ragged row counts, 4 to 17 reduction steps (the loop takes two per trip and
# finishes with one to three), several column tiles, a ragged last column tile
SPLIT_SHAPES = [(1000, 64, 128), (2048, 128, 256), (4133, 256, 256), (130, 256, 256), (1, 128, 128),
                (5000, 128, 1024), (777, 96, 160), (256, 112, 128), (384, 80, 144), (1500, 128, 172),
                (640, 176, 96), (129, 272, 80), (16, 128, 128), (47, 256, 128), (20000, 384, 128)]


@pytest.mark.parametrize("n,k,m", SPLIT_SHAPES)
def test_split_forward_and_data_gradient(split, n, k, m):
    mg = split
    say(f"bf16x3 update n={n} k={k} m={m}")
    ldk, ldm = k + 4, m + 8  # pitches of their own
    z = gg.normal(41, 1, n, k, ld=ldk)
    w = gg.glorot(41, 2, k, m, ld=ldm)
    gr = gg.normal(41, 3, n, m, ld=ldm)
    z64, w64, g64 = z[:, :k].astype(np.float64), w[:, :m].astype(np.float64), gr[:, :m].astype(np.float64)
    zd, wd, gd = dev(z), dev(w), dev(gr)
    for relu in (False, True):
        out = torch.full((n, ldm), 9.0, device="cuda")
        mg.update(mg.OP_FWD_RELU if relu else mg.OP_FWD, zd, wd, out, n, k, m)
        o = out.cpu().numpy()
        assert_close(o[:, :m], oracle.update_fwd(z64, w64, relu), RTOL_F32, f"fwd relu={relu}")
        assert np.all(o[:, m:] == 9.0)
    href = oracle.update_fwd(z64, w64, True)
    hd = torch.zeros(n, ldm, device="cuda")
    hd[:, :m] = dev(href.astype(np.float32))
    h64 = hd.cpu().numpy()[:, :m].astype(np.float64)
    for ref_t, ref_np in ((None, None), (hd, h64)):
        dp = oracle.relu_grad(g64, ref_np)
        dz = torch.full((n, ldk), 9.0, device="cuda")
        mg.update(mg.OP_DGRAD, gd, wd, dz, n, k, m, relu_ref=ref_t)
        o = dz.cpu().numpy()
        assert_close(o[:, :k], oracle.update_dgrad(dp, w64), RTOL_F32, "dgrad")
        assert np.all(o[:, k:] == 9.0)
        # the weight gradient takes the path for whole 128 x 128 tiles (rows beyond the last
        # multiple of 16 go to the fp32 kernel and are added)
        for beta in (0.0, 1.0):
            dw = torch.full((k, ldm), 2.0, device="cuda")
            mg.update(mg.OP_WGRAD, zd, gd, dw, n, k, m, relu_ref=ref_t, beta=beta)
            o = dw.cpu().numpy()
            assert_close(o[:, :m], oracle.update_wgrad(z64, dp) + 2.0 * beta, RTOL_F32, f"wgrad beta={beta}")
            assert np.all(o[:, m:] == 2.0)


def test_split_is_exact_where_fp32_is(split):
    """Small integers have one bf16 term and sums below 2^24; values with sixteen significant
    bits times {-1, 0, 1, 2} have two terms and sums below 2^24: every partial product and every
    partial sum is exact in fp32, so the result must equal the oracle's bit for bit."""
    mg = split
    rng = np.random.default_rng(5)
    n, k, m = 1000, 256, 128
    say("bf16x3 exactness, one-term integers")
    a = rng.integers(-255, 256, size=(n, k)).astype(np.float32)
    w = rng.integers(-255, 256, size=(k, m)).astype(np.float32)
    out = torch.empty(n, m, device="cuda")
    mg.update(mg.OP_FWD, dev(a), dev(w), out, n, k, m)
    assert np.array_equal(out.cpu().numpy().astype(np.float64),
                          oracle.update_fwd(a.astype(np.float64), w.astype(np.float64), False))
    say("bf16x3 exactness, two-term features")
    k = 64
    p, q = rng.integers(-127, 128, size=(n, k)), rng.integers(-127, 128, size=(n, k))
    a = (p + q / 256.0).astype(np.float32)
    w = rng.integers(-1, 3, size=(k, m)).astype(np.float32)
    assert np.array_equal(a.astype(np.float64), p + q / 256.0)
    out = torch.empty(n, m, device="cuda")
    mg.update(mg.OP_FWD, dev(a), dev(w), out, n, k, m)
    assert np.array_equal(out.cpu().numpy().astype(np.float64),
                          oracle.update_fwd(a.astype(np.float64), w.astype(np.float64), False))
    say("bf16x3 exactness, weight gradient with two-term features")
    kk, mm = 128, 256
    p, q = rng.integers(-127, 128, size=(n, kk)), rng.integers(-127, 128, size=(n, kk))
    a = (p + q / 256.0).astype(np.float32)
    g = rng.integers(-1, 3, size=(n, mm)).astype(np.float32)
    dw = torch.empty(kk, mm, device="cuda")
    mg.update(mg.OP_WGRAD, dev(a), dev(g), dw, n, kk, mm)
    assert np.array_equal(dw.cpu().numpy().astype(np.float64),
                          oracle.update_wgrad(a.astype(np.float64), g.astype(np.float64)))
    say("bf16x3 exactness, two-term weights in the data gradient")
    kk, mm = 128, 64  # dZ[n x kk] = G[n x mm] W[kk x mm]^T
    g = rng.integers(-1, 3, size=(n, mm)).astype(np.float32)
    p, q = rng.integers(-127, 128, size=(kk, mm)), rng.integers(-127, 128, size=(kk, mm))
    w = (p + q / 256.0).astype(np.float32)
    dz = torch.empty(n, kk, device="cuda")
    mg.update(mg.OP_DGRAD, dev(g), dev(w), dz, n, kk, mm)
    assert np.array_equal(dz.cpu().numpy().astype(np.float64),
                          oracle.update_dgrad(g.astype(np.float64), w.astype(np.float64)))


def _worst_error(got, a64, w64):
    ref = a64 @ w64
    bound = np.abs(a64) @ np.abs(w64)
    return float(np.max(np.abs(got.astype(np.float64) - ref) / bound))


def test_split_error_is_not_above_the_fp32_path(mg):
    """max |C - A W| / (|A| |W|) of both paths against fp64, on inputs with a wide spread of
    magnitudes: the three-term path must stay within 1.5 times the fp32 MFMA path's error and
    below 2^-20."""
    rng = np.random.default_rng(9)
    n, k, m = 4096, 256, 256
    a = (rng.standard_normal((n, k)) * np.exp2(rng.integers(-12, 13, size=(n, k)))).astype(np.float32)
    w = (rng.standard_normal((k, m)) * np.exp2(rng.integers(-6, 7, size=(k, m)))).astype(np.float32)
    a64, w64 = a.astype(np.float64), w.astype(np.float64)
    errs = {}
    try:
        for mode, name in ((mg.ARITH_FP32, "fp32"), (mg.ARITH_BF16X3, "bf16x3")):
            say(f"error of the {name} path")
            mg.set_update_arith(mode)
            out = torch.empty(n, m, device="cuda")
            mg.update(mg.OP_FWD, dev(a), dev(w), out, n, k, m)
            errs[name] = _worst_error(out.cpu().numpy(), a64, w64)
    finally:
        mg.set_update_arith(mg.ARITH_FP32)
    print(errs)
    assert errs["bf16x3"] < 2.0 ** -20
    assert errs["bf16x3"] <= 1.5 * errs["fp32"]


@pytest.mark.parametrize("n,k,m", [(1000, 100, 128), (1000, 64, 32), (900, 128, 200), (500, 48, 128)])
def test_products_outside_the_split_path_do_not_change(mg, n, k, m):
    """Reduction depths that are not whole steps, narrow outputs and the weight gradient keep the
    fp32 MFMA kernels: bit-identical results in both modes."""
    say(f"mode-independent products n={n} k={k} m={m}")
    z, w, gr = dev(gg.normal(43, 1, n, k)), dev(gg.glorot(43, 2, k, m)), dev(gg.normal(43, 3, n, m))
    res = {}
    try:
        for mode in (mg.ARITH_FP32, mg.ARITH_BF16X3):
            mg.set_update_arith(mode)
            out = torch.empty(n, m, device="cuda")
            dz = torch.empty(n, k, device="cuda")
            dw = torch.empty(k, m, device="cuda")
            if k % 16 or k < 64 or m <= 64:
                mg.update(mg.OP_FWD_RELU, z, w, out, n, k, m)
            else:
                out.zero_()
            if m % 16 or m < 64 or k <= 64:
                mg.update(mg.OP_DGRAD, gr, w, dz, n, k, m)
            else:
                dz.zero_()
            mg.update(mg.OP_WGRAD, z, gr, dw, n, k, m)
            res[mode] = (out.cpu().numpy(), dz.cpu().numpy(), dw.cpu().numpy())
    finally:
        mg.set_update_arith(mg.ARITH_FP32)
    for x, y in zip(res[mg.ARITH_FP32], res[mg.ARITH_BF16X3]):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("n_chunks", [1, 4])
def test_split_config2_shape_end_to_end(split, n_chunks):
    say(f"bf16x3, config 2 shape at R-MAT scale 15, end to end, chunks={n_chunks}")
    src, dst, n = gg.config_graph("c2", scale_override=15)
    x = gg.normal(gg.MASTER_SEED, 1, n, 128)
    ws = [gg.glorot(gg.MASTER_SEED, 10, 128, 256), gg.glorot(gg.MASTER_SEED, 11, 256, 256),
          gg.glorot(gg.MASTER_SEED, 12, 256, 16)]
    y = gg.labels(gg.MASTER_SEED, 5, n, 16)
    check_model(split, "c2@15 bf16x3", src, dst, n, x, ws, y, n_chunks)


def test_set_update_arith_rejects_unknown_modes(mg):
    with pytest.raises(mg.MixGCNError):
        mg.set_update_arith(7)
    mg.set_update_arith(mg.ARITH_FP32)
