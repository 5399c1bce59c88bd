"""Pins for the CPU oracle: everything here checks the oracle against something that is NOT
the oracle's own formula -- hand-worked fixtures, dense brute force built independently with
numpy, closed forms, invariants and finite differences.  No GPU needed."""
import math
import os

import numpy as np
import pytest

import graphgen as gg
import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------------------------------
# independent dense constructions (numpy only)
# ------------------------------------------------------------------------------------------
def dense_atilde(src, dst, n, symmetrize=True, self_loops=True):
    a = np.zeros((n, n), dtype=bool)
    for u, v in zip(src, dst):
        if u == v:
            continue
        a[u, v] = True
        if symmetrize:
            a[v, u] = True
    if self_loops:
        a[np.arange(n), np.arange(n)] = True
    return a


def dense_ahat(at):
    d = at.sum(axis=1).astype(np.float64)
    with np.errstate(divide="ignore"):
        s = np.where(d > 0, 1.0 / np.sqrt(d), 0.0)
    return s[:, None] * at.astype(np.float64) * s[None, :]


def csr_to_dense(g, vals=None):
    m = np.zeros((g.n, g.n), dtype=np.float64)
    for u in range(g.n):
        for e in range(g.rowptr[u], g.rowptr[u + 1]):
            m[u, g.col[e]] += 1.0 if vals is None else vals[e]
    return m


HAND_GRAPHS = {
    "path5": ([0, 1, 2, 3], [1, 2, 3, 4], 5),
    "star6": ([0, 0, 0, 0, 0], [1, 2, 3, 4, 5], 6),
    "k4": ([0, 0, 0, 1, 1, 2], [1, 2, 3, 2, 3, 3], 4),
    "two_components": ([0, 1, 3, 4], [1, 2, 4, 5], 7),  # node 6 isolated
    "dups_and_selfedges": ([0, 0, 1, 2, 2, 3, 1, 0], [1, 1, 0, 2, 3, 3, 2, 0], 4),
    "reverse_listed": ([4, 3, 2, 1], [3, 2, 1, 0], 5),
}


@pytest.mark.parametrize("name", sorted(HAND_GRAPHS))
@pytest.mark.parametrize("sym", [True, False])
@pytest.mark.parametrize("loops", [True, False])
def test_csr_matches_dense_boolean(name, sym, loops):
    src, dst, n = HAND_GRAPHS[name]
    g = oracle.build_csr(src, dst, n, symmetrize=sym, self_loops=loops)
    ref = dense_atilde(src, dst, n, sym, loops)
    assert g.nnz == int(ref.sum())
    assert np.array_equal(csr_to_dense(g) > 0, ref)
    assert np.array_equal(g.rowptr, np.concatenate([[0], np.cumsum(ref.sum(axis=1))]))
    for u in range(n):
        cols = g.col[g.rowptr[u]:g.rowptr[u + 1]]
        assert np.all(np.diff(cols.astype(np.int64)) > 0)  # strictly ascending => no duplicates
        assert np.array_equal(cols, np.nonzero(ref[u])[0])


def test_csr_random_64_nodes_vs_dense():
    rng = np.random.default_rng(7)
    for trial in range(20):
        n = int(rng.integers(2, 65))
        e = int(rng.integers(0, 4 * n))
        src = rng.integers(0, n, e)
        dst = rng.integers(0, n, e)
        g = oracle.normalize(oracle.build_csr(src, dst, n))
        at = dense_atilde(src, dst, n)
        assert np.array_equal(csr_to_dense(g) > 0, at)
        assert np.array_equal(g.deg, at.sum(axis=1))
        np.testing.assert_allclose(csr_to_dense(g, g.val), dense_ahat(at), rtol=1e-15, atol=0)


def test_csr_rejects_out_of_range():
    with pytest.raises(ValueError):
        oracle.build_csr([0, 5], [1, 2], 4)


def test_csr_invariants_er_and_rmat():
    for src, dst, n in [gg.config_graph("c1"), gg.config_graph("c2", scale_override=14)]:
        g = oracle.normalize(oracle.build_csr(src, dst, n))
        assert g.rowptr[0] == 0 and g.rowptr[-1] == g.nnz and np.all(np.diff(g.rowptr) >= 1)
        rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(g.rowptr))
        keys = rows * n + g.col
        assert np.all(np.diff(keys) > 0)  # sorted by (row, col), no duplicates
        # every row holds its own index
        has_diag = np.zeros(n, dtype=bool)
        has_diag[rows[g.col == rows]] = True
        assert has_diag.all()
        # (u, v) stored <=> (v, u) stored
        assert np.array_equal(np.sort(keys), np.sort(g.col.astype(np.int64) * n + rows))
        assert int(g.deg.sum()) == g.nnz
        # expected pair set, built independently with numpy sets
        m = src != dst
        a = np.concatenate([src[m].astype(np.int64) * n + dst[m], dst[m].astype(np.int64) * n + src[m],
                            np.arange(n, dtype=np.int64) * (n + 1)])
        assert np.array_equal(np.unique(a), keys)


def test_er_mean_degree():
    src, dst, n = gg.config_graph("c1")
    assert abs(2 * len(src) / n - 10.0) < 0.3


# ------------------------------------------------------------------------------------------
# A_hat values
# ------------------------------------------------------------------------------------------
def test_golden_path3_ahat():
    ref = np.loadtxt(os.path.join(GOLD, "path3_ahat.txt"))
    g = oracle.normalize(oracle.build_csr([0, 1], [1, 2], 3))
    np.testing.assert_allclose(csr_to_dense(g, g.val), ref, rtol=1e-15)
    np.testing.assert_allclose(csr_to_dense(g, g.val_f32.astype(np.float64)), ref, rtol=2e-7)


@pytest.mark.parametrize("n,k", [(16, 2), (50, 4), (1000, 10)])
def test_regular_graph_values_and_row_sums(n, k):
    src, dst = gg.ring_lattice_edges(n, k)
    g = oracle.normalize(oracle.build_csr(src, dst, n))
    assert np.all(g.deg == k + 1)
    np.testing.assert_allclose(g.val, 1.0 / (k + 1), rtol=1e-15)
    z = oracle.spmm(g, np.ones((n, 3)))
    np.testing.assert_allclose(z, 1.0, rtol=1e-14)


def test_eigenvector_identity_any_graph():
    # A_hat d^(1/2) = d^(1/2):  sum_v At_uv d_u^-1/2 d_v^-1/2 d_v^1/2 = d_u^-1/2 * d_u
    for src, dst, n in [gg.config_graph("c1"), gg.config_graph("c2", scale_override=15)]:
        g = oracle.normalize(oracle.build_csr(src, dst, n))
        r = np.sqrt(g.deg.astype(np.float64))[:, None]
        np.testing.assert_allclose(oracle.spmm(g, r), r, rtol=1e-12)


def test_complete_graph_is_column_mean():
    n = 12
    iu = np.triu_indices(n, 1)
    g = oracle.normalize(oracle.build_csr(iu[0], iu[1], n))
    h = np.random.default_rng(0).normal(size=(n, 5))
    np.testing.assert_allclose(oracle.spmm(g, h), np.tile(h.mean(axis=0), (n, 1)), rtol=1e-13)


def test_edgeless_graph_is_identity():
    n = 9
    g = oracle.normalize(oracle.build_csr([], [], n))
    assert g.nnz == n and np.all(g.val == 1.0) and np.all(g.deg == 1)
    h = np.random.default_rng(1).normal(size=(n, 4))
    assert np.array_equal(oracle.spmm(g, h), h)


def test_val_f32_symmetric_and_close():
    src, dst, n = gg.config_graph("c1")
    g = oracle.transpose(oracle.normalize(oracle.build_csr(src, dst, n)))
    assert np.array_equal(g.t_rowptr, g.rowptr) and np.array_equal(g.t_col, g.col)
    assert np.array_equal(g.t_val, g.val)  # A_hat^T == A_hat bit for bit on symmetrised input
    np.testing.assert_allclose(g.val_f32, g.val, rtol=1.5e-7)
    dense = csr_to_dense(g, g.val_f32.astype(np.float64))
    assert np.array_equal(dense, dense.T)


# ------------------------------------------------------------------------------------------
# products
# ------------------------------------------------------------------------------------------
def test_spmm_vs_dense_with_slices_and_row_ranges():
    rng = np.random.default_rng(3)
    n = 61
    src = rng.integers(0, n, 300)
    dst = rng.integers(0, n, 300)
    g = oracle.normalize(oracle.build_csr(src, dst, n))
    ah = dense_ahat(dense_atilde(src, dst, n))
    h = rng.normal(size=(n, 24))
    np.testing.assert_allclose(oracle.spmm(g, h), ah @ h, rtol=1e-12, atol=1e-14)
    z = oracle.spmm(g, h, c0=5, c1=17, r0=10, r1=33)
    ref = np.zeros_like(h)
    ref[10:33, 5:17] = (ah @ h)[10:33, 5:17]
    np.testing.assert_allclose(z, ref, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------------------------------
# S-SpMM (Sec. 3.2.1, Eq. 4) and the bitmap form of the ReLU mask
# ------------------------------------------------------------------------------------------
def unpack_bits(bits, m):
    """numpy-only reading of the bitmap layout: column j is bit j % 32 of word j // 32."""
    n = bits.shape[0]
    out = np.zeros((n, m), dtype=bool)
    for j in range(m):
        out[:, j] = (bits[:, j // 32] >> np.uint32(j % 32)) & np.uint32(1)
    return out


def test_relu_bitmap_layout_and_counts():
    rng = np.random.default_rng(11)
    x = rng.normal(size=(37, 70))
    x[3, 5] = 0.0       # zero is not positive
    x[4, 6] = -0.0
    x[5, 33] = np.nan   # neither is NaN
    bits = oracle.relu_bitmap(x)
    assert bits.shape == (37, 3) and bits.dtype == np.uint32
    np.testing.assert_array_equal(unpack_bits(bits, 70), x > 0)
    assert not (bits[:, 2] >> np.uint32(6)).any()  # bits past column 70 stay clear
    one = np.full((2, 40), -1.0)
    one[1, 35] = 2.0
    b = oracle.relu_bitmap(one)
    assert b[0].tolist() == [0, 0] and b[1].tolist() == [0, 1 << 3]


def test_sspmm_vs_dense_masked_product_slices_and_transpose():
    rng = np.random.default_rng(12)
    n = 53
    src = rng.integers(0, n, 260)
    dst = rng.integers(0, n, 260)
    h = rng.normal(size=(n, 40))
    mask = rng.random(size=(n, 40)) < 0.5
    bits = oracle.relu_bitmap(np.where(mask, 1.0, -1.0))
    g = oracle.normalize(oracle.build_csr(src, dst, n))
    ah = dense_ahat(dense_atilde(src, dst, n))
    np.testing.assert_allclose(oracle.sspmm(g, h, bits), (ah @ h) * mask, rtol=1e-12, atol=1e-14)
    z = oracle.sspmm(g, h, bits, c0=4, c1=36, r0=7, r1=40)
    ref = np.zeros_like(h)
    ref[7:40, 4:36] = ((ah @ h) * mask)[7:40, 4:36]
    np.testing.assert_allclose(z, ref, rtol=1e-12, atol=1e-14)
    # directed graph: the transposed operator is the dense transpose
    gd = oracle.transpose(oracle.normalize(oracle.build_csr(src, dst, n, symmetrize=False)))
    ad = dense_ahat(dense_atilde(src, dst, n, symmetrize=False))
    np.testing.assert_allclose(oracle.sspmm(gd, h, bits, transposed=True), (ad.T @ h) * mask,
                               rtol=1e-12, atol=1e-14)


def test_sspmm_complement_identity_and_regular_graph_closed_form():
    rng = np.random.default_rng(13)
    n, k = 64, 6
    src, dst = gg.ring_lattice_edges(n, k)
    g = oracle.normalize(oracle.build_csr(src, dst, n))
    mask = rng.random(size=(n, 33)) < 0.5
    bits = oracle.relu_bitmap(np.where(mask, 1.0, -1.0))
    nbits = oracle.relu_bitmap(np.where(mask, -1.0, 1.0))
    h = rng.normal(size=(n, 33))
    # every output is either kept or zero: the two halves add up to the plain aggregation exactly
    np.testing.assert_array_equal(oracle.sspmm(g, h, bits) + oracle.sspmm(g, h, nbits),
                                  oracle.spmm(g, h))
    # k-regular graph with self-loops: A_hat 1 = 1, so S-SpMM of the all-ones matrix is the mask
    np.testing.assert_allclose(oracle.sspmm(g, np.ones((n, 33)), bits), mask.astype(np.float64),
                               rtol=0, atol=1e-15)


# ------------------------------------------------------------------------------------------
# node reordering (Sec. 3.2.2): reverse Cuthill-McKee, bandwidth, Proposition 3.5
# ------------------------------------------------------------------------------------------
def scrambled(src, dst, n, seed):
    perm = np.random.default_rng(seed).permutation(n)
    return perm[np.asarray(src)], perm[np.asarray(dst)]


def test_rcm_golden_hand_example():
    edges, pos, b = [], None, None
    for line in open(os.path.join(GOLD, "rcm_hand6.txt")):
        t = line.split()
        if not t or t[0] == "#":
            continue
        if t[0] == "pos":
            pos = [int(x) for x in t[1:]]
        elif t[0] == "bandwidth":
            b = int(t[1])
        else:
            edges.append((int(t[0]), int(t[1])))
    g = oracle.build_csr([e[0] for e in edges], [e[1] for e in edges], 6)
    got = oracle.rcm(g)
    assert got.tolist() == pos
    assert oracle.bandwidth(g, got) == b


def test_rcm_closed_forms_path_cycle_star_complete():
    n = 40
    # a path, however it is labelled, is laid out end to end: bandwidth 1; two paths as well
    s, d = scrambled(np.arange(n - 1), np.arange(1, n), n, 1)
    g = oracle.build_csr(s, d, n)
    pos = oracle.rcm(g)
    assert sorted(pos.tolist()) == list(range(n))
    assert oracle.bandwidth(g, pos) == 1 and oracle.bandwidth(g) > 1
    a = np.r_[np.arange(0, 19), np.arange(20, 39)]
    s, d = scrambled(a, a + 1, n, 2)
    g = oracle.build_csr(s, d, n)
    assert oracle.bandwidth(g, oracle.rcm(g)) == 1
    # a cycle is folded: bandwidth 2
    s, d = scrambled(np.arange(n), (np.arange(n) + 1) % n, n, 3)
    g = oracle.build_csr(s, d, n)
    assert oracle.bandwidth(g, oracle.rcm(g)) == 2
    # a star started from a leaf: leaf, centre, the other leaves -> the centre is n - 2 places
    # away from the last leaf
    s, d = scrambled(np.zeros(n - 1, dtype=int), np.arange(1, n), n, 4)
    g = oracle.build_csr(s, d, n)
    assert oracle.bandwidth(g, oracle.rcm(g)) == n - 2
    # complete graph: every sequence has bandwidth n - 1
    iu = np.triu_indices(12, 1)
    g = oracle.build_csr(iu[0], iu[1], 12)
    assert oracle.bandwidth(g, oracle.rcm(g)) == 11 == oracle.bandwidth(g)


def test_rcm_grid_and_brute_force_lower_bound():
    # r x c grid, scrambled: breadth-first levels from a corner are anti-diagonals of at most
    # min(r, c) nodes and edges join consecutive levels, so the bandwidth stays below 2 min(r, c)
    r, c = 7, 30
    idx = np.arange(r * c).reshape(r, c)
    s = np.r_[idx[:, :-1].ravel(), idx[:-1, :].ravel()]
    d = np.r_[idx[:, 1:].ravel(), idx[1:, :].ravel()]
    s, d = scrambled(s, d, r * c, 5)
    g = oracle.build_csr(s, d, r * c)
    b = oracle.bandwidth(g, oracle.rcm(g))
    assert r <= b < 2 * r and oracle.bandwidth(g) > 4 * r
    # tiny graphs: never better than the optimum found by trying every sequence
    import itertools
    rng = np.random.default_rng(6)
    for _ in range(5):
        n = 7
        s, d = rng.integers(0, n, 9), rng.integers(0, n, 9)
        g = oracle.build_csr(s, d, n)
        best = min(oracle.bandwidth(g, np.array(p, dtype=np.uint32))
                   for p in itertools.permutations(range(n)))
        got = oracle.bandwidth(g, oracle.rcm(g))
        assert best <= got <= oracle.bandwidth(g) or got <= n - 1


def test_bandwidth_definition_vs_numpy():
    rng = np.random.default_rng(7)
    n = 200
    s, d = rng.integers(0, n, 900), rng.integers(0, n, 900)
    g = oracle.build_csr(s, d, n)
    pos = rng.permutation(n).astype(np.uint32)
    keep = s != d
    assert oracle.bandwidth(g) == np.abs(s[keep] - d[keep]).max()
    assert oracle.bandwidth(g, pos) == np.abs(pos[s[keep]].astype(np.int64) - pos[d[keep]]).max()


def test_pipeline_stages_is_proposition_3_5():
    for n in (10, 100, 4096, 1 << 20):
        for b in (0, 1, n // 3, n // 2, n - 2, n - 1):
            s = oracle.pipeline_stages(n, b)
            assert s == -(-2 * n // (n - b))            # ceil(2n / (n - b))
            assert (n - b) * s >= 2 * n and (s == 1 or (n - b) * (s - 1) < 2 * n)
        assert oracle.pipeline_stages(n, n) == 0 and oracle.pipeline_stages(n, n + 5) == 0
    assert oracle.pipeline_stages(100, 0) == 2  # no dependence at all still needs two batches


def test_transpose_on_directed_input_adjoint_and_dense():
    rng = np.random.default_rng(4)
    n = 40
    src = rng.integers(0, n, 200)
    dst = rng.integers(0, n, 200)
    g = oracle.transpose(oracle.normalize(oracle.build_csr(src, dst, n, symmetrize=False)))
    ah = dense_ahat(dense_atilde(src, dst, n, symmetrize=False))
    assert not np.array_equal(ah, ah.T)
    x = rng.normal(size=(n, 6))
    y = rng.normal(size=(n, 6))
    np.testing.assert_allclose(oracle.spmm(g, y, transposed=True), ah.T @ y, rtol=1e-12, atol=1e-14)
    lhs = np.sum(oracle.spmm(g, x) * y)
    rhs = np.sum(x * oracle.spmm(g, y, transposed=True))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    # columns of the transpose ascend too
    for u in range(n):
        assert np.all(np.diff(g.t_col[g.t_rowptr[u]:g.t_rowptr[u + 1]].astype(np.int64)) > 0)


def test_column_sum_identity():
    src, dst, n = gg.config_graph("c2", scale_override=12)
    g = oracle.normalize(oracle.build_csr(src, dst, n))
    h = gg.normal(1, 2, n, 8).astype(np.float64)
    colsum_ahat = np.bincount(g.col, weights=g.val, minlength=n)  # 1^T A_hat
    np.testing.assert_allclose(oracle.spmm(g, h).sum(axis=0), colsum_ahat @ h, rtol=1e-10)


def test_updates_vs_numpy_matmul():
    rng = np.random.default_rng(5)
    z = rng.normal(size=(37, 11))
    w = rng.normal(size=(11, 7))
    dp = rng.normal(size=(37, 7))
    p = z @ w
    np.testing.assert_allclose(oracle.update_fwd(z, w, relu=False), p, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.update_fwd(z, w, relu=True), np.maximum(p, 0), rtol=1e-12,
                               atol=1e-14)
    np.testing.assert_allclose(oracle.update_dgrad(dp, w), dp @ w.T, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.update_wgrad(z, dp), z.T @ dp, rtol=1e-12, atol=1e-13)
    outer = sum(np.outer(z[v], dp[v]) for v in range(37))
    np.testing.assert_allclose(oracle.update_wgrad(z, dp), outer, rtol=1e-12, atol=1e-13)
    href = rng.normal(size=(37, 7))
    href[3, 2] = 0.0
    np.testing.assert_array_equal(oracle.relu_grad(dp, href), dp * (href > 0))


def test_wgrad_spans_several_row_blocks():
    rng = np.random.default_rng(6)
    z = rng.normal(size=(9000, 3))
    dp = rng.normal(size=(9000, 2))
    np.testing.assert_allclose(oracle.update_wgrad(z, dp), z.T @ dp, rtol=1e-11, atol=1e-12)


def test_golden_star4_layer():
    ref = np.loadtxt(os.path.join(GOLD, "star4_layer.txt"))
    g = oracle.normalize(oracle.build_csr([0, 0, 0], [1, 2, 3], 4))
    h = np.array([[1.0], [2.0], [3.0], [-10.0]])
    w = np.array([[1.0, -1.0]])
    z = oracle.spmm(g, h)
    np.testing.assert_allclose(oracle.update_fwd(z, w, relu=False), ref, rtol=1e-15)
    np.testing.assert_allclose(oracle.update_fwd(z, w, relu=True), np.maximum(ref, 0), rtol=1e-15)


def test_edgeless_graph_layer_is_mlp_layer():
    n = 10
    rng = np.random.default_rng(8)
    g = oracle.normalize(oracle.build_csr([], [], n))
    x = rng.normal(size=(n, 6))
    w = rng.normal(size=(6, 4))
    out = oracle.update_fwd(oracle.spmm(g, x), w, relu=True)
    np.testing.assert_allclose(out, np.maximum(x @ w, 0), rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------------------------------
# loss
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("c", [8, 16, 172, 47])
def test_loss_at_zero_weights_is_ln_c(c):
    n = 50
    y = gg.labels(1, 9, n, c)
    loss, d = oracle.softmax_xent(np.zeros((n, c)), y)
    assert abs(loss - math.log(c)) < 1e-14
    np.testing.assert_allclose(d.sum(axis=1), 0.0, atol=1e-16)
    freq = np.bincount(y, minlength=c) / n
    np.testing.assert_allclose(d.sum(axis=0), 1.0 / c - freq, atol=1e-15)


def test_loss_vs_scipy_and_shift_invariance():
    from scipy.special import log_softmax

    rng = np.random.default_rng(9)
    x = rng.normal(size=(33, 7)) * 5
    y = rng.integers(0, 7, 33).astype(np.int32)
    loss, d = oracle.softmax_xent(x, y)
    ls = log_softmax(x, axis=1)
    assert abs(loss + ls[np.arange(33), y].mean()) < 1e-13
    oh = np.eye(7)[y]
    np.testing.assert_allclose(d, (np.exp(ls) - oh) / 33, atol=1e-15)
    loss2, _ = oracle.softmax_xent(x + 1000.0, y)  # max subtraction keeps it finite
    assert abs(loss - loss2) < 1e-9


# ------------------------------------------------------------------------------------------
# whole forward + backward
# ------------------------------------------------------------------------------------------
def _tiny_problem(seed, n=12, dims=(4, 3, 3, 2)):
    rng = np.random.default_rng(seed)
    e = 2 * n
    src = rng.integers(0, n, e)
    dst = rng.integers(0, n, e)
    g = oracle.normalize(oracle.build_csr(src, dst, n))
    x = rng.normal(size=(n, dims[0]))
    ws = [rng.normal(size=(dims[i], dims[i + 1])) for i in range(len(dims) - 1)]
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    return g, src, dst, x, ws, y


def test_linear_activation_closed_form():
    g, src, dst, x, ws, y = _tiny_problem(11)
    ah = dense_ahat(dense_atilde(src, dst, g.n))
    out = oracle.gcn_step(g, x, ws, y, linear=True, backward=False)
    ref = np.linalg.matrix_power(ah, 3) @ x @ ws[0] @ ws[1] @ ws[2]
    np.testing.assert_allclose(out["logits"], ref, rtol=1e-11, atol=1e-13)


def test_forward_vs_dense_definition():
    g, src, dst, x, ws, y = _tiny_problem(12)
    ah = dense_ahat(dense_atilde(src, dst, g.n))
    h = x
    for l, w in enumerate(ws):
        h = ah @ h @ w
        if l < len(ws) - 1:
            h = np.maximum(h, 0)
    out = oracle.gcn_step(g, x, ws, y, backward=False)
    np.testing.assert_allclose(out["logits"], h, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_gradients_vs_central_finite_differences(seed):
    g, src, dst, x, ws, y = _tiny_problem(seed)
    base = oracle.gcn_step(g, x, ws, y, want_dx=True)
    # stay off the ReLU kinks: every pre-activation must be clear of 0 by more than the step
    for l in (1, 2):
        pre = base["Z"][l - 1] @ ws[l - 1]
        if np.min(np.abs(pre)) < 1e-3:
            pytest.skip("sample too close to a ReLU kink")
    hstep = 1e-5

    def loss_at(xx, wws):
        return oracle.gcn_step(g, xx, wws, y, backward=False)["loss"]

    for l, w in enumerate(ws):
        num = np.zeros_like(w)
        for idx in np.ndindex(*w.shape):
            wp = [a.copy() for a in ws]
            wm = [a.copy() for a in ws]
            wp[l][idx] += hstep
            wm[l][idx] -= hstep
            num[idx] = (loss_at(x, wp) - loss_at(x, wm)) / (2 * hstep)
        np.testing.assert_allclose(base["dW"][l], num, rtol=2e-6, atol=1e-9)
    num = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += hstep
        xm[idx] -= hstep
        num[idx] = (loss_at(xp, ws) - loss_at(xm, ws)) / (2 * hstep)
    np.testing.assert_allclose(base["dX"], num, rtol=2e-6, atol=1e-9)


def test_gradients_fd_on_directed_graph_pins_transpose_in_backward():
    rng = np.random.default_rng(31)
    n = 10
    src = rng.integers(0, n, 25)
    dst = rng.integers(0, n, 25)
    g = oracle.normalize(oracle.build_csr(src, dst, n, symmetrize=False))
    x = rng.normal(size=(n, 3))
    ws = [rng.normal(size=(3, 3)), rng.normal(size=(3, 2))]
    y = rng.integers(0, 2, n).astype(np.int32)
    base = oracle.gcn_step(g, x, ws, y, want_dx=True, linear=True)
    hstep = 1e-5
    num = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += hstep
        xm[idx] -= hstep
        num[idx] = (oracle.gcn_step(g, xp, ws, y, linear=True, backward=False)["loss"]
                    - oracle.gcn_step(g, xm, ws, y, linear=True, backward=False)["loss"]) / (2 * hstep)
    np.testing.assert_allclose(base["dX"], num, rtol=2e-6, atol=1e-9)


def test_step_matches_composition_of_calls():
    g, src, dst, x, ws, y = _tiny_problem(41, n=30, dims=(5, 6, 4))
    out = oracle.gcn_step(g, x, ws, y, want_dx=True)
    z0 = oracle.spmm(g, x)
    h1 = oracle.update_fwd(z0, ws[0], relu=True)
    z1 = oracle.spmm(g, h1)
    logits = oracle.update_fwd(z1, ws[1], relu=False)
    loss, dp1 = oracle.softmax_xent(logits, y)
    assert loss == out["loss"]
    np.testing.assert_array_equal(out["logits"], logits)
    np.testing.assert_array_equal(out["dW"][1], oracle.update_wgrad(z1, dp1))
    dh1 = oracle.spmm(g, oracle.update_dgrad(dp1, ws[1]), transposed=True)
    dp0 = oracle.relu_grad(dh1, h1)
    np.testing.assert_array_equal(out["dW"][0], oracle.update_wgrad(z0, dp0))
    np.testing.assert_array_equal(out["dX"],
                                  oracle.spmm(g, oracle.update_dgrad(dp0, ws[0]), transposed=True))


def _round_bf16(a):
    """bf16 (8 exponent bits, 7 fraction bits) round-to-nearest-even of doubles, written from
    the format: go through fp32 and round its low 16 bits away with numpy integer arithmetic."""
    u = np.asarray(a, dtype=np.float64).astype(np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def _is_bf16(a):
    return np.array_equal(_round_bf16(a), np.asarray(a, dtype=np.float64))


def _round_as(q):
    if q == oracle.Q_BF16:
        return _round_bf16
    return lambda a: np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


@pytest.mark.parametrize("q", [oracle.Q_F32, oracle.Q_BF16])
def test_every_call_with_storage_rounding_is_the_unrounded_call_rounded_once(q):
    """q rounds a result where it is stored and nowhere else: each single call with q equals
    the same call without q, rounded by an independent implementation of the format."""
    g, src, dst, x, ws, y = _tiny_problem(43, n=40, dims=(6, 5, 4))
    rnd = _round_as(q)
    rng = np.random.default_rng(5)
    bits = oracle.relu_bitmap(rng.normal(size=(g.n, 6)))
    np.testing.assert_array_equal(oracle.spmm(g, x, q=q), rnd(oracle.spmm(g, x)))
    np.testing.assert_array_equal(oracle.spmm(g, x, transposed=True, q=q),
                                  rnd(oracle.spmm(g, x, transposed=True)))
    np.testing.assert_array_equal(oracle.sspmm(g, x, bits, q=q), rnd(oracle.sspmm(g, x, bits)))
    for relu in (True, False):
        np.testing.assert_array_equal(oracle.update_fwd(x, ws[0], relu, q=q),
                                      rnd(oracle.update_fwd(x, ws[0], relu)))
    dp = rng.normal(size=(g.n, 5))
    np.testing.assert_array_equal(oracle.update_dgrad(dp, ws[0], q=q),
                                  rnd(oracle.update_dgrad(dp, ws[0])))
    href = rng.normal(size=(g.n, 5))
    np.testing.assert_array_equal(oracle.relu_grad(dp, href, q=q), rnd(oracle.relu_grad(dp, href)))
    assert not _is_bf16(oracle.spmm(g, x)) and _is_bf16(oracle.spmm(g, x, q=oracle.Q_BF16))


def _composed_step(g, x, ws, y, q, skip=None):
    """The 3-layer step as a sequence of the single calls, every stored n x F tensor rounded
    with q where it is written -- except the one named by `skip` (to show that leaving any one
    rounding out changes the result)."""
    skip = set((skip or "").split("+"))

    def qq(name):
        return oracle.Q_NONE if name in skip else q

    rnd = _round_as(q)
    L = len(ws)
    hs, zs = [x], []
    for l in range(L):
        zs.append(oracle.spmm(g, hs[l], q=qq(f"Z{l}")))
        hs.append(oracle.update_fwd(zs[l], ws[l], relu=l < L - 1, q=qq(f"H{l + 1}")))
    loss, dp = oracle.softmax_xent(hs[L], y)
    if "dlogits" not in skip:
        dp = rnd(dp)
    dws = [None] * L
    dx = None
    for l in range(L - 1, -1, -1):
        dws[l] = oracle.update_wgrad(zs[l], dp)
        dz = oracle.update_dgrad(dp, ws[l], q=qq(f"dZ{l}"))
        dh = oracle.spmm(g, dz, transposed=True, q=qq(f"dH{l}"))
        if l == 0:
            dx = dh
            break
        dp = oracle.relu_grad(dh, hs[l], q=qq(f"dP{l - 1}"))
    return {"loss": loss, "Z": zs, "H": hs, "dW": dws, "dX": dx}


# dP_{l-1} = dH_l (.) mask is rounded like dH_l, and rounding twice is rounding once: the two
# are one rounding point, left out together
ROUNDING_POINTS = (["Z0", "Z1", "Z2", "H1", "H2", "H3", "dlogits"] +
                   ["dZ2", "dZ1", "dZ0", "dH2+dP1", "dH1+dP0", "dH0"])


@pytest.mark.parametrize("q", [oracle.Q_F32, oracle.Q_BF16])
def test_rounded_step_is_the_composition_of_the_rounded_calls(q):
    """The bf16 (and fp32) storage mode of the whole step: exactly the tensors that are stored as
    n x F arrays -- Z_l, H_l including the logits, the loss gradient, dZ_l, dH_l, dP_l -- are
    rounded where they are written; the loss and dW are not."""
    g, src, dst, x, ws, y = _tiny_problem(44, n=48, dims=(6, 7, 5, 4))
    x = _round_as(q)(x)
    out = oracle.gcn_step(g, x, ws, y, want_dx=True, q=q)
    ref = _composed_step(g, x, ws, y, q)
    assert out["loss"] == ref["loss"]
    for l in range(3):
        np.testing.assert_array_equal(out["Z"][l], ref["Z"][l])
        np.testing.assert_array_equal(out["H"][l + 1], ref["H"][l + 1])
        np.testing.assert_array_equal(out["dW"][l], ref["dW"][l])
    np.testing.assert_array_equal(out["dX"], ref["dX"])
    if q == oracle.Q_BF16:
        for l in range(3):
            assert _is_bf16(out["Z"][l]) and _is_bf16(out["H"][l + 1])
            assert not _is_bf16(out["dW"][l])
        assert _is_bf16(out["dX"]) and _is_bf16(out["logits"])
        assert not _is_bf16(np.array([out["loss"]]))


@pytest.mark.parametrize("skip", ROUNDING_POINTS)
def test_leaving_out_any_one_rounding_point_changes_the_bf16_step(skip):
    """Sensitivity of the pin above: the composition with one rounding left out no longer
    equals the step, so a rounding dropped from (or moved inside) the step would be seen."""
    g, src, dst, x, ws, y = _tiny_problem(44, n=48, dims=(6, 7, 5, 4))
    x = _round_bf16(x)
    out = oracle.gcn_step(g, x, ws, y, want_dx=True, q=oracle.Q_BF16)
    ref = _composed_step(g, x, ws, y, oracle.Q_BF16, skip=skip)
    same = all(np.array_equal(out["dW"][l], ref["dW"][l]) for l in range(3))
    same = same and np.array_equal(out["dX"], ref["dX"]) and out["loss"] == ref["loss"]
    same = same and all(np.array_equal(out["H"][l + 1], ref["H"][l + 1]) for l in range(3))
    assert not same


def test_relu_sign_input_replaces_only_the_derivative_decision():
    """relu_sign stands in for H_l in dP_{l-1} = dH_l (.) 1[. > 0] and in nothing else: the
    oracle's own activations give the step unchanged; a stand-in with planted flips gives the
    composition of the single calls with relu_grad taken from the stand-in; the forward pass,
    the loss and the gradients of the layers at and above the stand-in do not move."""
    g, src, dst, x, ws, y = _tiny_problem(45, n=50, dims=(5, 6, 6, 3))
    base = oracle.gcn_step(g, x, ws, y, want_dx=True)
    again = oracle.gcn_step(g, x, ws, y, want_dx=True,
                            relu_sign=[None, base["H"][1], base["H"][2], None])
    for l in range(3):
        np.testing.assert_array_equal(base["dW"][l], again["dW"][l])
    np.testing.assert_array_equal(base["dX"], again["dX"])
    rng = np.random.default_rng(9)
    s2 = base["H"][2].copy()
    flip = rng.random(s2.shape) < 0.2
    s2[flip] = np.where(s2[flip] > 0, 0.0, 1.0)  # a zero becomes "positive" and the reverse
    got = oracle.gcn_step(g, x, ws, y, want_dx=True, relu_sign=[None, None, s2, None])
    assert got["loss"] == base["loss"]
    for l in range(3):
        np.testing.assert_array_equal(got["H"][l + 1], base["H"][l + 1])
    np.testing.assert_array_equal(got["dW"][2], base["dW"][2])
    _, dp2 = oracle.softmax_xent(base["logits"], y)
    dh2 = oracle.spmm(g, oracle.update_dgrad(dp2, ws[2]), transposed=True)
    dp1 = oracle.relu_grad(dh2, s2)
    np.testing.assert_array_equal(got["dW"][1], oracle.update_wgrad(base["Z"][1], dp1))
    dh1 = oracle.spmm(g, oracle.update_dgrad(dp1, ws[1]), transposed=True)
    dp0 = oracle.relu_grad(dh1, base["H"][1])
    np.testing.assert_array_equal(got["dW"][0], oracle.update_wgrad(base["Z"][0], dp0))
    assert not np.array_equal(got["dW"][1], base["dW"][1])
    assert not np.array_equal(got["dW"][0], base["dW"][0])


def test_bf16_quantiser_rounds_to_nearest_even():
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up.
    z = np.array([[1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.3]])
    w = np.eye(4)
    out = oracle.update_fwd(z, w, relu=False, q=oracle.Q_BF16)
    assert out[0, 0] == 1.0 and out[0, 1] == 1.0 + 2.0 ** -6 and out[0, 2] == 1.0 + 2.0 ** -7
    assert out[0, 3] == np.float32(-0.30078125)
    out32 = oracle.update_fwd(z, w, relu=False, q=oracle.Q_F32)
    assert np.array_equal(out32, z.astype(np.float32).astype(np.float64))


# ------------------------------------------------------------------------------------------
# GraphSAGE (mean) and GIN: the other two architectures of the paper's experiments (Sec. 4).
# Pins: dense brute force written from the cited definitions, closed forms, special cases that
# reduce to a perceptron, central finite differences for every gradient.
# ------------------------------------------------------------------------------------------
def _tiny_variant_problem(seed, n=11, dims=(4, 3, 2), loops=False):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, n, 2 * n)
    dst = rng.integers(0, n, 2 * n)
    g = oracle.build_csr(src, dst, n, True, loops)
    x = rng.normal(size=(n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    return rng, g, src, dst, x, y


def test_mean_weights_row_sums_dense_form_and_transpose():
    rng, g, src, dst, x, y = _tiny_variant_problem(51, n=40)
    oracle.normalize_mean(g)
    a = dense_atilde(src, dst, g.n, True, False).astype(np.float64)
    deg = a.sum(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        am = np.where(deg[:, None] > 0, a / deg[:, None], 0.0)
    assert np.array_equal(g.deg, deg.astype(np.uint32))
    np.testing.assert_allclose(csr_to_dense(g, g.val), am, rtol=0, atol=1e-15)
    # rows with neighbors sum to one; the mean of a constant is the constant
    ones = oracle.spmm(g, np.ones((g.n, 3)))
    assert np.allclose(ones[deg > 0], 1.0) and np.all(ones[deg == 0] == 0.0)
    h = rng.normal(size=(g.n, 5))
    np.testing.assert_allclose(oracle.spmm(g, h), am @ h, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.spmm(g, h, transposed=True), am.T @ h, rtol=1e-12, atol=1e-14)
    # the fp32 encoding is the rounded reciprocal of the row count
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    assert np.array_equal(g.val_f32, (1.0 / deg[rows]).astype(np.float32))


@pytest.mark.parametrize("eps", [0.0, 0.25, -1.0])
def test_sum_weights_dense_form_and_regular_graph(eps):
    rng, g, src, dst, x, y = _tiny_variant_problem(52, n=30, loops=True)
    oracle.normalize_sum(g, eps)
    a = dense_atilde(src, dst, g.n, True, False).astype(np.float64)
    want = a + (1.0 + eps) * np.eye(g.n)
    np.testing.assert_allclose(csr_to_dense(g, g.val), want, rtol=0, atol=0)
    h = rng.normal(size=(g.n, 4))
    np.testing.assert_allclose(oracle.spmm(g, h), (1 + eps) * h + a @ h, rtol=1e-12, atol=1e-13)
    # k-regular ring: every row of (A + (1 + eps) I) 1 is k + 1 + eps
    s, d = gg.ring_lattice_edges(50, 6)
    r = oracle.normalize_sum(oracle.build_csr(s, d, 50, True, True), eps)
    np.testing.assert_allclose(oracle.spmm(r, np.ones((50, 2))), 6 + 1 + eps, rtol=1e-14)


def test_sage_forward_vs_dense_definition_and_concat_order():
    rng, g, src, dst, x, y = _tiny_variant_problem(53)
    oracle.normalize_mean(g)
    ws = [rng.normal(size=(8, 3)), rng.normal(size=(6, 2))]
    a = dense_atilde(src, dst, g.n, True, False).astype(np.float64)
    h = x
    for l, w in enumerate(ws):
        d = h.shape[1]
        mean = np.zeros_like(h)
        for v in range(g.n):  # the definition, node by node
            nb = np.nonzero(a[v])[0]
            if len(nb):
                mean[v] = h[nb].mean(axis=0)
        h = h @ w[:d] + mean @ w[d:]  # own features meet the FIRST d rows of W
        if l < len(ws) - 1:
            h = np.maximum(h, 0)
    out = oracle.sage_step(g, x, ws, y, backward=False)
    np.testing.assert_allclose(out["logits"], h, rtol=1e-11, atol=1e-13)


def test_sage_special_cases_reduce_to_a_perceptron():
    rng, g, src, dst, x, y = _tiny_variant_problem(54)
    oracle.normalize_mean(g)
    w0, w1 = rng.normal(size=(8, 3)), rng.normal(size=(6, 2))
    # neighbor half of every W zero: the graph does not matter
    w0z, w1z = w0.copy(), w1.copy()
    w0z[4:] = 0
    w1z[3:] = 0
    out = oracle.sage_step(g, x, [w0z, w1z], y, backward=False)
    np.testing.assert_allclose(out["logits"], np.maximum(x @ w0[:4], 0) @ w1[:3], rtol=1e-12, atol=1e-14)
    # a graph of self-loops only: the mean is the node itself, so W_self + W_neigh acts on it
    n = g.n
    loops = oracle.normalize_mean(oracle.build_csr(np.arange(0), np.arange(0), n, True, True))
    out = oracle.sage_step(loops, x, [w0, w1], y, backward=False)
    ref = np.maximum(x @ (w0[:4] + w0[4:]), 0) @ (w1[:3] + w1[3:])
    np.testing.assert_allclose(out["logits"], ref, rtol=1e-12, atol=1e-14)


def test_gin_forward_vs_dense_definition():
    rng, g, src, dst, x, y = _tiny_variant_problem(55, loops=True)
    eps = 0.3
    oracle.normalize_sum(g, eps)
    w1s = [rng.normal(size=(4, 5)), rng.normal(size=(3, 4))]
    w2s = [rng.normal(size=(5, 3)), rng.normal(size=(4, 2))]
    a = dense_atilde(src, dst, g.n, True, False)
    h = x
    for l in range(2):
        agg = np.zeros_like(h)
        for v in range(g.n):  # (1 + eps) h_v + sum over the neighbors
            agg[v] = (1 + eps) * h[v] + h[np.nonzero(a[v])[0]].sum(axis=0)
        h = np.maximum(agg @ w1s[l], 0) @ w2s[l]
        if l == 0:
            h = np.maximum(h, 0)
    out = oracle.gin_step(g, x, w1s, w2s, y, backward=False)
    np.testing.assert_allclose(out["logits"], h, rtol=1e-11, atol=1e-13)


def _fd_check(loss_at, params, grads, hstep=1e-6):
    for p, gr in zip(params, grads):
        num = np.zeros_like(p)
        for idx in np.ndindex(*p.shape):
            old = p[idx]
            p[idx] = old + hstep
            lp = loss_at()
            p[idx] = old - hstep
            lm = loss_at()
            p[idx] = old
            num[idx] = (lp - lm) / (2 * hstep)
        np.testing.assert_allclose(gr, num, rtol=5e-6, atol=2e-9)


@pytest.mark.parametrize("seed", [61, 62, 63])
def test_sage_gradients_vs_central_finite_differences(seed):
    rng, g, src, dst, x, y = _tiny_variant_problem(seed, dims=(4, 3, 3, 2))
    oracle.normalize_mean(g)
    ws = [rng.normal(size=(8, 3)), rng.normal(size=(6, 3)), rng.normal(size=(6, 2))]
    base = oracle.sage_step(g, x, ws, y, want_dx=True)
    for l in (0, 1):
        if np.min(np.abs(base["X"][l] @ ws[l])) < 1e-4:
            pytest.skip("sample too close to a ReLU kink")
    _fd_check(lambda: oracle.sage_step(g, x, ws, y, backward=False)["loss"], ws + [x],
              base["dW"] + [base["dX"]])


@pytest.mark.parametrize("seed", [71, 74, 75])
def test_gin_gradients_vs_central_finite_differences(seed):
    rng, g, src, dst, x, y = _tiny_variant_problem(seed, loops=True)
    oracle.normalize_sum(g, 0.2)
    w1s = [rng.normal(size=(4, 3)) * 0.5, rng.normal(size=(3, 3)) * 0.5]
    w2s = [rng.normal(size=(3, 3)) * 0.5, rng.normal(size=(3, 2)) * 0.5]
    base = oracle.gin_step(g, x, w1s, w2s, y, want_dx=True)
    for l in (0, 1):
        # a row of T that the inner ReLU zeroed gives a pre-activation of exactly 0 that no small
        # step moves: not a kink for the difference quotient
        pre2 = np.abs(base["T"][l] @ w2s[l])
        if np.min(np.abs(base["Z"][l] @ w1s[l])) < 1e-4 or \
                (l == 0 and np.min(pre2[pre2 > 0]) < 1e-4):
            pytest.skip("sample too close to a ReLU kink")
    _fd_check(lambda: oracle.gin_step(g, x, w1s, w2s, y, backward=False)["loss"], w1s + w2s + [x],
              base["dW1"] + base["dW2"] + [base["dX"]])


def test_sage_gradient_fd_on_a_directed_graph_pins_the_transposed_mean():
    """On a directed graph D^-1 A and its transpose differ in pattern AND values."""
    rng = np.random.default_rng(81)
    n = 10
    src, dst = rng.integers(0, n, 25), rng.integers(0, n, 25)
    g = oracle.normalize_mean(oracle.build_csr(src, dst, n, False, False))
    x = rng.normal(size=(n, 3))
    ws = [rng.normal(size=(6, 3)), rng.normal(size=(6, 2))]
    y = rng.integers(0, 2, n).astype(np.int32)
    base = oracle.sage_step(g, x, ws, y, want_dx=True)
    if np.min(np.abs(base["X"][0] @ ws[0])) < 1e-4:
        pytest.skip("sample too close to a ReLU kink")
    _fd_check(lambda: oracle.sage_step(g, x, ws, y, backward=False)["loss"], [x], [base["dX"]])


# ------------------------------------------------------------------------------------------
# dropout mask of the S-SpMM's forward use (Sec. 3.2.1): the generator and the bitmap
# ------------------------------------------------------------------------------------------
def test_splitmix64_published_test_vector():
    want = [int(l, 16) for l in open(os.path.join(GOLD, "splitmix64_seed0.txt"))
            if l.strip() and not l.startswith("#")]
    assert [oracle.splitmix64(0, i) for i in range(len(want))] == want
    # a seed shifts the sequence: output i of seed s + k * gamma is output i + k of seed s
    gamma = 0x9E3779B97F4A7C15
    assert oracle.splitmix64((5 * gamma) % 2 ** 64, 2) == oracle.splitmix64(0, 7)


def test_dropout_bitmap_is_the_thresholded_generator_and_has_the_right_density():
    n, m, seed = 257, 70, 12345
    for keep in (0.0, 0.25, 0.5, 0.9, 1.0):
        bits = oracle.dropout_bitmap(seed, n, m, keep)
        got = unpack_bits(bits, m)
        # bits past the last column are clear
        assert np.all(unpack_bits(bits, 32 * bits.shape[1])[:, m:] == 0)
        # element by element from the generator (python integers), on a sample of the rows
        thr = int(keep * 2 ** 32)
        for v in (0, 1, 100, n - 1):
            ref = [(oracle.splitmix64(seed, v * m + j) >> 32) < thr for j in range(m)]
            assert list(got[v].astype(bool)) == ref
        if keep in (0.0, 1.0):
            assert got.sum() == (0 if keep == 0.0 else n * m)
        else:  # binomial: 5 standard deviations
            sd = math.sqrt(n * m * keep * (1 - keep))
            assert abs(got.sum() - n * m * keep) < 5 * sd
    # another seed gives another mask; the same seed the same one
    a = oracle.dropout_bitmap(1, n, m, 0.5)
    assert np.array_equal(a, oracle.dropout_bitmap(1, n, m, 0.5))
    b = unpack_bits(oracle.dropout_bitmap(2, n, m, 0.5), m)
    agree = (unpack_bits(a, m) == b).mean()
    assert 0.45 < agree < 0.55
    # rows are not copies of each other, columns neither (index = v * m + j, not v or j alone)
    g = unpack_bits(a, m).astype(np.float64)
    assert abs(np.corrcoef(g[0::2].ravel()[:8000], g[1::2].ravel()[:8000])[0, 1]) < 0.05


def test_dropout_mask_in_the_sspmm_keeps_about_half_of_the_outputs():
    rng = np.random.default_rng(7)
    n = 50
    g = oracle.normalize(oracle.build_csr(rng.integers(0, n, 200), rng.integers(0, n, 200), n))
    h = rng.normal(size=(n, 40))
    bits = oracle.dropout_bitmap(99, n, 40, 0.5)
    z = oracle.sspmm(g, h, bits)
    full = oracle.spmm(g, h)
    keep = unpack_bits(bits, 40).astype(bool)
    np.testing.assert_allclose(z, np.where(keep, full, 0.0), rtol=0, atol=0)
    assert 0.4 < keep.mean() < 0.6


def test_dropout_gcn_forward_vs_dense_and_gradients_vs_finite_differences():
    """The masked step: forward against the dense definition with the mask read back bit by bit,
    gradients against central differences (the mask is a constant of the step)."""
    g, src, dst, x, ws, y = _tiny_problem(91)
    seed, keep = 777, 0.6
    base = oracle.gcn_dropout_step(g, x, ws, y, seed, keep, want_dx=True)
    ah = dense_ahat(dense_atilde(src, dst, g.n))
    h = x
    for l, w in enumerate(ws):
        m = unpack_bits(oracle.dropout_bitmap(seed + l, g.n, w.shape[0], keep), w.shape[0])
        h = ((ah @ h) * m) @ w
        if l < len(ws) - 1:
            h = np.maximum(h, 0)
    np.testing.assert_allclose(base["logits"], h, rtol=1e-11, atol=1e-13)
    for l in (1, 2):
        pre = base["Z"][l - 1] @ ws[l - 1]
        if np.min(np.abs(pre[pre != 0])) < 1e-4:
            pytest.skip("sample too close to a ReLU kink")
    _fd_check(lambda: oracle.gcn_dropout_step(g, x, ws, y, seed, keep, backward=False)["loss"],
              ws + [x], base["dW"] + [base["dX"]])
    # keep = 1 is the plain step
    plain = oracle.gcn_step(g, x, ws, y)
    full = oracle.gcn_dropout_step(g, x, ws, y, seed, 1.0)
    np.testing.assert_allclose(full["logits"], plain["logits"], rtol=1e-12, atol=1e-14)
    for a, b in zip(full["dW"], plain["dW"]):
        np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-14)
