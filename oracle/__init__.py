"""ctypes binding of the CPU oracle (``gcn_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports this module and this
module never imports the product package.

All floating-point tensors are float64 numpy arrays (C-contiguous, ld == number of columns).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_gcn.so")
_lib = None

Q_NONE, Q_F32, Q_BF16 = 0, 1, 2


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "gcn_oracle.cpp")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", "-o", _SO, src]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        lib = ctypes.CDLL(_SO)
        p, i64, i32, u32, u64 = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32,
                                 ctypes.c_uint64)
        lib.oracle_num_threads.restype = i32
        lib.oracle_set_num_threads.argtypes = [i32]
        lib.oracle_build_csr.argtypes = [p, p, u64, u32, i32, i32, p, p]
        lib.oracle_build_csr.restype = i64
        lib.oracle_normalize.argtypes = [p, p, u32, p, p, p, p]
        lib.oracle_normalize.restype = None
        lib.oracle_transpose.argtypes = [p, p, p, u32, p, p, p]
        lib.oracle_transpose.restype = None
        lib.oracle_spmm.argtypes = [p, p, p, p, i64, p, i64, i64, i64, i64, i64, i32]
        lib.oracle_spmm.restype = None
        lib.oracle_rcm.argtypes = [p, p, u32, p]
        lib.oracle_rcm.restype = None
        lib.oracle_bandwidth.argtypes = [p, p, u32, p]
        lib.oracle_bandwidth.restype = i64
        lib.oracle_pipeline_stages.argtypes = [i64, i64]
        lib.oracle_pipeline_stages.restype = i64
        lib.oracle_relu_bitmap.argtypes = [p, i64, i64, i64, p, i64]
        lib.oracle_relu_bitmap.restype = None
        lib.oracle_splitmix64.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        lib.oracle_splitmix64.restype = ctypes.c_uint64
        lib.oracle_dropout_bitmap.argtypes = [ctypes.c_uint64, i64, i64, ctypes.c_double, p, i64]
        lib.oracle_dropout_bitmap.restype = None
        lib.oracle_sspmm.argtypes = [p, p, p, p, i64, p, i64, i64, i64, i64, i64, p, i64, i32]
        lib.oracle_sspmm.restype = None
        lib.oracle_update_fwd.argtypes = [p, i64, p, i64, p, i64, i64, i64, i64, i32, i32]
        lib.oracle_update_fwd.restype = None
        lib.oracle_relu_grad.argtypes = [p, i64, p, i64, p, i64, i64, i64, i32]
        lib.oracle_relu_grad.restype = None
        lib.oracle_update_dgrad.argtypes = [p, i64, p, i64, p, i64, i64, i64, i64, i32]
        lib.oracle_update_dgrad.restype = None
        lib.oracle_update_wgrad.argtypes = [p, i64, p, i64, p, i64, i64, i64, i64]
        lib.oracle_update_wgrad.restype = None
        lib.oracle_softmax_xent.argtypes = [p, i64, p, i64, i64, p, i64]
        lib.oracle_softmax_xent.restype = ctypes.c_double
        lib.oracle_gcn_step.argtypes = [p, p, p, p, p, p, i64, i32, p, p, p, p, p, p, p, p, i32, i32, p]
        lib.oracle_gcn_step.restype = ctypes.c_double
        _lib = lib
    return _lib


def num_threads() -> int:
    return _load().oracle_num_threads()


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(n)


def _p(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    assert a.ndim == 2
    return a


class Graph:
    """Sorted CSR of A_tilde with its normalisation (and, if asked, the transpose)."""

    def __init__(self, rowptr, col, n):
        self.n = int(n)
        self.rowptr = rowptr
        self.col = col
        self.nnz = int(rowptr[-1])
        self.deg = self.dinv = self.val = self.val_f32 = None
        self.t_rowptr = self.t_col = self.t_val = None


def build_csr(src, dst, n, symmetrize=True, self_loops=True) -> Graph:
    src = np.ascontiguousarray(src, dtype=np.uint32)
    dst = np.ascontiguousarray(dst, dtype=np.uint32)
    e = len(src)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    col = np.empty((2 if symmetrize else 1) * e + n, dtype=np.uint32)
    nnz = _load().oracle_build_csr(_p(src), _p(dst), e, n, int(symmetrize), int(self_loops),
                                   _p(rowptr), _p(col))
    if nnz < 0:
        raise ValueError("edge endpoint out of range")
    return Graph(rowptr, col[:nnz].copy(), n)


def normalize(g: Graph) -> Graph:
    g.deg = np.empty(g.n, dtype=np.uint32)
    g.dinv = np.empty(g.n, dtype=np.float64)
    g.val = np.empty(g.nnz, dtype=np.float64)
    g.val_f32 = np.empty(g.nnz, dtype=np.float32)
    _load().oracle_normalize(_p(g.rowptr), _p(g.col), g.n, _p(g.deg), _p(g.dinv), _p(g.val),
                             _p(g.val_f32))
    return g


def transpose(g: Graph) -> Graph:
    g.t_rowptr = np.empty(g.n + 1, dtype=np.int64)
    g.t_col = np.empty(g.nnz, dtype=np.uint32)
    g.t_val = np.empty(g.nnz, dtype=np.float64)
    _load().oracle_transpose(_p(g.rowptr), _p(g.col), _p(g.val), g.n, _p(g.t_rowptr),
                             _p(g.t_col), _p(g.t_val))
    return g


def spmm(g: Graph, H, c0=0, c1=None, r0=0, r1=None, transposed=False, q=Q_NONE, out=None):
    """Z[r0:r1, c0:c1] = (A_hat or A_hat^T)[r0:r1, :] @ H[:, c0:c1]; other entries untouched."""
    H = _f64(H)
    c1 = H.shape[1] if c1 is None else c1
    r1 = g.n if r1 is None else r1
    Z = np.zeros_like(H) if out is None else out
    if transposed:
        if g.t_rowptr is None:
            transpose(g)
        rp, cl, vl = g.t_rowptr, g.t_col, g.t_val
    else:
        rp, cl, vl = g.rowptr, g.col, g.val
    _load().oracle_spmm(_p(rp), _p(cl), _p(vl), _p(H), H.shape[1], _p(Z), Z.shape[1], c0, c1, r0,
                        r1, q)
    return Z


def rcm(g: Graph):
    """Reverse Cuthill-McKee positions pos[v] (uint32[n]) of the nodes of g."""
    pos = np.empty(g.n, dtype=np.uint32)
    _load().oracle_rcm(_p(g.rowptr), _p(g.col), g.n, _p(pos))
    return pos


def bandwidth(g: Graph, pos=None) -> int:
    """max |pos[u] - pos[v]| over the stored entries; pos None = identity."""
    if pos is not None:
        pos = np.ascontiguousarray(pos, dtype=np.uint32)
    return int(_load().oracle_bandwidth(_p(g.rowptr), _p(g.col), g.n,
                                        _p(pos) if pos is not None else None))


def pipeline_stages(n: int, b: int) -> int:
    """Smallest number of batches s with (n - b) / (2 n) >= 1 / s; 0 if there is none."""
    return int(_load().oracle_pipeline_stages(n, b))


def relu_bitmap(X):
    """uint32 bitmap [n, ceil(m / 32)]: bit (j % 32) of word j // 32 of row v is X[v, j] > 0."""
    X = _f64(X)
    n, m = X.shape
    bits = np.zeros((n, (m + 31) // 32), dtype=np.uint32)
    _load().oracle_relu_bitmap(_p(X), m, n, m, _p(bits), bits.shape[1])
    return bits


def splitmix64(seed: int, i: int) -> int:
    """Output i (from 0) of SplitMix64 started at `seed`."""
    return int(_load().oracle_splitmix64(seed & (2 ** 64 - 1), i))


def dropout_bitmap(seed: int, n: int, m: int, keep: float):
    """uint32 bitmap [n, ceil(m / 32)] of the kept elements of an n x m tensor: element (v, j) is
    kept iff splitmix64(seed, v * m + j) >> 32 < keep * 2^32."""
    bits = np.zeros((n, (m + 31) // 32), dtype=np.uint32)
    _load().oracle_dropout_bitmap(seed & (2 ** 64 - 1), n, m, float(keep), _p(bits), bits.shape[1])
    return bits


def sspmm(g: Graph, H, bits, c0=0, c1=None, r0=0, r1=None, transposed=False, q=Q_NONE, out=None):
    """S-SpMM: Z[r0:r1, c0:c1] = ((A_hat or A_hat^T) @ H)[r0:r1, c0:c1] masked by the bitmap."""
    H = _f64(H)
    bits = np.ascontiguousarray(bits, dtype=np.uint32)
    c1 = H.shape[1] if c1 is None else c1
    r1 = g.n if r1 is None else r1
    Z = np.zeros_like(H) if out is None else out
    if transposed:
        if g.t_rowptr is None:
            transpose(g)
        rp, cl, vl = g.t_rowptr, g.t_col, g.t_val
    else:
        rp, cl, vl = g.rowptr, g.col, g.val
    _load().oracle_sspmm(_p(rp), _p(cl), _p(vl), _p(H), H.shape[1], _p(Z), Z.shape[1], c0, c1, r0,
                         r1, _p(bits), bits.shape[1], q)
    return Z


def update_fwd(Z, W, relu: bool, q=Q_NONE):
    Z, W = _f64(Z), _f64(W)
    n, k = Z.shape
    m = W.shape[1]
    out = np.empty((n, m), dtype=np.float64)
    _load().oracle_update_fwd(_p(Z), k, _p(W), m, _p(out), m, n, k, m, int(relu), q)
    return out


def relu_grad(G, Href, q=Q_NONE):
    G = _f64(G)
    Href = None if Href is None else _f64(Href)
    n, m = G.shape
    out = np.empty((n, m), dtype=np.float64)
    _load().oracle_relu_grad(_p(G), m, _p(Href), m, _p(out), m, n, m, q)
    return out


def update_dgrad(dP, W, q=Q_NONE):
    dP, W = _f64(dP), _f64(W)
    n, m = dP.shape
    k = W.shape[0]
    out = np.empty((n, k), dtype=np.float64)
    _load().oracle_update_dgrad(_p(dP), m, _p(W), m, _p(out), k, n, k, m, q)
    return out


def update_wgrad(Z, dP):
    Z, dP = _f64(Z), _f64(dP)
    n, k = Z.shape
    m = dP.shape[1]
    out = np.empty((k, m), dtype=np.float64)
    _load().oracle_update_wgrad(_p(Z), k, _p(dP), m, _p(out), m, n, k, m)
    return out


def softmax_xent(logits, labels, want_grad=True):
    logits = _f64(logits)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    n, c = logits.shape
    d = np.empty((n, c), dtype=np.float64) if want_grad else None
    loss = _load().oracle_softmax_xent(_p(logits), c, _p(labels), n, c, _p(d), c)
    return loss, d


def gcn_step(g: Graph, X, Ws, labels, want_dx=False, linear=False, q=Q_NONE, backward=True,
             relu_sign=None):
    """One forward(+backward) pass of an L-layer GCN.  Returns a dict with loss, logits,
    Z (list), H (list, H[0] = X), dW (list) and dX.  relu_sign: optional list of L + 1 entries
    (None or an n x dims[l] array for l = 1..L-1) whose signs replace those of H_l in the
    backward pass's ReLU derivative (see oracle_gcn_step)."""
    X = _f64(X)
    Ws = [_f64(w) for w in Ws]
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    L = len(Ws)
    n = g.n
    dims = np.array([X.shape[1]] + [w.shape[1] for w in Ws], dtype=np.int64)
    for l, w in enumerate(Ws):
        assert w.shape[0] == dims[l]
    if g.t_rowptr is None:
        transpose(g)
    Zs = [np.empty((n, int(dims[l])), dtype=np.float64) for l in range(L)]
    Hs = [X] + [np.empty((n, int(dims[l + 1])), dtype=np.float64) for l in range(L)]
    dWs = [np.empty_like(w) for w in Ws] if backward else None
    dX = np.empty_like(X) if (want_dx and backward) else None
    PtrArr = ctypes.c_void_p * L
    PtrArr1 = ctypes.c_void_p * (L + 1)
    w_arr = PtrArr(*[w.ctypes.data for w in Ws])
    z_arr = PtrArr(*[z.ctypes.data for z in Zs])
    h_arr = PtrArr1(*[h.ctypes.data for h in Hs])
    dw_arr = PtrArr(*[d.ctypes.data for d in dWs]) if backward else None
    sign_arr = None
    if relu_sign is not None:
        assert len(relu_sign) == L + 1
        signs = [None if a is None else _f64(a) for a in relu_sign]
        for l, a in enumerate(signs):
            assert a is None or (0 < l < L and a.shape == (n, int(dims[l])))
        sign_arr = PtrArr1(*[None if a is None else a.ctypes.data for a in signs])
    loss = _load().oracle_gcn_step(_p(g.rowptr), _p(g.col), _p(g.val), _p(g.t_rowptr),
                                   _p(g.t_col), _p(g.t_val), n, L, _p(dims), _p(X), w_arr, _p(labels),
                                   z_arr, h_arr, dw_arr, _p(dX), int(linear), q, sign_arr)
    return {"loss": loss, "logits": Hs[L], "Z": Zs, "H": Hs, "dW": dWs, "dX": dX}


# ------------------------------------------------------------------------------------------
# The two other architectures of the paper's experiments (Sec. 4, "The Model and Datasets":
# GCN, GraphSAGE, GIN).  The paper prints no equations for them, so these follow the works it
# cites: GraphSAGE with the mean aggregator and concatenation (Hamilton et al. 2017, Alg. 1,
# without the optional output normalisation), GIN with a two-layer perceptron (Xu et al. 2019,
# Eq. 4.1).  Plain numpy in fp64 on top of spmm(); matmul is the library primitive of each
# update.  No bias, no dropout, ReLU between layers and none after the last, as in gcn_step.
# ------------------------------------------------------------------------------------------
def _rows_of_entries(g: Graph):
    return np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))


def normalize_mean(g: Graph) -> Graph:
    """A_hat = D^-1 A on the stored pattern: every stored entry of row u is 1 / deg(u), deg(u)
    the number of stored entries of the row (the neighbors of u; u itself only if the graph was
    built with self-loops).  val_f32 is the fp32 encoding (float)(1 / (double)deg)."""
    deg = np.diff(g.rowptr).astype(np.uint32)
    rows = _rows_of_entries(g)
    g.deg = deg
    with np.errstate(divide="ignore"):
        inv = np.where(deg > 0, 1.0 / deg.astype(np.float64), 0.0)
    g.dinv = inv
    g.val = inv[rows]
    g.val_f32 = inv.astype(np.float32)[rows]
    g.t_rowptr = g.t_col = g.t_val = None
    return g


def normalize_sum(g: Graph, eps: float = 0.0) -> Graph:
    """A_hat = A + eps I on the stored pattern of A + I: 1 for a neighbor, 1 + eps for the node
    itself (GIN's (1 + eps) h_v + sum of the neighbors).  val_f32 adds in fp32."""
    rows = _rows_of_entries(g)
    diag = rows == g.col.astype(np.int64)
    g.deg = np.diff(g.rowptr).astype(np.uint32)
    g.dinv = np.zeros(g.n, dtype=np.float64)
    g.val = np.where(diag, 1.0 + float(eps), 1.0)
    g.val_f32 = np.where(diag, np.float32(1.0) + np.float32(eps), np.float32(1.0)).astype(np.float32)
    g.t_rowptr = g.t_col = g.t_val = None
    return g


def _loss_and_grad(logits, labels, backward):
    loss, d = softmax_xent(logits, labels, want_grad=backward)
    return loss, d


def _sign_of(relu_sign, key, l, own):
    """The array whose signs decide a ReLU derivative: the caller's stand-in (see
    oracle_gcn_step: relu_sign) when there is one for layer l, else the oracle's own activation."""
    if relu_sign is None:
        return own
    a = relu_sign.get(key, None) if isinstance(relu_sign, dict) else relu_sign
    if a is None or a[l] is None:
        return own
    a = np.asarray(a[l], dtype=np.float64)
    assert a.shape == own.shape
    return a


def sage_step(g: Graph, X, Ws, labels, want_dx=False, backward=True, relu_sign=None):
    """L-layer GraphSAGE (mean aggregator).  g: normalize_mean'd graph WITHOUT self-loops.
    Ws[l] has 2 d_l rows: the first d_l multiply the node's own features, the last d_l the mean
    of its neighbors' (the concatenation [h_v | mean]).
        M_l = A_hat H_l;  X_l = [H_l | M_l];  P_l = X_l W_l;  H_{l+1} = relu(P_l), last: P_l.
    Backward: dW_l = X_l^T dP_l;  dX_l = dP_l W_l^T;  dH_l = dX_l[:, :d] + A_hat^T dX_l[:, d:];
    dP_{l-1} = dH_l (.) 1[H_l > 0].  relu_sign: optional list indexed like H whose entries stand
    in for H_l in that derivative."""
    X = _f64(X)
    Ws = [_f64(w) for w in Ws]
    L = len(Ws)
    if g.t_rowptr is None:
        transpose(g)
    Hs, Xs = [X], []
    for l, w in enumerate(Ws):
        d = Hs[l].shape[1]
        assert w.shape[0] == 2 * d
        xc = np.concatenate([Hs[l], spmm(g, Hs[l])], axis=1)
        p = xc @ w
        Xs.append(xc)
        Hs.append(np.maximum(p, 0.0) if l < L - 1 else p)
    loss, dP = _loss_and_grad(Hs[L], labels, backward)
    out = {"loss": loss, "logits": Hs[L], "H": Hs, "X": Xs, "dW": None, "dX": None}
    if not backward:
        return out
    dWs = [None] * L
    for l in range(L - 1, -1, -1):
        d = Hs[l].shape[1]
        dWs[l] = Xs[l].T @ dP
        if l == 0 and not want_dx:
            break
        dXc = dP @ Ws[l].T
        dH = dXc[:, :d] + spmm(g, np.ascontiguousarray(dXc[:, d:]), transposed=True)
        if l == 0:
            out["dX"] = dH
            break
        dP = dH * (_sign_of(relu_sign, "H", l, Hs[l]) > 0)
    out["dW"] = dWs
    return out


def gin_step(g: Graph, X, W1s, W2s, labels, want_dx=False, backward=True, relu_sign=None):
    """L-layer GIN.  g: normalize_sum'd graph WITH self-loops (their value carries 1 + eps).
        Z_l = A_hat H_l;  T_l = relu(Z_l W1_l);  P_l = T_l W2_l;  H_{l+1} = relu(P_l), last: P_l.
    Backward: dW2_l = T_l^T dP_l;  dT_l = dP_l W2_l^T (.) 1[T_l > 0];  dW1_l = Z_l^T dT_l;
    dZ_l = dT_l W1_l^T;  dH_l = A_hat^T dZ_l;  dP_{l-1} = dH_l (.) 1[H_l > 0].  relu_sign: optional
    dict {"H": list indexed like H, "T": list indexed like T} of stand-ins for the two derivatives."""
    X = _f64(X)
    W1s = [_f64(w) for w in W1s]
    W2s = [_f64(w) for w in W2s]
    L = len(W1s)
    if g.t_rowptr is None:
        transpose(g)
    Hs, Zs, Ts = [X], [], []
    for l in range(L):
        z = spmm(g, Hs[l])
        t = np.maximum(z @ W1s[l], 0.0)
        p = t @ W2s[l]
        Zs.append(z)
        Ts.append(t)
        Hs.append(np.maximum(p, 0.0) if l < L - 1 else p)
    loss, dP = _loss_and_grad(Hs[L], labels, backward)
    out = {"loss": loss, "logits": Hs[L], "H": Hs, "Z": Zs, "T": Ts, "dW1": None, "dW2": None,
           "dX": None}
    if not backward:
        return out
    dW1s, dW2s = [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        dW2s[l] = Ts[l].T @ dP
        dT = (dP @ W2s[l].T) * (_sign_of(relu_sign, "T", l, Ts[l]) > 0)
        dW1s[l] = Zs[l].T @ dT
        if l == 0 and not want_dx:
            break
        dH = spmm(g, dT @ W1s[l].T, transposed=True)
        if l == 0:
            out["dX"] = dH
            break
        dP = dH * (_sign_of(relu_sign, "H", l, Hs[l]) > 0)
    out["dW1"], out["dW2"] = dW1s, dW2s
    return out


def gcn_dropout_step(g: Graph, X, Ws, labels, seed: int, keep: float, want_dx=False, backward=True,
                     relu_sign=None):
    """L-layer GCN in the order of Algorithm 2 with the output mask of Sec. 3.2.1 / Eq. 4 on every
    aggregation: Z_l = (A_hat H_l) (.) M_l, M_l = dropout_bitmap(seed + l, n, d_l, keep), P_l =
    Z_l W_l, H_{l+1} = relu(P_l) (none after the last).  The mask is a constant of the step, so
    the backward pass multiplies by it where the forward pass did:
    dW_l = Z_l^T dP_l;  dZ_l = dP_l W_l^T;  dH_l = A_hat^T (dZ_l (.) M_l);  dP_{l-1} = dH_l (.) 1[H_l > 0].
    No rescaling by 1 / keep (Eq. 4 multiplies by the 0/1 mask)."""
    X = _f64(X)
    Ws = [_f64(w) for w in Ws]
    L = len(Ws)
    n = g.n
    if g.t_rowptr is None:
        transpose(g)
    bits = [dropout_bitmap(seed + l, n, Ws[l].shape[0], keep) for l in range(L)]
    masks = []
    for l in range(L):
        d = Ws[l].shape[0]
        cols = np.arange(d)
        masks.append(((bits[l][:, cols // 32] >> (cols % 32).astype(np.uint32)) & 1).astype(np.float64))
    Hs, Zs = [X], []
    for l, w in enumerate(Ws):
        z = sspmm(g, Hs[l], bits[l])
        p = z @ w
        Zs.append(z)
        Hs.append(np.maximum(p, 0.0) if l < L - 1 else p)
    loss, dP = _loss_and_grad(Hs[L], labels, backward)
    out = {"loss": loss, "logits": Hs[L], "H": Hs, "Z": Zs, "M": masks, "dW": None, "dX": None}
    if not backward:
        return out
    dWs = [None] * L
    for l in range(L - 1, -1, -1):
        dWs[l] = Zs[l].T @ dP
        if l == 0 and not want_dx:
            break
        dH = spmm(g, (dP @ Ws[l].T) * masks[l], transposed=True)
        if l == 0:
            out["dX"] = dH
            break
        dP = dH * (_sign_of(relu_sign, "H", l, Hs[l]) > 0)
    out["dW"] = dWs
    return out
