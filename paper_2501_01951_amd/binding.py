"""ctypes binding of libmixgcn.so: argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmixgcn.so")
_lib = None

F32, BF16 = 0, 1
OP_FWD, OP_FWD_RELU, OP_DGRAD, OP_WGRAD = 0, 1, 2, 3
SYMMETRIZE, ADD_SELF_LOOPS, BUILD_TRANSPOSE, INPUT_ON_HOST = 1, 2, 4, 8
NORM_SYM, NORM_MEAN, NORM_SUM = 0, 1, 2
EPI_RELU, EPI_ACCUMULATE = 1, 2
ARITH_FP32, ARITH_BF16X3 = 0, 1
AGG_FIRST, UPDATE_FIRST = 0, 1


class MixGCNError(RuntimeError):
    def __init__(self, code: int, where: str):
        lib = load_library()
        msg = lib.mixgcn_last_error().decode()
        kind = lib.mixgcn_strerror(code).decode()
        super().__init__(f"{where}: {kind} ({code}): {msg}")
        self.code = code


class _GraphView(ctypes.Structure):
    _fields_ = [
        ("n_nodes", ctypes.c_uint32), ("flags", ctypes.c_uint32), ("nnz", ctypes.c_int64),
        ("rowptr", ctypes.c_void_p), ("col", ctypes.c_void_p), ("val", ctypes.c_void_p),
        ("deg", ctypes.c_void_p), ("dinv", ctypes.c_void_p), ("t_rowptr", ctypes.c_void_p),
        ("t_col", ctypes.c_void_p), ("t_val", ctypes.c_void_p),
    ]


class LayerDesc(ctypes.Structure):
    _fields_ = [
        ("f_in", ctypes.c_int32), ("f_out", ctypes.c_int32), ("ld_h", ctypes.c_int64),
        ("ld_z", ctypes.c_int64), ("ld_out", ctypes.c_int64), ("ld_w", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("relu", ctypes.c_int32), ("n_chunks", ctypes.c_int32),
        ("order", ctypes.c_int32),
    ]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libmixgcn.so; builds it first only if it has never been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build

        _build.build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u32, u64, f32 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                   ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float)
    lib.mixgcn_version.restype = ctypes.c_int
    lib.mixgcn_last_error.restype = ctypes.c_char_p
    lib.mixgcn_strerror.restype = ctypes.c_char_p
    lib.mixgcn_strerror.argtypes = [ctypes.c_int]
    lib.mixgcn_build_csr.argtypes = [vp, vp, u64, u32, u32, vp, ctypes.POINTER(vp)]
    lib.mixgcn_normalize.argtypes = [vp, ctypes.c_int, vp]
    lib.mixgcn_normalize_mode.argtypes = [vp, ctypes.c_int, ctypes.c_float, vp]
    lib.mixgcn_aggregate_ex.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, i64, vp, i64, i32, i32,
                                        i64, i64, ctypes.c_int, vp]
    lib.mixgcn_aggregate.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, i64, vp, i64, i32, i32,
                                     i64, i64, vp]
    lib.mixgcn_graph_reserve_streams.argtypes = [vp, i32]
    lib.mixgcn_graph_reserve_streams.restype = ctypes.c_int
    lib.mixgcn_aggregate_scratch_bytes.argtypes = [i64]
    lib.mixgcn_aggregate_scratch_bytes.restype = i64
    lib.mixgcn_aggregate_scratch_need.argtypes = [ctypes.c_int, i32, i64, i64]
    lib.mixgcn_aggregate_scratch_need.restype = i64
    lib.mixgcn_aggregate_static.argtypes = lib.mixgcn_aggregate.argtypes
    lib.mixgcn_aggregate_static.restype = ctypes.c_int
    lib.mixgcn_aggregate_masked.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, i64, vp, i64, i32,
                                            i32, i64, i64, vp, i64, vp]
    lib.mixgcn_relu_bitmap.argtypes = [ctypes.c_int, vp, i64, i64, i32, vp, i64, vp]
    lib.mixgcn_dropout_bitmap.argtypes = [u64, i64, i32, ctypes.c_double, vp, i64, vp]
    lib.mixgcn_apply_bitmap.argtypes = [ctypes.c_int, vp, i64, i64, i32, vp, i64, vp]
    lib.mixgcn_reorder_rcm.argtypes = [vp, vp, vp]
    lib.mixgcn_bandwidth.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int64), vp]
    lib.mixgcn_pipeline_stages.argtypes = [i64, i64]
    lib.mixgcn_pipeline_stages.restype = i64
    lib.mixgcn_relabel_edges.argtypes = [vp, vp, u64, vp, u32, vp, vp, vp]
    lib.mixgcn_permute_rows.argtypes = [ctypes.c_int, vp, i64, vp, i64, i64, i32, vp, vp]
    dp = ctypes.POINTER(ctypes.c_double)
    lib.mixgcn_measure_peaks.argtypes = [dp, dp, dp, dp, dp, dp, vp]
    lib.mixgcn_update.argtypes = [ctypes.c_int, ctypes.c_int, vp, i64, vp, i64, vp, i64, i64, i32,
                                  i32, vp, i64, f32, vp]
    lib.mixgcn_layer_fwd.argtypes = [vp, ctypes.POINTER(LayerDesc), vp, vp, vp, vp, vp]
    lib.mixgcn_layer_bwd.argtypes = [vp, ctypes.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp, vp, vp]
    lib.mixgcn_forward_pipelined.argtypes = [vp, i32, ctypes.POINTER(LayerDesc), vp, vp, vp, vp, i64, vp]
    lib.mixgcn_backward_pipelined.argtypes = [vp, i32, ctypes.POINTER(LayerDesc), vp, vp, vp, vp, vp,
                                              vp, vp, i64, vp]
    lib.mixgcn_pipeline_window.argtypes = [i64, i32, i64, i32, ctypes.POINTER(ctypes.c_int64),
                                           ctypes.POINTER(ctypes.c_int64),
                                           ctypes.POINTER(ctypes.c_int32),
                                           ctypes.POINTER(ctypes.c_int32)]
    lib.mixgcn_softmax_xent.argtypes = [ctypes.c_int, vp, i64, vp, i64, i32, vp, i64, vp, vp]
    lib.mixgcn_set_update_arith.argtypes = [ctypes.c_int]
    lib.mixgcn_set_update_arith.restype = ctypes.c_int
    lib.mixgcn_set_aggregate_whole_rows.argtypes = [ctypes.c_int]
    lib.mixgcn_set_aggregate_whole_rows.restype = ctypes.c_int
    lib.mixgcn_graph_info.argtypes = [vp, ctypes.POINTER(_GraphView)]
    lib.mixgcn_graph_free.argtypes = [vp]
    lib.mixgcn_pipeline_create.argtypes = [vp, vp, ctypes.POINTER(vp)]
    lib.mixgcn_pipeline_destroy.argtypes = [vp]
    lib.mixgcn_stream_create_cu_subset.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                   ctypes.POINTER(vp)]
    lib.mixgcn_stream_destroy.argtypes = [vp]
    lib.mixgcn_pipeline_timing.argtypes = [vp, ctypes.c_int]
    lib.mixgcn_pipeline_timing_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                                ctypes.POINTER(ctypes.c_int64)]
    for name in ("build_csr", "normalize", "aggregate", "aggregate_masked", "relu_bitmap",
                 "measure_peaks", "reorder_rcm", "bandwidth", "relabel_edges", "permute_rows",
                 "update", "layer_fwd", "layer_bwd",
                 "softmax_xent", "graph_info", "graph_free", "pipeline_create", "pipeline_destroy",
                 "pipeline_timing", "pipeline_timing_read", "stream_create_cu_subset", "stream_destroy"):
        getattr(lib, "mixgcn_" + name).restype = ctypes.c_int
    _lib = lib
    return lib


def version() -> int:
    return load_library().mixgcn_version()


def measure_peaks(stream=None):
    """Rates this device sustains on kernels that do nothing else, as a dict: streaming read and
    copy, random 128-byte gathers from L2 and from HBM (GB/s), fp32 and bf16 MFMA chains
    (TFLOP/s).  A measurement aid for bench.py."""
    v = [ctypes.c_double() for _ in range(6)]
    _check(load_library().mixgcn_measure_peaks(*[ctypes.byref(x) for x in v], _stream(stream)),
           "measure_peaks")
    names = ("read_GBps", "copy_GBps", "gather_l2_GBps", "gather_hbm_GBps", "mfma_f32_TFLOPs",
             "mfma_bf16_TFLOPs")
    return {k: x.value for k, x in zip(names, v)}


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise MixGCNError(rc, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ld(t) -> int:
    assert t.dim() == 2 and t.stride(1) == 1, "row-major 2-D tensor expected"
    return t.stride(0)


def _dtype_of(t) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


class _DevArray:
    """Exposes a library-owned device array through __cuda_array_interface__."""

    def __init__(self, ptr, count, typestr):
        self.__cuda_array_interface__ = {"shape": (count,), "typestr": typestr,
                                         "data": (int(ptr), False), "version": 2}


_TYPESTR = {torch.int64: "<i8", torch.int32: "<i4", torch.float32: "<f4"}


def _view_array(ptr, count, dtype, device):
    """Copy of a library-owned device array as a torch tensor (for tests and inspection)."""
    if not count:
        return torch.empty(0, dtype=dtype, device=device)
    return torch.as_tensor(_DevArray(ptr, count, _TYPESTR[dtype]), device=device).clone()


class Graph:
    """Owner of a mixgcn_graph handle."""

    def __init__(self, handle, device):
        self._h = handle
        self.device = device

    def info(self) -> _GraphView:
        v = _GraphView()
        _check(load_library().mixgcn_graph_info(self._h, ctypes.byref(v)), "graph_info")
        return v

    @property
    def n(self) -> int:
        return self.info().n_nodes

    @property
    def nnz(self) -> int:
        return self.info().nnz

    def arrays(self, transpose: bool = False):
        """Copies of rowptr, col, val (and deg, dinv) as torch tensors."""
        torch.cuda.synchronize()
        v = self.info()
        rp, cl, vl = (v.t_rowptr, v.t_col, v.t_val) if transpose else (v.rowptr, v.col, v.val)
        out = {
            "rowptr": _view_array(rp, v.n_nodes + 1, torch.int64, self.device),
            "col": _view_array(cl, v.nnz, torch.int32, self.device),
        }
        if vl:
            out["val"] = _view_array(vl, v.nnz, torch.float32, self.device)
        if v.deg:
            out["deg"] = _view_array(v.deg, v.n_nodes, torch.int32, self.device)
            out["dinv"] = _view_array(v.dinv, v.n_nodes, torch.float32, self.device)
        torch.cuda.synchronize()
        return out

    def free(self):
        if self._h:
            load_library().mixgcn_graph_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def cu_subset_stream(lo: int, hi: int, groups: int):
    """torch stream whose kernels run only on the CUs c with (c / 8) % groups in [lo, hi).
    The stream lives until the process ends."""
    h = ctypes.c_void_p()
    _check(load_library().mixgcn_stream_create_cu_subset(lo, hi, groups, ctypes.byref(h)),
           "stream_create_cu_subset")
    return torch.cuda.ExternalStream(h.value)


class Pipeline:
    """Two streams for the row-chunk pipeline (primary: aggregation, secondary: update)."""

    def __init__(self, primary=None, secondary=None):
        self.primary = primary if primary is not None else torch.cuda.current_stream()
        self.secondary = secondary if secondary is not None else torch.cuda.Stream()
        h = ctypes.c_void_p()
        _check(load_library().mixgcn_pipeline_create(ctypes.c_void_p(self.primary.cuda_stream),
                                                     ctypes.c_void_p(self.secondary.cuda_stream),
                                                     ctypes.byref(h)), "pipeline_create")
        self._h = h

    def timing(self, enable: bool) -> None:
        _check(load_library().mixgcn_pipeline_timing(self._h, int(enable)), "pipeline_timing")

    def timing_read(self, kind: int):
        """(total ms, launches) of one kernel kind since timing was enabled; synchronises."""
        ms, cnt = ctypes.c_double(), ctypes.c_int64()
        _check(load_library().mixgcn_pipeline_timing_read(self._h, kind, ctypes.byref(ms),
                                                          ctypes.byref(cnt)), "pipeline_timing_read")
        return ms.value, cnt.value

    def free(self):
        if self._h:
            load_library().mixgcn_pipeline_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def build_csr(src, dst, n_nodes: int, flags: int = SYMMETRIZE | ADD_SELF_LOOPS, stream=None) -> Graph:
    """src, dst: int32/uint32 torch tensors (cuda, or cpu with INPUT_ON_HOST)."""
    assert src.numel() == dst.numel() and src.element_size() == 4 and dst.element_size() == 4
    src, dst = src.contiguous(), dst.contiguous()
    on_host = not src.is_cuda
    if on_host:
        flags |= INPUT_ON_HOST
    dev = torch.device("cuda", torch.cuda.current_device()) if on_host else src.device
    h = ctypes.c_void_p()
    rc = load_library().mixgcn_build_csr(_ptr(src) if src.numel() else None,
                                         _ptr(dst) if dst.numel() else None, src.numel(), n_nodes,
                                         flags, _stream(stream), ctypes.byref(h))
    _check(rc, "build_csr")
    return Graph(h, dev)


def normalize(g: Graph, mode: int = 0, stream=None, eps: float = 0.0) -> None:
    """mode: NORM_SYM (GCN), NORM_MEAN (GraphSAGE mean), NORM_SUM (GIN; eps on the diagonal)."""
    _check(load_library().mixgcn_normalize_mode(g._h, mode, eps, _stream(stream)), "normalize")


def aggregate(g: Graph, H, Z, col_begin=0, col_end=None, row_begin=0, row_end=None,
              transpose=False, stream=None, relu=False, accumulate=False) -> None:
    col_end = H.shape[1] if col_end is None else col_end
    row_end = g.n if row_end is None else row_end
    if relu or accumulate:
        epi = (EPI_RELU if relu else 0) | (EPI_ACCUMULATE if accumulate else 0)
        _check(load_library().mixgcn_aggregate_ex(g._h, int(transpose), _dtype_of(H), _ptr(H),
                                                  _ld(H), _ptr(Z), _ld(Z), col_begin, col_end,
                                                  row_begin, row_end, epi, _stream(stream)),
               "aggregate_ex")
        return
    _check(load_library().mixgcn_aggregate(g._h, int(transpose), _dtype_of(H), _ptr(H), _ld(H),
                                           _ptr(Z), _ld(Z), col_begin, col_end, row_begin, row_end,
                                           _stream(stream)), "aggregate")


def aggregate_static(g: Graph, H, Z, col_begin=0, col_end=None, row_begin=0, row_end=None,
                     transpose=False, stream=None) -> None:
    """mixgcn_aggregate with the library's fixed scratch array: allocates nothing."""
    col_end = H.shape[1] if col_end is None else col_end
    row_end = g.n if row_end is None else row_end
    _check(load_library().mixgcn_aggregate_static(g._h, int(transpose), _dtype_of(H), _ptr(H),
                                                  _ld(H), _ptr(Z), _ld(Z), col_begin, col_end,
                                                  row_begin, row_end, _stream(stream)),
           "aggregate_static")


def graph_reserve_streams(g: Graph, n_streams: int) -> None:
    """Allocates the aggregation scratch of n_streams streams ahead of their first use."""
    _check(load_library().mixgcn_graph_reserve_streams(g._h, n_streams), "graph_reserve_streams")


def aggregate_scratch_bytes(nnz: int) -> int:
    return load_library().mixgcn_aggregate_scratch_bytes(nnz)


def aggregate_masked(g: Graph, H, Z, mask, col_begin=0, col_end=None, row_begin=0, row_end=None,
                     transpose=False, stream=None) -> None:
    """S-SpMM: Z = (A_hat H) masked by the bitmap `mask` (int32/uint32 tensor [n, words])."""
    col_end = H.shape[1] if col_end is None else col_end
    row_end = g.n if row_end is None else row_end
    assert mask.dtype in (torch.int32, torch.uint32) and mask.stride(1) == 1
    _check(load_library().mixgcn_aggregate_masked(g._h, int(transpose), _dtype_of(H), _ptr(H), _ld(H),
                                                  _ptr(Z), _ld(Z), col_begin, col_end, row_begin,
                                                  row_end, _ptr(mask), mask.stride(0),
                                                  _stream(stream)), "aggregate_masked")


def dropout_bitmap(seed: int, n_rows: int, n_cols: int, keep_probability: float, stream=None):
    """Bitmap [n_rows, ceil(n_cols / 32)] (int32 device tensor) of the elements a dropout with
    this seed keeps; see mixgcn_dropout_bitmap for the generator."""
    mask = torch.empty(n_rows, (n_cols + 31) // 32, dtype=torch.int32, device="cuda")
    _check(load_library().mixgcn_dropout_bitmap(seed & (2 ** 64 - 1), n_rows, n_cols,
                                                float(keep_probability), _ptr(mask), mask.stride(0),
                                                _stream(stream)), "dropout_bitmap")
    return mask


def apply_bitmap(X, mask, stream=None) -> None:
    """X <- X (.) M in place."""
    n, cols = X.shape
    _check(load_library().mixgcn_apply_bitmap(_dtype_of(X), _ptr(X), _ld(X), n, cols, _ptr(mask),
                                              mask.stride(0), _stream(stream)), "apply_bitmap")


def reorder_rcm(g: Graph, stream=None):
    """Reverse Cuthill-McKee positions pos[v] of the nodes of g (int32 tensor [n] on the device)."""
    pos = torch.empty(g.n, dtype=torch.int32, device="cuda")
    _check(load_library().mixgcn_reorder_rcm(g._h, _ptr(pos), _stream(stream)), "reorder_rcm")
    return pos


def bandwidth(g: Graph, pos=None, stream=None) -> int:
    b = ctypes.c_int64()
    _check(load_library().mixgcn_bandwidth(g._h, _ptr(pos), ctypes.byref(b), _stream(stream)),
           "bandwidth")
    return b.value


def pipeline_stages(n: int, b: int) -> int:
    return load_library().mixgcn_pipeline_stages(n, b)


def relabel_edges(src, dst, pos, n: int, stream=None):
    """(pos[src], pos[dst]) as new int32 device tensors."""
    so, do = torch.empty_like(src), torch.empty_like(dst)
    _check(load_library().mixgcn_relabel_edges(_ptr(src), _ptr(dst), src.numel(), _ptr(pos), n,
                                               _ptr(so), _ptr(do), _stream(stream)), "relabel_edges")
    return so, do


def permute_rows(X, pos, Y=None, stream=None):
    """Y[pos[v]] = X[v]."""
    if Y is None:
        Y = torch.empty_strided(X.shape, X.stride(), dtype=X.dtype, device=X.device)
    _check(load_library().mixgcn_permute_rows(_dtype_of(X), _ptr(X), _ld(X), _ptr(Y), _ld(Y),
                                              X.shape[0], X.shape[1], _ptr(pos), _stream(stream)),
           "permute_rows")
    return Y


def relu_bitmap(X, mask=None, stream=None):
    """Bitmap of the positive entries of X: int32 tensor [n, ceil(cols / 32)]."""
    n, cols = X.shape
    if mask is None:
        mask = torch.empty(n, (cols + 31) // 32, dtype=torch.int32, device=X.device)
    _check(load_library().mixgcn_relu_bitmap(_dtype_of(X), _ptr(X), _ld(X), n, cols, _ptr(mask),
                                             mask.stride(0), _stream(stream)), "relu_bitmap")
    return mask


def update(op: int, A, B, C, n_rows: int, k: int, m: int, relu_ref=None, beta: float = 0.0,
           stream=None) -> None:
    dt = _dtype_of(A)
    _check(load_library().mixgcn_update(op, dt, _ptr(A), _ld(A), _ptr(B), _ld(B), _ptr(C), _ld(C),
                                        n_rows, k, m, _ptr(relu_ref),
                                        _ld(relu_ref) if relu_ref is not None else 0, beta,
                                        _stream(stream)), "update")


def _desc(H_like_in, Z, Hout_like, W, relu: bool, n_chunks: int, order: int) -> LayerDesc:
    d = LayerDesc()
    d.f_in, d.f_out = W.shape[0], W.shape[1]
    d.ld_h, d.ld_z, d.ld_out, d.ld_w = _ld(H_like_in), _ld(Z), _ld(Hout_like), _ld(W)
    d.dtype = _dtype_of(Z)
    d.relu = int(relu)
    d.n_chunks = n_chunks
    d.order = order
    return d


def layer_fwd(g: Graph, H, W, Z, Hout, pipe: Pipeline, relu: bool = True, n_chunks: int = 1,
              order: int = AGG_FIRST) -> None:
    """Z: n x f_in (kept for backward) with AGG_FIRST; n x f_out workspace with UPDATE_FIRST."""
    d = _desc(H, Z, Hout, W, relu, n_chunks, order)
    _check(load_library().mixgcn_layer_fwd(g._h, ctypes.byref(d), _ptr(H), _ptr(W), _ptr(Z),
                                           _ptr(Hout), pipe._h), "layer_fwd")


def layer_bwd(g: Graph, Z, Hout, W, G, dW, dH, pipe: Pipeline, relu: bool = True,
              n_chunks: int = 1, order: int = AGG_FIRST, H=None) -> None:
    """H (the layer input) is needed only with UPDATE_FIRST."""
    assert _ld(dW) == _ld(W), "dW must have the leading dimension of W"
    assert dH is None or H is None or _ld(dH) == _ld(H), "dH must have the leading dimension of H"
    h_like = dH if dH is not None else (H if H is not None else Z)
    d = _desc(h_like, Z, G, W, relu, n_chunks, order)
    _check(load_library().mixgcn_layer_bwd(g._h, ctypes.byref(d), _ptr(H), _ptr(Z), _ptr(Hout),
                                           _ptr(W), _ptr(G), _ptr(dW), _ptr(dH), pipe._h),
           "layer_bwd")


def _ptr_array(tensors):
    return (ctypes.c_void_p * len(tensors))(*[None if t is None else t.data_ptr() for t in tensors])


def forward_pipelined(g: Graph, H0, Ws, Zs, Houts, pipe: Pipeline, bandwidth: int, n_chunks: int,
                      orders=None, last_relu: bool = False) -> None:
    """All layers as one cross-layer pipeline (ReLU on every layer but the last unless
    last_relu)."""
    L = len(Ws)
    orders = orders or [AGG_FIRST] * L
    ins = [H0] + list(Houts[:-1])
    descs = (LayerDesc * L)(*[_desc(ins[l], Zs[l], Houts[l], Ws[l], l < L - 1 or last_relu,
                                    n_chunks, orders[l]) for l in range(L)])
    _check(load_library().mixgcn_forward_pipelined(g._h, L, descs, _ptr(H0), _ptr_array(Ws),
                                                   _ptr_array(Zs), _ptr_array(Houts), bandwidth,
                                                   pipe._h), "forward_pipelined")


def backward_pipelined(g: Graph, H0, Zs, Houts, Ws, Gs, dWs, dH0, pipe: Pipeline, bandwidth: int,
                       n_chunks: int, orders=None, last_relu: bool = False) -> None:
    """Gs[l]: gradient with respect to Houts[l]; Gs[-1] is the loss gradient on entry, the others
    are written (Gs[l-1] = input gradient of layer l)."""
    L = len(Ws)
    orders = orders or [AGG_FIRST] * L
    ins = [H0] + list(Houts[:-1])
    for l in range(L):
        assert _ld(dWs[l]) == _ld(Ws[l]), "dW must have the leading dimension of W"
        assert _ld(Gs[l]) == _ld(Houts[l]), "G must have the leading dimension of Hout"
    descs = (LayerDesc * L)(*[_desc(ins[l], Zs[l], Houts[l], Ws[l], l < L - 1 or last_relu,
                                    n_chunks, orders[l]) for l in range(L)])
    _check(load_library().mixgcn_backward_pipelined(g._h, L, descs, _ptr(H0), _ptr_array(Zs),
                                                    _ptr_array(Houts), _ptr_array(Ws),
                                                    _ptr_array(Gs), _ptr_array(dWs), _ptr(dH0),
                                                    bandwidth, pipe._h), "backward_pipelined")


def pipeline_window(n_nodes: int, n_chunks: int, bandwidth: int, chunk: int):
    """(row_begin, row_end, first, last): the rows of batch `chunk` and the batches of its input
    that an aggregation of that batch reads.  Host arithmetic, no GPU needed."""
    r0, r1 = ctypes.c_int64(), ctypes.c_int64()
    f, l = ctypes.c_int32(), ctypes.c_int32()
    _check(load_library().mixgcn_pipeline_window(n_nodes, n_chunks, bandwidth, chunk,
                                                 ctypes.byref(r0), ctypes.byref(r1),
                                                 ctypes.byref(f), ctypes.byref(l)),
           "pipeline_window")
    return r0.value, r1.value, f.value, l.value


def set_aggregate_whole_rows(on: bool) -> None:
    """Measurement aid: aggregations without column slices (set before normalize)."""
    _check(load_library().mixgcn_set_aggregate_whole_rows(int(bool(on))), "set_aggregate_whole_rows")


def set_update_arith(mode: int) -> None:
    """ARITH_FP32 (default) or ARITH_BF16X3 for the update products of fp32 features."""
    _check(load_library().mixgcn_set_update_arith(mode), "set_update_arith")


def softmax_xent(logits, labels, dlogits, loss, stream=None) -> None:
    n, c = logits.shape
    _check(load_library().mixgcn_softmax_xent(_dtype_of(logits), _ptr(logits), _ld(logits),
                                              _ptr(labels), n, c,
                                              _ptr(dlogits), _ld(dlogits), _ptr(loss),
                                              _stream(stream)), "softmax_xent")
