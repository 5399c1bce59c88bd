"""Seeded synthetic inputs (edge lists and dense tensors) for the GCN hot path.

Thin ctypes binding over ``gen.c``.  This package produces *inputs only*: it contains none of
the method's arithmetic and is the only code shared by the CPU oracle's tests and the HIP
library's tests and benchmark.  Every value is a pure function of (seed, stream, index).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libgraphgen.so")
_lib = None

MASTER_SEED = 250101951


def build(force: bool = False) -> str:
    """Compile gen.c into libgraphgen.so (gcc, OpenMP)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, src, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        lib = ctypes.CDLL(_SO)
        u64, i64, i32, dbl = ctypes.c_uint64, ctypes.c_int64, ctypes.c_int32, ctypes.c_double
        p = ctypes.c_void_p
        lib.gg_rmat_edges.argtypes = [u64, ctypes.c_int, u64, dbl, dbl, dbl, ctypes.c_int, u64, p, p]
        lib.gg_rmat_edges.restype = None
        lib.gg_er_edges.argtypes = [u64, ctypes.c_uint32, dbl, p, p, u64]
        lib.gg_er_edges.restype = u64
        lib.gg_zipf_edges.argtypes = [u64, ctypes.c_uint32, u64, dbl, dbl, p, p]
        lib.gg_zipf_edges.restype = None
        lib.gg_fill_uniform.argtypes = [u64, u64, i64, i64, i64, dbl, dbl, p]
        lib.gg_fill_uniform.restype = None
        lib.gg_fill_normal.argtypes = [u64, u64, i64, i64, i64, p]
        lib.gg_fill_normal.restype = None
        lib.gg_fill_glorot.argtypes = [u64, u64, i64, i64, i64, p]
        lib.gg_fill_glorot.restype = None
        lib.gg_fill_labels.argtypes = [u64, u64, i64, i32, p]
        lib.gg_fill_labels.restype = None
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def rmat_edges(seed: int, scale: int, n_edges: int, a=0.57, b=0.19, c=0.19,
               scramble: bool = True, n_limit: int = 0):
    """Directed R-MAT edge list (src, dst) as uint32 arrays of length n_edges."""
    src = np.empty(n_edges, dtype=np.uint32)
    dst = np.empty(n_edges, dtype=np.uint32)
    _load().gg_rmat_edges(seed, scale, n_edges, a, b, c, int(scramble), n_limit, _ptr(src), _ptr(dst))
    return src, dst


def er_edges(seed: int, n: int, avg_degree: float):
    """Undirected G(n, p) with p = avg_degree / (n - 1); each pair {i<j} listed once."""
    p = avg_degree / (n - 1)
    lib = _load()
    cnt = lib.gg_er_edges(seed, n, p, None, None, 0)
    src = np.empty(cnt, dtype=np.uint32)
    dst = np.empty(cnt, dtype=np.uint32)
    lib.gg_er_edges(seed, n, p, _ptr(src), _ptr(dst), cnt)
    return src, dst


def zipf_edges(seed: int, n: int, n_edges: int, alpha: float = 2.1, max_degree: float = 1 << 20):
    """Directed edges: out-degrees follow a power law with tail exponent alpha (largest expected
    out-degree about max_degree), destinations uniform."""
    src = np.empty(n_edges, dtype=np.uint32)
    dst = np.empty(n_edges, dtype=np.uint32)
    _load().gg_zipf_edges(seed, n, n_edges, alpha, float(max_degree), _ptr(src), _ptr(dst))
    return src, dst


def _alloc(rows, cols, ld, out):
    ld = cols if ld is None else ld
    assert ld >= cols
    if out is None:
        out = np.empty((rows, ld), dtype=np.float32)
    assert out.dtype == np.float32 and out.flags.c_contiguous and out.shape == (rows, ld)
    return ld, out


def uniform(seed: int, stream: int, rows: int, cols: int, lo=-1.0, hi=1.0, ld=None, out=None):
    ld, out = _alloc(rows, cols, ld, out)
    _load().gg_fill_uniform(seed, stream, rows, cols, ld, lo, hi, _ptr(out))
    return out


def normal(seed: int, stream: int, rows: int, cols: int, ld=None, out=None):
    ld, out = _alloc(rows, cols, ld, out)
    _load().gg_fill_normal(seed, stream, rows, cols, ld, _ptr(out))
    return out


def glorot(seed: int, stream: int, fan_in: int, fan_out: int, ld=None, out=None):
    ld, out = _alloc(fan_in, fan_out, ld, out)
    _load().gg_fill_glorot(seed, stream, fan_in, fan_out, ld, _ptr(out))
    return out


def labels(seed: int, stream: int, n: int, n_classes: int):
    out = np.empty(n, dtype=np.int32)
    _load().gg_fill_labels(seed, stream, n, n_classes, _ptr(out))
    return out


# ---------------------------------------------------------------------------------------------
# Named workloads (shapes follow the benchmark configs; all sizes can be scaled down).
# ---------------------------------------------------------------------------------------------

def ring_lattice_edges(n: int, k: int):
    """k-regular circulant graph (k even): i -- i+1..i+k/2 (mod n).  Each pair listed once."""
    assert k % 2 == 0 and k < n
    i = np.repeat(np.arange(n, dtype=np.uint32), k // 2)
    off = np.tile(np.arange(1, k // 2 + 1, dtype=np.uint32), n)
    return i, ((i.astype(np.uint64) + off) % n).astype(np.uint32)


def config_graph(name: str, seed: int = MASTER_SEED, scale_override: int | None = None,
                 scramble: bool = True):
    """Edge list + node count for a named benchmark configuration.

    c1: Erdos-Renyi N=4096, average degree 10.
    c2: R-MAT scale 20, 16*N directed edges.
    c3: R-MAT scale 24, 8*N directed edges (average degree 16 after symmetrisation).
    c4: N = 111,000,000, 1.6e9 directed edges with power-law (alpha = 2.1) out-degrees;
        scale_override = s gives the same recipe at N = 2^s with 14.4 N edges.
    c5: R-MAT scale 22 with ids >= 2,450,000 rejected, 25*N directed edges.
    scramble = False keeps the R-MAT generator's own numbering (hubs at low ids) for c2, c3, c5.
    """
    if name == "c1":
        n = 4096
        s, d = er_edges(seed, n, 10.0)
        return s, d, n
    if name == "c2":
        scale = scale_override or 20
        n = 1 << scale
        s, d = rmat_edges(seed, scale, 16 * n, scramble=scramble)
        return s, d, n
    if name == "c3":
        scale = scale_override or 24
        n = 1 << scale
        s, d = rmat_edges(seed, scale, 8 * n, scramble=scramble)
        return s, d, n
    if name == "c4":
        if scale_override:
            n = 1 << scale_override
            e = int(14.4 * n)
        else:
            n, e = 111_000_000, 1_600_000_000
        s, d = zipf_edges(seed, n, e, 2.1, min(1 << 20, n // 64))
        return s, d, n
    if name == "c5":
        if scale_override:
            scale = scale_override
            n = int((1 << scale) * (2_450_000 / (1 << 22)))
        else:
            scale, n = 22, 2_450_000
        s, d = rmat_edges(seed, scale, 25 * n, n_limit=n, scramble=scramble)
        return s, d, n
    raise ValueError(name)
