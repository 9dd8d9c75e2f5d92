"""Python loader for the CPU oracle (test infrastructure, never the product path).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It compiles oracle/sparse_layer_oracle.cpp with g++ on first use
and calls it through ctypes; it imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparse_layer_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

ABS, SIGNED = 0, 1
FUSE_RELU, FUSE_POOL = 1, 2


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i32p, f32p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)
        L.oracle_k_from_rho.restype = ctypes.c_int64
        L.oracle_k_from_rho.argtypes = [ctypes.c_double, ctypes.c_int64]
        L.oracle_sparse_conv_fwd.restype = ctypes.c_int64
        L.oracle_sparse_conv_fwd.argtypes = [ctypes.c_int, i32p, ctypes.c_int, i32p, f32p, ctypes.c_int64,
                                             ctypes.c_int, i32p, f32p, f32p, ctypes.c_int, ctypes.c_int64,
                                             ctypes.c_int, ctypes.c_uint, ctypes.c_int, ctypes.c_int]
        L.oracle_attention_topk.restype = ctypes.c_int64
        L.oracle_attention_topk.argtypes = [ctypes.c_int, i32p, ctypes.c_int, i32p, f32p, ctypes.c_int64,
                                            ctypes.c_int, ctypes.c_int64, ctypes.c_int]
        L.oracle_sparse_relu.restype = ctypes.c_int64
        L.oracle_sparse_relu.argtypes = [ctypes.c_int, i32p, i32p, f32p, ctypes.c_int64, ctypes.c_int]
        L.oracle_sparse_maxpool.restype = ctypes.c_int64
        L.oracle_sparse_maxpool.argtypes = [ctypes.c_int, i32p, i32p, f32p, ctypes.c_int64, ctypes.c_int]
        L.oracle_sparse_conv_bwd.restype = ctypes.c_int64
        L.oracle_sparse_conv_bwd.argtypes = [ctypes.c_int, i32p, ctypes.c_int, i32p, f32p, ctypes.c_int64,
                                             ctypes.c_int, i32p, f32p, ctypes.c_int, i32p, f32p, ctypes.c_int64,
                                             f32p, f32p]
        L.oracle_result_rows.restype = ctypes.c_int64
        L.oracle_result_macs.restype = ctypes.c_int64
        L.oracle_result_threads.restype = ctypes.c_int
        L.oracle_fetch.restype = None
        L.oracle_fetch.argtypes = [i32p, f32p]
        _lib = L
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _fetch(L, rows: int, ndim: int, channels: int) -> Tuple[np.ndarray, np.ndarray]:
    coords = np.zeros((rows, 1 + ndim), dtype=np.int32)
    feats = np.zeros((rows, channels), dtype=np.float32)
    if rows:
        L.oracle_fetch(coords.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                       feats.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    return coords, feats


def k_from_rho(rho_up: float, n_sites: int) -> int:
    return int(_load().oracle_k_from_rho(float(rho_up), int(n_sites)))


def sparse_conv_fwd(extent: Sequence[int], batch: int, coords, feats, ksize: Sequence[int], w,
                    bias=None, *, k: Optional[int] = None, rho_up: Optional[float] = None,
                    topk_mode: int = ABS, relu: bool = False, pool: bool = False,
                    resp_only: bool = False, threads: int = 1, return_info: bool = False):
    """Algorithm 1 (+ optional ReLU, 2^d max-pool).  Returns (coords, feats)."""
    L = _load()
    ndim = len(extent)
    n_sites = int(np.prod([int(e) for e in extent]))
    if k is None:
        k = n_sites if rho_up is None else k_from_rho(rho_up, n_sites)
    ext, extp = _i32(extent)
    ks, ksp = _i32(ksize)
    c, cp = _i32(coords)
    f, fp = _f32(feats)
    wa, wp = _f32(w)
    c_in, c_out = int(wa.shape[1]), int(wa.shape[2])
    assert wa.shape[0] == int(np.prod(ks)) and f.shape == (c.shape[0], c_in) and c.shape[1] == 1 + ndim
    if bias is not None:
        ba, bp = _f32(bias)
        assert ba.shape == (c_out,)
    else:
        bp = ctypes.POINTER(ctypes.c_float)()
    fuse = (FUSE_RELU if relu else 0) | (FUSE_POOL if pool else 0)
    rows = L.oracle_sparse_conv_fwd(ndim, extp, int(batch), cp, fp, c.shape[0], c_in, ksp, wp, bp, c_out,
                                    int(k), int(topk_mode), fuse, int(bool(resp_only)), int(threads))
    if rows < 0:
        raise ValueError("oracle_sparse_conv_fwd: bad arguments")
    out = _fetch(L, int(rows), ndim, c_out)
    if return_info:
        return out + ({"macs": int(L.oracle_result_macs()), "threads": int(L.oracle_result_threads())},)
    return out


def sparse_conv_bwd(extent: Sequence[int], batch: int, coords, feats, ksize: Sequence[int], w, g_coords, g_feats,
                    return_info: bool = False):
    """Algorithm 2 with the masks of Eq. 3.  Returns (bp_data [rows, C_in], bp_filter [T, C_in, C_out])."""
    L = _load()
    ndim = len(extent)
    ext, extp = _i32(extent)
    ks, ksp = _i32(ksize)
    c, cp = _i32(coords)
    f, fp = _f32(feats)
    wa, wp = _f32(w)
    gc, gcp = _i32(g_coords)
    gf, gfp = _f32(g_feats)
    c_in, c_out = int(wa.shape[1]), int(wa.shape[2])
    assert wa.shape[0] == int(np.prod(ks)) and f.shape == (c.shape[0], c_in) and c.shape[1] == 1 + ndim
    assert gf.shape == (gc.shape[0], c_out) and gc.shape[1] == 1 + ndim
    bp_data = np.zeros((c.shape[0], c_in), dtype=np.float32)
    bp_filter = np.zeros(wa.shape, dtype=np.float32)
    visits = L.oracle_sparse_conv_bwd(ndim, extp, int(batch), cp, fp, c.shape[0], c_in, ksp, wp, c_out, gcp, gfp,
                                      gc.shape[0], bp_data.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                      bp_filter.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if visits < 0:
        raise ValueError("oracle_sparse_conv_bwd: bad arguments")
    if return_info:
        return bp_data, bp_filter, {"visits": int(visits)}
    return bp_data, bp_filter


def attention_topk(extent: Sequence[int], batch: int, coords, resp, k: int, topk_mode: int = ABS):
    L = _load()
    ext, extp = _i32(extent)
    c, cp = _i32(coords)
    f, fp = _f32(resp)
    rows = L.oracle_attention_topk(len(extent), extp, int(batch), cp, fp, c.shape[0], f.shape[1], int(k),
                                   int(topk_mode))
    if rows < 0:
        raise ValueError("oracle_attention_topk: bad arguments")
    return _fetch(L, int(rows), len(extent), f.shape[1])


def sparse_relu(extent: Sequence[int], coords, feats):
    L = _load()
    ext, extp = _i32(extent)
    c, cp = _i32(coords)
    f, fp = _f32(feats)
    rows = L.oracle_sparse_relu(len(extent), extp, cp, fp, c.shape[0], f.shape[1])
    if rows < 0:
        raise ValueError("oracle_sparse_relu: bad arguments")
    return _fetch(L, int(rows), len(extent), f.shape[1])


def sparse_maxpool(extent: Sequence[int], coords, feats):
    L = _load()
    ext, extp = _i32(extent)
    c, cp = _i32(coords)
    f, fp = _f32(feats)
    rows = L.oracle_sparse_maxpool(len(extent), extp, cp, fp, c.shape[0], f.shape[1])
    if rows < 0:
        raise ValueError("oracle_sparse_maxpool: bad arguments")
    return _fetch(L, int(rows), len(extent), f.shape[1])


def sparse_to_dense(extent: Sequence[int], batch: int, coords, feats) -> np.ndarray:
    """sparseToDense (appendix table of architectures): dense [batch, channels, *extent], the rows' values at
    their sites and zero elsewhere.  Written out as the definition, one row at a time."""
    coords = np.asarray(coords)
    feats = np.asarray(feats, dtype=np.float32)
    dense = np.zeros((int(batch), feats.shape[1], *[int(e) for e in extent]), dtype=np.float32)
    for r in range(coords.shape[0]):
        dense[(int(coords[r, 0]), slice(None)) + tuple(int(v) for v in coords[r, 1:])] = feats[r]
    return dense


def density_regulariser(out_feats, n_sites_total: int, rho_up: float, o: float, b1: float, b2: float, lam: float, w):
    """Adaptive density regularisation (Sec. 3.5, Eq. 4), in double.  Returns (rho, b, R, grad) with
    R = lam * sum over un-pruned weights of (w + b)^2 and grad = dR/dw on those weights, 0 on pruned ones."""
    out_feats = np.asarray(out_feats)
    w64 = np.asarray(w, dtype=np.float64)
    entries = int(np.count_nonzero(out_feats))
    rho = entries / (float(n_sites_total) * out_feats.shape[1])
    if rho > rho_up:
        b = o + b1 * (rho - rho_up)      # exceeds the available resources
    else:
        b = -b2 * (rho_up - rho)         # not using all resources
    alive = w64 != 0.0
    reg = 0.0
    grad = np.zeros_like(w64)
    for i in np.flatnonzero(alive.ravel()):
        t = w64.ravel()[i] + b
        reg += t * t
        grad.ravel()[i] = 2.0 * lam * t
    return rho, b, lam * reg, grad


def prune_weights(w, warned, eps: float):
    """One-warning-shot pruning (Sec. 3.6) of one epoch's end.  Returns (new w, new warned, removed, left)."""
    w = np.array(w, dtype=np.float32, copy=True)
    warned = np.array(warned, dtype=np.uint8, copy=True)
    removed = 0
    for i in range(w.size):
        wi = w.flat[i]
        small = wi != 0.0 and abs(wi) < np.float32(eps)
        if small and warned.flat[i]:
            w.flat[i] = 0.0        # second time in a row: remove
            warned.flat[i] = 0
            removed += 1
        else:
            warned.flat[i] = 1 if small else 0
    return w, warned, removed, int(np.count_nonzero(w))
