"""ctypes binding of libscnn.so: argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libscnn.so")
_lib = None

ABS, SIGNED = 0, 1
FUSE_RELU, FUSE_MAXPOOL2 = 1, 2
FLAG_CAND_OVERFLOW, FLAG_OUT_OVERFLOW, FLAG_BAD_COORD, FLAG_UNSORTED = 1, 2, 4, 8
NNZ_LEN = 4

EXPORTED_SYMBOLS = [
    "scnn_last_error", "scnn_version", "scnn_k_from_rho", "sparse_conv_fwd_max_rows", "sparse_conv_fwd_workspace",
    "sparse_conv_fwd", "attention_topk_workspace", "attention_topk", "sparse_relu_workspace", "sparse_relu",
    "sparse_maxpool_workspace", "sparse_maxpool", "scnn_validate_rows", "scnn_profile_enable",
    "scnn_profile_stage_count", "scnn_set_conv_path", "scnn_calibration_copy", "scnn_profile_stage_name", "scnn_profile_collect",
    "sparse_conv_bwd_workspace", "sparse_conv_bwd", "sparse_to_dense",
    "density_regulariser_workspace", "density_regulariser", "prune_weights", "sparse_conv_fwd_chained",
    "sparse_relu_static_max_rows", "sparse_relu_static", "scnn_last_conv_kernel",
]


class ScnnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libscnn error {code}: {msg}")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libscnn.so.  If it was never built, build it once (tests and the benchmark
    normally find it already built in-tree); a missing compiler is an error, not a fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build
        build(force=False)
    L = ctypes.CDLL(_LIB_PATH)
    i32p = ctypes.POINTER(ctypes.c_int32)
    vp, i64, sz, ci, cu, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int, ctypes.c_uint, ctypes.c_double
    L.scnn_last_error.restype = ctypes.c_char_p
    L.scnn_version.restype = ci
    L.scnn_k_from_rho.restype = i64
    L.scnn_k_from_rho.argtypes = [dbl, i64]
    L.sparse_conv_fwd_max_rows.restype = i64
    L.sparse_conv_fwd_max_rows.argtypes = [ci, i32p, ci, i64, i32p]
    L.sparse_conv_fwd_workspace.restype = sz
    L.sparse_conv_fwd_workspace.argtypes = [ci, i32p, ci, i64, ci, ci, i32p, cu, i64]
    L.sparse_conv_fwd.restype = ci
    L.sparse_conv_fwd.argtypes = [ci, i32p, ci, vp, vp, i64, ci, i32p, vp, vp, ci, dbl, ci, cu, vp, vp, i64, i64, vp,
                                  vp, sz, vp]
    L.sparse_conv_bwd_workspace.restype = sz
    L.sparse_conv_bwd_workspace.argtypes = [ci, i32p, ci, i64, ci, ci, i32p, i64]
    L.sparse_conv_bwd.restype = ci
    L.sparse_conv_bwd.argtypes = [ci, i32p, ci, vp, vp, i64, ci, i32p, vp, ci, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    L.attention_topk_workspace.restype = sz
    L.attention_topk_workspace.argtypes = [ci, i32p, ci, i64, ci]
    L.attention_topk.restype = ci
    L.attention_topk.argtypes = [ci, i32p, ci, vp, vp, i64, ci, i64, ci, vp, vp, i64, vp, vp, sz, vp]
    L.sparse_relu_workspace.restype = sz
    L.sparse_relu_workspace.argtypes = [i64, ci]
    L.sparse_relu.restype = ci
    L.sparse_relu.argtypes = [ci, vp, vp, i64, ci, vp, vp, i64, vp, vp, sz, vp]
    L.sparse_relu_static_max_rows.restype = i64
    L.sparse_relu_static_max_rows.argtypes = []
    L.sparse_relu_static.restype = ci
    L.sparse_relu_static.argtypes = [ci, vp, vp, i64, ci, vp, vp, i64, vp, vp]
    L.sparse_maxpool_workspace.restype = sz
    L.sparse_maxpool_workspace.argtypes = [ci, i32p, ci, i64, ci]
    L.sparse_maxpool.restype = ci
    L.sparse_maxpool.argtypes = [ci, i32p, ci, ci, vp, vp, i64, ci, vp, vp, i64, vp, vp, sz, vp]
    L.sparse_to_dense.restype = ci
    L.sparse_to_dense.argtypes = [ci, i32p, ci, vp, vp, i64, vp, ci, vp, vp]
    L.sparse_conv_fwd_chained.restype = ci
    L.sparse_conv_fwd_chained.argtypes = [ci, i32p, ci, vp, vp, i64, vp, ci, i32p, vp, vp, ci, dbl, ci, cu, vp, vp, i64,
                                          i64, vp, vp, sz, vp]
    L.density_regulariser_workspace.restype = sz
    L.density_regulariser_workspace.argtypes = []
    L.density_regulariser.restype = ci
    L.density_regulariser.argtypes = [vp, i64, vp, ci, i64, dbl, dbl, dbl, dbl, dbl, vp, i64, vp, vp, vp, sz, vp]
    L.prune_weights.restype = ci
    L.prune_weights.argtypes = [vp, vp, i64, ctypes.c_float, vp, vp]
    L.scnn_validate_rows.restype = ci
    L.scnn_validate_rows.argtypes = [ci, i32p, ci, vp, i64, vp, sz, vp]
    L.scnn_calibration_copy.restype = ci
    L.scnn_calibration_copy.argtypes = [vp, vp, sz, vp]
    L.scnn_last_conv_kernel.restype = ctypes.c_char_p
    L.scnn_last_conv_kernel.argtypes = []
    L.scnn_set_conv_path.restype = ci
    L.scnn_set_conv_path.argtypes = [ci]
    L.scnn_profile_enable.restype = ci
    L.scnn_profile_enable.argtypes = [ci]
    L.scnn_profile_stage_count.restype = ci
    L.scnn_profile_stage_name.restype = ctypes.c_char_p
    L.scnn_profile_stage_name.argtypes = [ci]
    L.scnn_profile_collect.restype = ci
    L.scnn_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    _lib = L
    return L


def _check(L, rc: int):
    if rc != 0:
        raise ScnnError(rc, L.scnn_last_error().decode())


def _i32arr(v: Sequence[int]):
    return (ctypes.c_int32 * len(v))(*[int(x) for x in v])


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}")
    return t.contiguous()


def k_from_rho(rho_up: float, n_sites: int) -> int:
    return int(load_library().scnn_k_from_rho(float(rho_up), int(n_sites)))


def sparse_conv_fwd_max_rows(extent, batch, nnz_in, ksize) -> int:
    L = load_library()
    r = int(L.sparse_conv_fwd_max_rows(len(extent), _i32arr(extent), int(batch), int(nnz_in), _i32arr(ksize)))
    if r < 0:
        _check(L, r)
    return r


def sparse_conv_fwd_workspace(extent, batch, nnz_in, c_in, c_out, ksize, fuse=0, cand_capacity=0) -> int:
    L = load_library()
    r = int(L.sparse_conv_fwd_workspace(len(extent), _i32arr(extent), int(batch), int(nnz_in), int(c_in), int(c_out),
                                        _i32arr(ksize), int(fuse), int(cand_capacity)))
    if r == 0:
        raise ScnnError(-1, L.scnn_last_error().decode())
    return r


def _finish(out_coords, out_feats, nnz, sync):
    if not sync:
        return out_coords, out_feats, nnz
    n = nnz.cpu()
    rows, flags = int(n[0]), int(n[2])
    if flags & (FLAG_CAND_OVERFLOW | FLAG_OUT_OVERFLOW):
        raise ScnnError(-2, f"capacity exceeded (rows={rows}, candidates={int(n[1])}, flags={flags})")
    return out_coords[:rows], out_feats[:rows], n


def sparse_conv_fwd(extent, batch, coords, feats, ksize, w, bias=None, *, rho_up=1.0, topk_mode=ABS, relu=False,
                    pool=False, out_capacity: Optional[int] = None, cand_capacity: int = 0, workspace=None,
                    out=None, stream=None, sync=True):
    """Forward sparse convolution + attention (+ReLU, +2^d max-pool).  Returns (out_coords, out_feats, nnz)
    where nnz is the int64[4] counter vector (device tensor when sync=False, host tensor otherwise)."""
    L = load_library()
    ndim = len(extent)
    coords = _dev(coords, torch.int32, "coords")
    feats = _dev(feats, torch.float32, "feats")
    w = _dev(w, torch.float32, "w")
    if bias is not None:
        bias = _dev(bias, torch.float32, "bias")
    nnz_in, c_in = feats.shape
    taps, c_in_w, c_out = w.shape
    if c_in_w != c_in or coords.shape != (nnz_in, 1 + ndim):
        raise ValueError("shape mismatch between coords, feats and w")
    t = 1
    for s in ksize:
        t *= int(s)
    if t != taps:
        raise ValueError("w.shape[0] != prod(ksize)")
    if bias is not None and bias.shape != (c_out,):
        raise ValueError("bias must be [c_out]")
    fuse = (FUSE_RELU if relu else 0) | (FUSE_MAXPOOL2 if pool else 0)
    ext, ks = _i32arr(extent), _i32arr(ksize)
    dev = feats.device
    if cand_capacity <= 0:
        cand_capacity = int(L.sparse_conv_fwd_max_rows(ndim, ext, int(batch), nnz_in, ks))
    if out_capacity is None:
        out_capacity = cand_capacity
    need = int(L.sparse_conv_fwd_workspace(ndim, ext, int(batch), nnz_in, c_in, c_out, ks, fuse, cand_capacity))
    if need == 0:
        raise ScnnError(-1, L.scnn_last_error().decode())
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    if out is None:
        out_coords = torch.empty((out_capacity, 1 + ndim), dtype=torch.int32, device=dev)
        out_feats = torch.empty((out_capacity, c_out), dtype=torch.float32, device=dev)
        nnz = torch.zeros(NNZ_LEN, dtype=torch.int64, device=dev)
    else:
        out_coords, out_feats, nnz = out
    rc = L.sparse_conv_fwd(ndim, ext, int(batch), _ptr(coords), _ptr(feats), nnz_in, c_in, ks, _ptr(w), _ptr(bias),
                           c_out, float(rho_up), int(topk_mode), fuse, _ptr(out_coords), _ptr(out_feats),
                           int(out_capacity), int(cand_capacity), _ptr(nnz), _ptr(workspace), workspace.numel(),
                           _stream(stream))
    _check(L, rc)
    return _finish(out_coords, out_feats, nnz, sync)


def sparse_conv_bwd(extent, batch, coords, feats, ksize, w, g_coords, g_feats, *, workspace=None, out=None,
                    stream=None, sync=True):
    """Back-propagation through the convolution (Algorithm 2 with the masks of Eq. 3).
    Returns (bp_data [rows, C_in], bp_filter [T, C_in, C_out], info int64[4])."""
    L = load_library()
    ndim = len(extent)
    coords = _dev(coords, torch.int32, "coords")
    feats = _dev(feats, torch.float32, "feats")
    w = _dev(w, torch.float32, "w")
    g_coords = _dev(g_coords, torch.int32, "g_coords")
    g_feats = _dev(g_feats, torch.float32, "g_feats")
    nnz_in, c_in = feats.shape
    taps, c_in_w, c_out = w.shape
    g_rows = g_feats.shape[0]
    if c_in_w != c_in or coords.shape != (nnz_in, 1 + ndim):
        raise ValueError("shape mismatch between coords, feats and w")
    if g_feats.shape[1] != c_out or g_coords.shape != (g_rows, 1 + ndim):
        raise ValueError("shape mismatch between g_coords, g_feats and w")
    t = 1
    for s in ksize:
        t *= int(s)
    if t != taps:
        raise ValueError("w.shape[0] != prod(ksize)")
    ext, ks = _i32arr(extent), _i32arr(ksize)
    dev = feats.device
    need = int(L.sparse_conv_bwd_workspace(ndim, ext, int(batch), nnz_in, c_in, c_out, ks, g_rows))
    if need == 0:
        raise ScnnError(-1, L.scnn_last_error().decode())
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    if out is None:
        bp_data = torch.empty((nnz_in, c_in), dtype=torch.float32, device=dev)
        bp_filter = torch.empty((taps, c_in, c_out), dtype=torch.float32, device=dev)
        info = torch.zeros(NNZ_LEN, dtype=torch.int64, device=dev)
    else:
        bp_data, bp_filter, info = out
    rc = L.sparse_conv_bwd(ndim, ext, int(batch), _ptr(coords), _ptr(feats), nnz_in, c_in, ks, _ptr(w), c_out,
                           _ptr(g_coords), _ptr(g_feats), g_rows, _ptr(bp_data), _ptr(bp_filter), _ptr(info),
                           _ptr(workspace), workspace.numel(), _stream(stream))
    _check(L, rc)
    if sync:
        info = info.cpu()
    return bp_data, bp_filter, info


def sparse_conv_bwd_workspace(extent, batch, nnz_in, c_in, c_out, ksize, g_rows) -> int:
    L = load_library()
    r = int(L.sparse_conv_bwd_workspace(len(extent), _i32arr(extent), int(batch), int(nnz_in), int(c_in), int(c_out),
                                        _i32arr(ksize), int(g_rows)))
    if r == 0:
        raise ScnnError(-1, L.scnn_last_error().decode())
    return r


class ChainedLayer:
    """One layer of a chain that runs without host reads: buffers sized once from capacities, the input row count
    taken on the device.  `in_capacity` bounds the rows of the input arrays.  Run a chain once eagerly before
    capturing it in a HIP graph: the first launch of a matrix-core kernel sets that kernel's shared-memory attribute,
    which is not a stream operation."""

    def __init__(self, extent, batch, in_capacity, c_in, ksize, w, *, bias=None, rho_up=1.0, topk_mode=ABS,
                 relu=False, pool=False):
        L = load_library()
        self.extent, self.batch, self.ksize = tuple(int(e) for e in extent), int(batch), tuple(int(k) for k in ksize)
        self.ndim = len(self.extent)
        self.w = _dev(w, torch.float32, "w")
        self.bias = None if bias is None else _dev(bias, torch.float32, "bias")
        self.c_in, self.c_out = int(c_in), int(self.w.shape[2])
        self.in_capacity = max(1, int(in_capacity))
        self.rho_up, self.topk_mode = float(rho_up), int(topk_mode)
        self.fuse = (FUSE_RELU if relu else 0) | (FUSE_MAXPOOL2 if pool else 0)
        ext, ks = _i32arr(self.extent), _i32arr(self.ksize)
        self.cand_capacity = int(L.sparse_conv_fwd_max_rows(self.ndim, ext, self.batch, self.in_capacity, ks))
        need = int(L.sparse_conv_fwd_workspace(self.ndim, ext, self.batch, self.in_capacity, self.c_in, self.c_out, ks,
                                               self.fuse, self.cand_capacity))
        if need == 0:
            raise ScnnError(-1, L.scnn_last_error().decode())
        dev = self.w.device
        self.out_extent = tuple((e + 1) // 2 for e in self.extent) if pool else self.extent
        n_out = self.batch
        for e in self.out_extent:
            n_out *= e
        self.out_capacity = min(self.cand_capacity, n_out)
        self.workspace = torch.empty(need, dtype=torch.uint8, device=dev)
        self.out_coords = torch.empty((self.out_capacity, 1 + self.ndim), dtype=torch.int32, device=dev)
        self.out_feats = torch.empty((self.out_capacity, self.c_out), dtype=torch.float32, device=dev)
        self.nnz = torch.zeros(NNZ_LEN, dtype=torch.int64, device=dev)

    def __call__(self, coords, feats, nnz_in_dev, stream=None):
        """Enqueue the layer; returns (out_coords, out_feats, nnz) -- full-capacity buffers, the count stays on the
        device in nnz[0]."""
        L = load_library()
        if coords.shape[0] > self.in_capacity or feats.shape != (coords.shape[0], self.c_in):
            raise ValueError("input arrays do not fit this layer")
        rc = L.sparse_conv_fwd_chained(self.ndim, _i32arr(self.extent), self.batch, _ptr(coords), _ptr(feats),
                                       coords.shape[0], _ptr(nnz_in_dev), self.c_in, _i32arr(self.ksize), _ptr(self.w),
                                       _ptr(self.bias), self.c_out, self.rho_up, self.topk_mode, self.fuse,
                                       _ptr(self.out_coords), _ptr(self.out_feats), self.out_capacity,
                                       self.cand_capacity, _ptr(self.nnz), _ptr(self.workspace),
                                       self.workspace.numel(), _stream(stream))
        _check(L, rc)
        return self.out_coords, self.out_feats, self.nnz


def attention_topk(extent, batch, coords, resp, k, topk_mode=ABS, *, out_capacity=None, workspace=None, stream=None,
                   sync=True):
    L = load_library()
    ndim = len(extent)
    coords = _dev(coords, torch.int32, "coords")
    resp = _dev(resp, torch.float32, "resp")
    rows, ch = resp.shape
    ext = _i32arr(extent)
    dev = resp.device
    if out_capacity is None:
        out_capacity = rows
    need = int(L.attention_topk_workspace(ndim, ext, int(batch), rows, ch))
    if need == 0:
        raise ScnnError(-1, "attention_topk_workspace: bad arguments")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out_coords = torch.empty((out_capacity, 1 + ndim), dtype=torch.int32, device=dev)
    out_feats = torch.empty((out_capacity, ch), dtype=torch.float32, device=dev)
    nnz = torch.zeros(NNZ_LEN, dtype=torch.int64, device=dev)
    rc = L.attention_topk(ndim, ext, int(batch), _ptr(coords), _ptr(resp), rows, ch, int(k), int(topk_mode),
                          _ptr(out_coords), _ptr(out_feats), int(out_capacity), _ptr(nnz), _ptr(workspace),
                          workspace.numel(), _stream(stream))
    _check(L, rc)
    return _finish(out_coords, out_feats, nnz, sync)


def sparse_relu(ndim, coords, feats, *, out_capacity=None, workspace=None, stream=None, sync=True):
    L = load_library()
    coords = _dev(coords, torch.int32, "coords")
    feats = _dev(feats, torch.float32, "feats")
    rows, ch = feats.shape
    dev = feats.device
    if out_capacity is None:
        out_capacity = rows
    need = int(L.sparse_relu_workspace(rows, ch))
    if need == 0:
        raise ScnnError(-1, "sparse_relu_workspace: bad arguments")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out_coords = torch.empty((out_capacity, 1 + ndim), dtype=torch.int32, device=dev)
    out_feats = torch.empty((out_capacity, ch), dtype=torch.float32, device=dev)
    nnz = torch.zeros(NNZ_LEN, dtype=torch.int64, device=dev)
    rc = L.sparse_relu(int(ndim), _ptr(coords), _ptr(feats), rows, ch, _ptr(out_coords), _ptr(out_feats),
                       int(out_capacity), _ptr(nnz), _ptr(workspace), workspace.numel(), _stream(stream))
    _check(L, rc)
    return _finish(out_coords, out_feats, nnz, sync)


def sparse_relu_static_max_rows() -> int:
    return int(load_library().sparse_relu_static_max_rows())


def sparse_relu_static(ndim, coords, feats, out_coords, out_feats, nnz, *, stream=None):
    """sparse_relu on the library's own scratch array: every buffer is the caller's, nothing is allocated here."""
    L = load_library()
    coords = _dev(coords, torch.int32, "coords")
    feats = _dev(feats, torch.float32, "feats")
    rows, ch = feats.shape
    rc = L.sparse_relu_static(int(ndim), _ptr(coords), _ptr(feats), rows, ch, _ptr(out_coords), _ptr(out_feats),
                              int(out_feats.shape[0]), _ptr(nnz), _stream(stream))
    _check(L, rc)


def sparse_maxpool(extent, batch, coords, feats, window=2, *, out_capacity=None, workspace=None, stream=None,
                   sync=True):
    L = load_library()
    ndim = len(extent)
    coords = _dev(coords, torch.int32, "coords")
    feats = _dev(feats, torch.float32, "feats")
    rows, ch = feats.shape
    ext = _i32arr(extent)
    dev = feats.device
    if out_capacity is None:
        out_capacity = rows
    need = int(L.sparse_maxpool_workspace(ndim, ext, int(batch), rows, ch))
    if need == 0:
        raise ScnnError(-1, "sparse_maxpool_workspace: bad arguments")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out_coords = torch.empty((out_capacity, 1 + ndim), dtype=torch.int32, device=dev)
    out_feats = torch.empty((out_capacity, ch), dtype=torch.float32, device=dev)
    nnz = torch.zeros(NNZ_LEN, dtype=torch.int64, device=dev)
    rc = L.sparse_maxpool(ndim, ext, int(batch), int(window), _ptr(coords), _ptr(feats), rows, ch, _ptr(out_coords),
                          _ptr(out_feats), int(out_capacity), _ptr(nnz), _ptr(workspace), workspace.numel(),
                          _stream(stream))
    _check(L, rc)
    return _finish(out_coords, out_feats, nnz, sync)


def sparse_to_dense(extent, batch, coords, feats, *, rows_dev=None, out=None, stream=None):
    """Dense fp32 [batch, channels, *extent] holding the rows' values, zero elsewhere."""
    L = load_library()
    coords = _dev(coords, torch.int32, "coords")
    feats = _dev(feats, torch.float32, "feats")
    rows, ch = feats.shape
    if out is None:
        out = torch.empty((int(batch), ch, *[int(e) for e in extent]), dtype=torch.float32, device=feats.device)
    _check(L, L.sparse_to_dense(len(extent), _i32arr(extent), int(batch), _ptr(coords), _ptr(feats), rows,
                                _ptr(rows_dev), ch, _ptr(out), _stream(stream)))
    return out


def density_regulariser(out_feats, n_sites_total, rho_up, o, b1, b2, lam, w, *, rows_dev=None, want_grad=True,
                        stream=None):
    """Eq. 4.  Returns (result double[4] = {rho, b, lambda * sum (w + b)^2, entries} on the device, grad_w or None)."""
    L = load_library()
    out_feats = _dev(out_feats, torch.float32, "out_feats")
    w = _dev(w, torch.float32, "w")
    rows, ch = out_feats.shape
    dev = w.device
    grad = torch.empty_like(w) if want_grad else None
    result = torch.zeros(4, dtype=torch.float64, device=dev)
    need = int(L.density_regulariser_workspace())
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(L, L.density_regulariser(_ptr(out_feats), rows, _ptr(rows_dev), ch, int(n_sites_total), float(rho_up),
                                    float(o), float(b1), float(b2), float(lam), _ptr(w), w.numel(), _ptr(grad),
                                    _ptr(result), _ptr(ws), need, _stream(stream)))
    return result, grad


def prune_weights(w, warned, eps, *, stream=None):
    """One-warning-shot pruning, in place on w (fp32) and warned (uint8).  Returns counts int64[2] on the device."""
    L = load_library()
    if not (w.is_cuda and warned.is_cuda and w.dtype == torch.float32 and warned.dtype == torch.uint8):
        raise ValueError("w must be a float32 and warned a uint8 GPU tensor")
    if not (w.is_contiguous() and warned.is_contiguous()) or w.numel() != warned.numel():
        raise ValueError("w and warned must be contiguous and of equal size")
    counts = torch.zeros(2, dtype=torch.int64, device=w.device)
    _check(L, L.prune_weights(_ptr(w), _ptr(warned), w.numel(), float(eps), _ptr(counts), _stream(stream)))
    return counts


def validate_rows(extent, batch, coords, stream=None) -> None:
    """Raises ScnnError if coords are out of the grid (-1) or not strictly ascending (-4).  Synchronises."""
    L = load_library()
    coords = _dev(coords, torch.int32, "coords")
    ws = torch.empty(256, dtype=torch.uint8, device=coords.device)
    rc = L.scnn_validate_rows(len(extent), _i32arr(extent), int(batch), _ptr(coords), coords.shape[0], _ptr(ws), 256,
                              _stream(stream))
    _check(L, rc)


def profile_enable(on) -> None:
    """Per-stage HIP-event timing of sparse_conv_fwd calls made from this thread: False / 0 = off, True / 1 = every
    stage, 2 = only the convolution stage (two events per call), 3 = the same on every fourth call."""
    _check(load_library(), load_library().scnn_profile_enable(int(on)))


def profile_collect():
    """Waits for the recorded calls; returns ({stage name: total ms}, number of calls)."""
    L = load_library()
    n = L.scnn_profile_stage_count()
    ms = (ctypes.c_double * n)()
    calls = ctypes.c_int64(0)
    _check(L, L.scnn_profile_collect(ms, ctypes.byref(calls)))
    return {L.scnn_profile_stage_name(i).decode(): float(ms[i]) for i in range(n)}, int(calls.value)


def set_conv_path(path: int) -> None:
    """0 = choose the convolution kernel by shape and size, 1 = always the vector kernels, 2 = a matrix-core kernel
    whenever one takes the shape, 3 = the pair-list matrix-core kernel where it takes the shape."""
    L = load_library()
    _check(L, L.scnn_set_conv_path(int(path)))


def last_conv_kernel() -> str:
    """Kernel family launched by this thread's last sparse_conv_fwd call."""
    return load_library().scnn_last_conv_kernel().decode()


def calibration_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """Plain streaming copy of src into dst (same byte size, a multiple of 16)."""
    L = load_library()
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    _check(L, L.scnn_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)))
