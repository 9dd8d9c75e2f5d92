"""Host-side bookkeeping for the benchmark: work and traffic counts (no layer arithmetic)."""
from __future__ import annotations

import itertools
from typing import Sequence

import numpy as np


def count_mac_nz(extent: Sequence[int], coords: np.ndarray, feats: np.ndarray, ksize: Sequence[int],
                 w: np.ndarray) -> int:
    """Non-zero multiply-adds of the convolution (the MAC term of the paper's Eq. 1):
    #{(row q, ic, tap, oc): feats[q, ic] != 0, w[tap, ic, oc] != 0, q - delta inside the grid}."""
    d = len(extent)
    h = [(s - 1) // 2 for s in ksize]
    nz_in = feats != 0                      # [rows, c_in]
    nnz_w = (w != 0).sum(axis=2)            # [T, c_in]
    total = 0
    for t, off in enumerate(itertools.product(*[range(s) for s in ksize])):
        if not nnz_w[t].any():
            continue
        ok = np.ones(coords.shape[0], dtype=bool)
        for a in range(d):
            p = coords[:, 1 + a] - (off[a] - h[a])
            ok &= (p >= 0) & (p < extent[a])
        cnt = nz_in[ok].sum(axis=0)         # [c_in]
        total += int((cnt.astype(np.int64) * nnz_w[t].astype(np.int64)).sum())
    return total


def count_bwd_visits(extent: Sequence[int], batch: int, coords: np.ndarray, feats: np.ndarray, ksize: Sequence[int],
                     w: np.ndarray, g_coords: np.ndarray) -> int:
    """Loop-nest visits of the backward pass that meet a stored gradient row (each visit is one multiply-add into
    bp_data and one into bp_filter):
    #{(row q, ic, tap, oc): feats[q, ic] != 0, w[tap, ic, oc] != 0, the gradient has a row at q - delta}."""
    d = len(extent)
    h = [(s - 1) // 2 for s in ksize]
    n = int(np.prod([int(e) for e in extent]))
    occ = np.zeros(batch * n, dtype=bool)
    glin = np.zeros(g_coords.shape[0], dtype=np.int64)
    for a in range(d):
        glin = glin * int(extent[a]) + g_coords[:, 1 + a]
    occ[g_coords[:, 0].astype(np.int64) * n + glin] = True
    nz_in = feats != 0
    nnz_w = (w != 0).sum(axis=2)
    total = 0
    for t, off in enumerate(itertools.product(*[range(s) for s in ksize])):
        if not nnz_w[t].any():
            continue
        ok = np.ones(coords.shape[0], dtype=bool)
        lin = np.zeros(coords.shape[0], dtype=np.int64)
        for a in range(d):
            p = coords[:, 1 + a].astype(np.int64) - (off[a] - h[a])
            ok &= (p >= 0) & (p < extent[a])
            lin = lin * int(extent[a]) + np.clip(p, 0, extent[a] - 1)
        ok &= occ[coords[:, 0].astype(np.int64) * n + lin]
        cnt = nz_in[ok].sum(axis=0)
        total += int((cnt.astype(np.int64) * nnz_w[t].astype(np.int64)).sum())
    return total


def algorithmic_bytes(ndim: int, nnz_in: int, c_in: int, taps: int, c_out: int, n_cand: int, rows_out: int) -> dict:
    """Bytes the method itself must move: inputs, filter, outputs, plus one write and one read of the
    candidate response matrix (no output can be emitted before its whole (sample, channel) column is known)."""
    b_in = nnz_in * (4 * (1 + ndim) + 4 * c_in)
    b_w = 4 * taps * c_in * c_out
    b_out = rows_out * (4 * (1 + ndim) + 4 * c_out)
    b_resp = 2 * 4 * n_cand * c_out + 4 * n_cand * (1 + ndim)
    return {"min": b_in + b_w + b_out, "alg": b_in + b_w + b_out + b_resp, "resp": b_resp}
