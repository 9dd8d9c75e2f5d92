"""Brute-force dense statement of the layer, for pinning the oracle on tiny grids.

Independent of oracle/ and of the HIP package: the sparse map is scattered to a
dense array, convolved as a plain zero-padded cross-correlation with python /
numpy loops in float64, and the k-selection is a full python sort.  Only usable
for tiny inputs.
"""
from __future__ import annotations

import itertools

import numpy as np


def scatter_dense(extent, batch, coords, feats):
    c = feats.shape[1]
    x = np.zeros((batch, c, *extent), dtype=np.float64)
    for r in range(coords.shape[0]):
        idx = (int(coords[r, 0]), slice(None)) + tuple(int(v) for v in coords[r, 1:])
        x[idx] = feats[r].astype(np.float64)
    return x


def dense_cross_correlation(x, w, ksize):
    """out[b, oc, p] = sum_{delta, ic} w[tap(delta), ic, oc] * x[b, ic, p + delta], zero outside."""
    batch, c_in = x.shape[:2]
    extent = x.shape[2:]
    d = len(extent)
    c_out = w.shape[2]
    h = [(s - 1) // 2 for s in ksize]
    out = np.zeros((batch, c_out, *extent), dtype=np.float64)
    for p in itertools.product(*[range(e) for e in extent]):
        for t, off in enumerate(itertools.product(*[range(s) for s in ksize])):
            q = tuple(p[a] + off[a] - h[a] for a in range(d))
            if any(q[a] < 0 or q[a] >= extent[a] for a in range(d)):
                continue
            for b in range(batch):
                xv = x[(b, slice(None)) + q]          # [c_in]
                out[(b, slice(None)) + p] += xv @ w[t].astype(np.float64)  # [c_in] @ [c_in, c_out]
    return out


def lin_of(p, extent):
    lin = 0
    for a, e in enumerate(extent):
        lin = lin * e + p[a]
    return lin


def layer_dense(extent, batch, coords, feats, ksize, w, bias=None, k=None, mode=0, relu=False, pool=False):
    """Returns dict {(b, site tuple, oc): float32 value} of surviving entries, and the output extent."""
    extent = tuple(int(e) for e in extent)
    x = scatter_dense(extent, batch, coords, feats)
    resp = dense_cross_correlation(x, w, ksize).astype(np.float32)
    c_out = w.shape[2]
    n_sites = int(np.prod(extent))
    if k is None:
        k = n_sites
    kept = {}
    for b in range(batch):
        for oc in range(c_out):
            cand = []
            for p in itertools.product(*[range(e) for e in extent]):
                v = np.float32(resp[(b, oc) + p])
                if v == 0:
                    continue
                if bias is not None:
                    v = np.float32(v + np.float32(bias[oc]))
                    if v == 0:
                        continue
                score = abs(float(v)) if mode == 0 else float(v)
                cand.append((-score, lin_of(p, extent), p, v))
            cand.sort(key=lambda c: (c[0], c[1]))
            for _, _, p, v in cand[:k]:
                kept[(b, p, oc)] = v
    if relu:
        kept = {key: v for key, v in kept.items() if v > 0}
    out_extent = extent
    if pool:
        pooled = {}
        for (b, p, oc), v in kept.items():
            pp = tuple(c // 2 for c in p)
            key = (b, pp, oc)
            if key not in pooled or v > pooled[key]:
                pooled[key] = v
        kept = pooled
        out_extent = tuple((e + 1) // 2 for e in extent)
    return kept, out_extent


def entries_to_rows(kept, extent, channels):
    sites = sorted({(b, lin_of(p, extent), p) for (b, p, _) in kept})
    coords = np.zeros((len(sites), 1 + len(extent)), dtype=np.int32)
    feats = np.zeros((len(sites), channels), dtype=np.float32)
    row_of = {}
    for i, (b, _, p) in enumerate(sites):
        coords[i, 0] = b
        coords[i, 1:] = p
        row_of[(b, p)] = i
    for (b, p, oc), v in kept.items():
        feats[row_of[(b, p)], oc] = v
    return coords, feats


def rows_to_entries(coords, feats):
    out = {}
    for r in range(coords.shape[0]):
        for c in range(feats.shape[1]):
            if feats[r, c] != 0:
                out[(int(coords[r, 0]), tuple(int(v) for v in coords[r, 1:]), c)] = feats[r, c]
    return out
