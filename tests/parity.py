"""Comparison rules between the HIP path and the oracle (test-side logic only).

Values must agree within 1e-5 relative / 1e-6 absolute (fp32, different
accumulation order).  Coordinate sets must be identical except for entries whose
score lies within that tolerance of the k-th largest score of their (sample,
channel) column, where either choice is accepted; entries with |v| <= 1e-6 may
be present on one side only (exact-cancellation case).
"""
from __future__ import annotations

import numpy as np

RTOL, ATOL = 1e-5, 1e-6


def lin_index(coords: np.ndarray, extent) -> np.ndarray:
    lin = np.zeros(coords.shape[0], dtype=np.int64)
    for a, e in enumerate(extent):
        lin = lin * int(e) + coords[:, 1 + a].astype(np.int64)
    return lin


def assert_rows_well_formed(coords, feats, extent, batch):
    """Strictly ascending (b, lin), coordinates in range, no all-zero row."""
    if coords.shape[0] == 0:
        return
    n = int(np.prod([int(e) for e in extent]))
    assert coords[:, 0].min() >= 0 and coords[:, 0].max() < batch
    for a, e in enumerate(extent):
        assert coords[:, 1 + a].min() >= 0 and coords[:, 1 + a].max() < e
    key = coords[:, 0].astype(np.int64) * n + lin_index(coords, extent)
    assert (np.diff(key) > 0).all(), "rows not strictly ascending"
    assert (feats != 0).any(axis=1).all(), "all-zero output row"


def column(coords, feats, extent, b, oc):
    """lin -> value of the non-zero entries of column (b, oc)."""
    sel = coords[:, 0] == b
    lin = lin_index(coords[sel], extent)
    v = feats[sel, oc]
    nz = v != 0
    return lin[nz], v[nz]


def check_column(all_lin, all_val, got_lin, got_val, k, mode, relu=False, where=""):
    """all_*: every non-zero response of the column from the oracle (before selection).
    got_*: the HIP path's surviving entries of that column.  Returns the band size."""
    score = np.abs(all_val) if mode == 0 else all_val
    order = np.lexsort((all_lin, -score.astype(np.float64)))
    n = len(all_lin)
    kept_idx = order[: min(k, n)] if k > 0 else order[:0]
    if 0 < k < n:
        tau = float(score[order[k - 1]])
        band_mask = np.abs(score.astype(np.float64) - tau) <= RTOL * abs(tau) + ATOL
    else:
        band_mask = np.zeros(n, dtype=bool)
    tiny = np.abs(all_val) <= ATOL
    kept_mask = np.zeros(n, dtype=bool)
    kept_mask[kept_idx] = True
    if relu:
        expect_mask = kept_mask & (all_val > 0)
    else:
        expect_mask = kept_mask
    pos = {int(l): i for i, l in enumerate(all_lin)}
    got = {int(l): float(v) for l, v in zip(got_lin, got_val)}
    # everything the oracle keeps outside the band must be there, with the right value
    for i in np.nonzero(expect_mask & ~band_mask & ~tiny)[0]:
        l = int(all_lin[i])
        assert l in got, f"{where}: entry lin={l} v={all_val[i]} missing"
    for l, v in got.items():
        if l not in pos:
            assert abs(v) <= ATOL, f"{where}: spurious entry lin={l} v={v}"
            continue
        i = pos[l]
        assert abs(v - float(all_val[i])) <= RTOL * abs(float(all_val[i])) + ATOL, \
            f"{where}: value mismatch lin={l}: {v} vs {all_val[i]}"
        assert expect_mask[i] or band_mask[i] or tiny[i], f"{where}: entry lin={l} v={v} should have been dropped"
    if not relu:
        slack = int(tiny.sum())
        assert abs(len(got) - int(expect_mask.sum())) <= slack, \
            f"{where}: kept count {len(got)} != {int(expect_mask.sum())}"
    return int(band_mask.sum())
