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
    """all_*: every non-zero response of the column from the oracle (before selection), ascending lin.
    got_*: the HIP path's surviving entries of that column, ascending lin.  Returns the band size."""
    all_lin = np.asarray(all_lin, dtype=np.int64)
    all_val = np.asarray(all_val)
    got_lin = np.asarray(got_lin, dtype=np.int64)
    got_val = np.asarray(got_val)
    n = len(all_lin)
    assert n < 2 or (np.diff(all_lin) > 0).all(), f"{where}: oracle column not ascending"
    score = np.abs(all_val) if mode == 0 else all_val
    # descending score, ties by ascending lin (the input is ascending in lin and the sort is stable)
    order = np.argsort(-score.astype(np.float64), kind="stable")
    kept_mask = np.zeros(n, dtype=bool)
    if k > 0:
        kept_mask[order[: min(k, n)]] = True
    if 0 < k < n:
        tau = float(score[order[k - 1]])
        band_mask = np.abs(score.astype(np.float64) - tau) <= RTOL * abs(tau) + ATOL
    else:
        band_mask = np.zeros(n, dtype=bool)
    tiny = np.abs(all_val) <= ATOL
    expect_mask = kept_mask & (all_val > 0) if relu else kept_mask
    # where each of the HIP path's entries sits in the oracle's column
    idx = np.searchsorted(all_lin, got_lin)
    idx_c = np.minimum(idx, max(n - 1, 0))
    known = (idx < n) & (all_lin[idx_c] == got_lin) if n else np.zeros(len(got_lin), dtype=bool)
    # everything the oracle keeps outside the band must be there
    present = np.zeros(n, dtype=bool)
    present[idx_c[known]] = True
    missing = np.nonzero(expect_mask & ~band_mask & ~tiny & ~present)[0]
    assert len(missing) == 0, f"{where}: {len(missing)} entries missing, first lin={all_lin[missing[0]]} v={all_val[missing[0]]}"
    # an entry the oracle does not have at all must be a rounding residue
    spurious = np.nonzero(~known & (np.abs(got_val) > ATOL))[0]
    assert len(spurious) == 0, f"{where}: spurious entry lin={got_lin[spurious[0]]} v={got_val[spurious[0]]}"
    # values, and nothing kept that should have been dropped
    ref = all_val[idx_c[known]].astype(np.float64)
    bad = np.nonzero(np.abs(got_val[known].astype(np.float64) - ref) > RTOL * np.abs(ref) + ATOL)[0]
    assert len(bad) == 0, \
        f"{where}: value mismatch lin={got_lin[known][bad[0]]}: {got_val[known][bad[0]]} vs {ref[bad[0]]} ({len(bad)} in all)"
    ok = (expect_mask | band_mask | tiny)[idx_c[known]]
    assert ok.all(), f"{where}: entry lin={got_lin[known][~ok][0]} v={got_val[known][~ok][0]} should have been dropped"
    if not relu:
        slack = int(tiny.sum())
        assert abs(len(got_lin) - int(expect_mask.sum())) <= slack, \
            f"{where}: kept count {len(got_lin)} != {int(expect_mask.sum())}"
    return int(band_mask.sum())
