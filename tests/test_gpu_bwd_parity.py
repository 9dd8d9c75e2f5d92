"""GPU parity of the backward pass (Algorithm 2 with the masks of Eq. 3): the HIP library through its C ABI against
the CPU oracle on the same seeded inputs.

Tolerances.  Both results are sums of many signed products that largely cancel.  The vector kernels carry them in
fp64 and round once; the matrix-core kernels first add 32 products (bp_data) or the at most 128 products of one tap
within one 128-row tile (bp_filter) in fp32, which leaves a rounding error proportional to the sum of the magnitudes
of the products, A, not to the (cancelling) result: with fp32 unit roundoff u = 2^-24 = 6e-8, a chain of n products
is off by at most n * u times the magnitudes in the chain and typically (the errors add like a random walk) by a
fraction of u times them, so the whole sum is off by a fraction of u * A.  The bar on the matrix-core kernels is
1e-5 * |ref| + 1e-6 + c * A with c = 2e-8 (u / 3) for bp_data and c = 1e-7 (1.7 u) for bp_filter, whose fp32 chains
are four times longer; A comes from the oracle run on |x|, |w|, |g|.  The vector kernels (every shape outside the
matrix-core ones, and every shape under scnn_set_conv_path(1)) get no such term: 1e-5 * |ref| + 1e-6 alone.
Masked positions (x == 0, w == 0) must be exactly 0."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_1801_10585_amd as scnn
from workloads import make_config, make_filter, make_paper_runtime, random_sparse_sites

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL, ATOL, STOL_DATA, STOL_FILTER = 1e-5, 1e-6, 2e-8, 1e-7


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_bwd(extent, batch, coords, feats, ksize, w, g_coords, g_feats):
    d, f, info = scnn.sparse_conv_bwd(extent, batch, dev(coords), dev(feats), ksize, dev(w), dev(g_coords),
                                      dev(g_feats))
    assert int(info[0]) == coords.shape[0] and int(info[1]) == g_coords.shape[0]
    assert int(info[2]) == 0, f"status flags {int(info[2])}"
    return d.cpu().numpy(), f.cpu().numpy()


def magnitudes(extent, batch, coords, feats, ksize, w, gc, gf):
    """Sum of |product| behind every element of bp_data and bp_filter (same masks)."""
    return oracle.sparse_conv_bwd(extent, batch, coords, np.abs(feats), ksize, np.abs(w), gc, np.abs(gf))


def takes_matrix_cores(c_in, c_out):
    """The shapes whose backward pass runs on the fp32 matrix cores (stated at sparse_conv_bwd in the header)."""
    return c_out % 32 == 0 and c_out <= 128 and c_in % 16 == 0 and c_in <= 64


def check_data(got, ref, mag, feats, tag, matrix_cores):
    assert got.shape == ref.shape == feats.shape
    assert not got[feats == 0].any(), f"{tag}: gradient on a zero input value"
    err = np.abs(got.astype(np.float64) - ref)
    tol = RTOL * np.abs(ref) + ATOL + (STOL_DATA * mag if matrix_cores else 0.0)
    assert (err <= tol).all(), f"{tag}: bp_data off by {(err - tol).max():.3e} beyond tolerance at {np.argmax(err - tol)}"


def check_filter(got, ref, mag, w, tag, matrix_cores):
    assert got.shape == ref.shape == w.shape
    assert not got[w == 0].any(), f"{tag}: gradient on a pruned weight"
    err = np.abs(got.astype(np.float64) - ref)
    tol = RTOL * np.abs(ref) + ATOL + (STOL_FILTER * mag if matrix_cores else 0.0)
    assert (err <= tol).all(), f"{tag}: bp_filter off by {(err - tol).max():.3e} beyond tolerance"
    return float((err / np.maximum(tol, 1e-30)).max())


def gradient_rows(rng, extent, batch, coords, feats, ksize, w, rho_up, threads=1):
    """Gradient rows with the sparsity pattern of the layer's output (from the oracle's forward pass): random values
    where the output has an entry, zero where the selection dropped it."""
    yc, yf = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, rho_up=rho_up, threads=threads)
    g = rng.normal(size=yf.shape).astype(np.float32) * (yf != 0)
    return yc, g.astype(np.float32)


def full_check(extent, batch, coords, feats, ksize, w, gc, gf, tag, matrix_cores=None):
    """matrix_cores: whether the call runs on the matrix-core kernels (default: by shape, as the library chooses)."""
    if matrix_cores is None:
        matrix_cores = takes_matrix_cores(w.shape[1], w.shape[2])
    ref_d, ref_f = oracle.sparse_conv_bwd(extent, batch, coords, feats, ksize, w, gc, gf)
    mag_d, mag_f = magnitudes(extent, batch, coords, feats, ksize, w, gc, gf)
    got_d, got_f = gpu_bwd(extent, batch, coords, feats, ksize, w, gc, gf)
    check_data(got_d, ref_d, mag_d, feats, tag, matrix_cores)
    worst = check_filter(got_f, ref_f, mag_f, w, tag, matrix_cores)
    return got_d, got_f, worst


SMALL = [
    # extent, batch, c_in, c_out, ksize, density, filter density
    ((12, 9), 2, 1, 8, (3, 3), 0.3, 0.5),
    ((28, 28), 1, 3, 5, (3, 5), 0.2, 0.7),
    ((9, 10, 11), 2, 2, 3, (3, 3, 3), 0.15, 0.5),
    ((16, 16, 16), 3, 8, 4, (3, 3, 3), 0.1, 1.0),
    ((14, 12, 10), 1, 1, 1, (5, 3, 1), 0.2, 0.6),
    ((40, 40), 2, 17, 9, (5, 5), 0.1, 0.3),
]


@pytest.mark.parametrize("case", SMALL)
def test_backward_small_cases_every_element(case):
    extent, batch, c_in, c_out, ksize, density, fdens = case
    rng = np.random.default_rng(abs(hash(case)) % (2 ** 32))
    coords = random_sparse_sites(rng, extent, batch, density)
    feats = rng.normal(size=(coords.shape[0], c_in)).astype(np.float32)
    feats *= rng.random(feats.shape) >= 0.2
    w = make_filter(rng, ksize, c_in, c_out, fdens, 0.3)
    gc, gf = gradient_rows(rng, extent, batch, coords, feats, ksize, w, 0.2)
    say(f"bwd small {case}: rows={coords.shape[0]} g_rows={gc.shape[0]}")
    full_check(extent, batch, coords, feats, ksize, w, gc, gf, f"small {case}")
    # gradient rows unrelated to the input's neighbourhood (arbitrary sparse rows on the grid)
    gc2 = random_sparse_sites(rng, extent, batch, 0.3)
    gf2 = rng.normal(size=(gc2.shape[0], c_out)).astype(np.float32)
    full_check(extent, batch, coords, feats, ksize, w, gc2, gf2, f"small/random-g {case}")


WIDE = [
    # shapes that reach the matrix-core kernels: C_out = 16 or a multiple of 32 (<= 128), C_in a multiple of 16 (<= 64)
    ((20, 18, 16), 2, 16, 32, (3, 3, 3), 0.08, 0.5),
    ((24, 20, 22), 2, 32, 64, (3, 3, 3), 0.06, 1.0),
    ((18, 18, 18), 1, 48, 96, (3, 3, 3), 0.06, 0.5),
    ((16, 16, 16), 2, 64, 128, (3, 3, 3), 0.05, 0.3),
    ((48, 40), 3, 32, 32, (5, 5), 0.1, 0.5),
    ((14, 14, 14), 1, 64, 64, (5, 5, 5), 0.04, 0.3),
    # sixteen output channels: slabs of 16 output channels in the filter gradient, the half-chunk adjoint convolution
    ((20, 20, 20), 2, 16, 16, (3, 3, 3), 0.08, 1.0),
    ((18, 16, 20), 1, 32, 16, (3, 3, 3), 0.08, 0.6),
    ((36, 30), 2, 64, 16, (3, 3), 0.15, 1.0),
]


@pytest.mark.parametrize("case", WIDE)
@pytest.mark.parametrize("path", [0, 1])
def test_backward_wide_channels_both_kernel_families(case, path):
    extent, batch, c_in, c_out, ksize, density, fdens = case
    rng = np.random.default_rng(abs(hash(case)) % (2 ** 32))
    coords = random_sparse_sites(rng, extent, batch, density)
    feats = rng.normal(size=(coords.shape[0], c_in)).astype(np.float32)
    feats *= rng.random(feats.shape) >= 0.2
    w = make_filter(rng, ksize, c_in, c_out, fdens, 0.2)
    gc, gf = gradient_rows(rng, extent, batch, coords, feats, ksize, w, 0.3)
    say(f"bwd wide {case} path={path}: rows={coords.shape[0]} g_rows={gc.shape[0]}")
    scnn.set_conv_path(path)
    try:
        d1, f1, worst = full_check(extent, batch, coords, feats, ksize, w, gc, gf, f"wide {case} path={path}",
                                   matrix_cores=(path == 0))
        d2, f2 = gpu_bwd(extent, batch, coords, feats, ksize, w, gc, gf)
        assert np.array_equal(f1, f2), "bp_filter is not reproducible"
        if path == 1:
            assert np.array_equal(d1, d2), "bp_data of the vector kernel is not reproducible"
    finally:
        scnn.set_conv_path(0)
    say(f"  worst bp_filter error / tolerance = {worst:.3f}")


def test_backward_integer_data_is_exact():
    # small integers: every product and partial sum is exact in fp32, so both kernel families must match bit for bit
    rng = np.random.default_rng(77)
    extent, batch, c_in, c_out, ksize = (20, 20, 20), 2, 32, 64, (3, 3, 3)
    coords = random_sparse_sites(rng, extent, batch, 0.07)
    feats = rng.integers(-3, 4, size=(coords.shape[0], c_in)).astype(np.float32)
    w = rng.integers(-2, 3, size=(27, c_in, c_out)).astype(np.float32)
    gc = random_sparse_sites(rng, extent, batch, 0.2)
    gf = rng.integers(-3, 4, size=(gc.shape[0], c_out)).astype(np.float32)
    ref_d, ref_f = oracle.sparse_conv_bwd(extent, batch, coords, feats, ksize, w, gc, gf)
    for path in (0, 1):
        scnn.set_conv_path(path)
        try:
            d, f = gpu_bwd(extent, batch, coords, feats, ksize, w, gc, gf)
        finally:
            scnn.set_conv_path(0)
        assert np.array_equal(d, ref_d) and np.array_equal(f, ref_f), f"path {path}"


def test_backward_config4_full_size_sampled():
    wl = make_config(4)
    L = wl.layers[0]
    w = wl.filters[0]
    rng = np.random.default_rng(44)
    gc, gf = gradient_rows(rng, wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, w, L.rho_up, threads=16)
    say(f"bwd cfg4 rows={wl.coords.shape[0]} g_rows={gc.shape[0]}")
    got_d, got_f = gpu_bwd(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, w, gc, gf)
    # bp_data: a row depends on the gradient rows only -> the oracle on a sample of the input rows (one in ten)
    pick = np.sort(rng.choice(wl.coords.shape[0], size=(wl.coords.shape[0] + 9) // 10, replace=False))
    ref_d, _ = oracle.sparse_conv_bwd(wl.extent, wl.batch, wl.coords[pick], wl.feats[pick], L.ksize, w, gc, gf)
    mag_d, _ = magnitudes(wl.extent, wl.batch, wl.coords[pick], wl.feats[pick], L.ksize, w, gc, gf)
    check_data(got_d[pick], ref_d, mag_d, wl.feats[pick], "cfg4", True)
    say(f"bwd cfg4 bp_data: {len(pick)} rows compared")
    # bp_filter: element (t, ic, oc) depends on channel ic of the input and channel oc of the gradient only ->
    # blocks of 4 x 8 (ic, oc) pairs, all 27 taps each: 128 slices of the 2048
    worst = 0.0
    for _ in range(4):
        ics = np.sort(rng.choice(L.c_in, size=4, replace=False))
        ocs = np.sort(rng.choice(L.c_out, size=8, replace=False))
        xs, gs = np.ascontiguousarray(wl.feats[:, ics]), np.ascontiguousarray(gf[:, ocs])
        wsl = np.ascontiguousarray(w[:, ics][:, :, ocs])
        _, ref_f = oracle.sparse_conv_bwd(wl.extent, wl.batch, wl.coords, xs, L.ksize, wsl, gc, gs)
        _, mag = magnitudes(wl.extent, wl.batch, wl.coords, xs, L.ksize, wsl, gc, gs)
        worst = max(worst, check_filter(got_f[:, ics][:, :, ocs], ref_f, mag, wsl, f"cfg4 ic={ics} oc={ocs}", True))
    say(f"bwd cfg4 worst bp_filter error / tolerance = {worst:.3f}")
    assert not got_f[w == 0].any() and not got_d[wl.feats == 0].any()


@pytest.mark.parametrize("r,rho_f", [(32, 1.0), (64, 0.1), (128, 1.0)])
def test_backward_paper_runtime_workload(r, rho_f):
    wl = make_paper_runtime(r, rho_f)
    L = wl.layers[0]
    rng = np.random.default_rng(r)
    gc, gf = gradient_rows(rng, wl.extent, 1, wl.coords, wl.feats, L.ksize, wl.filters[0], L.rho_up)
    say(f"bwd paper runtime r={r} rho_f={rho_f} rows={wl.coords.shape[0]} g_rows={gc.shape[0]}")
    full_check(wl.extent, 1, wl.coords, wl.feats, L.ksize, wl.filters[0], gc, gf, wl.name)


def test_backward_config1_2d_and_config3_layer1():
    for idx in (1, 3):
        wl = make_config(idx)
        L = wl.layers[0]
        rng = np.random.default_rng(idx)
        gc, gf = gradient_rows(rng, wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], L.rho_up,
                               threads=16)
        say(f"bwd cfg{idx} rows={wl.coords.shape[0]} g_rows={gc.shape[0]}")
        if idx == 1:
            full_check(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], gc, gf, "cfg1")
        else:
            # 16 -> 32 channels at 64^3, batch 8: the oracle on one sample
            sel, gsel = wl.coords[:, 0] == 5, gc[:, 0] == 5
            cb, gb = wl.coords[sel].copy(), gc[gsel].copy()
            cb[:, 0] = 0
            gb[:, 0] = 0
            got_d, got_f = gpu_bwd(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], gc, gf)
            ref_d, _ = oracle.sparse_conv_bwd(wl.extent, 1, cb, wl.feats[sel], L.ksize, wl.filters[0], gb, gf[gsel])
            mag_d, _ = magnitudes(wl.extent, 1, cb, wl.feats[sel], L.ksize, wl.filters[0], gb, gf[gsel])
            check_data(got_d[sel], ref_d, mag_d, wl.feats[sel], "cfg3-L1 sample 5", True)
            assert not got_f[wl.filters[0] == 0].any()


def test_backward_empty_operands():
    extent, ksize = (8, 8, 8), (3, 3, 3)
    rng = np.random.default_rng(1)
    w = make_filter(rng, ksize, 4, 6, 0.5, 0.3)
    coords = random_sparse_sites(rng, extent, 2, 0.1)
    feats = rng.normal(size=(coords.shape[0], 4)).astype(np.float32)
    e_gc, e_gf = np.zeros((0, 4), np.int32), np.zeros((0, 6), np.float32)
    d, f = gpu_bwd(extent, 2, coords, feats, ksize, w, e_gc, e_gf)
    assert d.shape == feats.shape and not d.any() and not f.any()
    gc = random_sparse_sites(rng, extent, 2, 0.2)
    gf = rng.normal(size=(gc.shape[0], 6)).astype(np.float32)
    d, f = gpu_bwd(extent, 2, np.zeros((0, 4), np.int32), np.zeros((0, 4), np.float32), ksize, w, gc, gf)
    assert d.shape == (0, 4) and f.shape == w.shape and not f.any()
    # every weight pruned: nothing flows
    d, f = gpu_bwd(extent, 2, coords, feats, ksize, np.zeros_like(w), gc, gf)
    assert not d.any() and not f.any()


def test_backward_reports_bad_arguments_and_unsorted_rows():
    extent, ksize = (8, 8), (3, 3)
    rng = np.random.default_rng(2)
    w = make_filter(rng, ksize, 2, 3, 1.0, 0.3)
    coords = random_sparse_sites(rng, extent, 1, 0.3)
    feats = rng.normal(size=(coords.shape[0], 2)).astype(np.float32)
    gc = random_sparse_sites(rng, extent, 1, 0.3)
    gf = rng.normal(size=(gc.shape[0], 3)).astype(np.float32)
    with pytest.raises(scnn.ScnnError):
        scnn.sparse_conv_bwd(extent, 1, dev(coords), dev(feats), (2, 3), dev(w[:6]), dev(gc), dev(gf))
    with pytest.raises(ValueError):
        scnn.sparse_conv_bwd(extent, 1, dev(coords), dev(feats), ksize, dev(w), dev(gc), dev(gf[:, :2]))
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(scnn.ScnnError):
        scnn.sparse_conv_bwd(extent, 1, dev(coords), dev(feats), ksize, dev(w), dev(gc), dev(gf), workspace=small)
    _, _, info = scnn.sparse_conv_bwd(extent, 1, dev(coords), dev(feats), ksize, dev(w), dev(gc[::-1].copy()),
                                      dev(gf))
    assert int(info[2]) & scnn.FLAG_UNSORTED
    bad = coords.copy()
    bad[0, 1] = 99
    _, _, info = scnn.sparse_conv_bwd(extent, 1, dev(bad), dev(feats), ksize, dev(w), dev(gc), dev(gf))
    assert int(info[2]) & scnn.FLAG_BAD_COORD
