"""Pins of the oracle's backward pass (Algorithm 2 with the masks of Eq. 3) against things other than itself:
automatic differentiation of a library convolution, a hand-worked example, the adjoint identities of a bilinear
map, and the structural facts the paper states (fixed shapes, zero stays zero)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from workloads import make_filter, random_sparse_sites


def _dense(extent, batch, coords, feats):
    d = np.zeros((batch, feats.shape[1], *extent), dtype=np.float64)
    for r in range(coords.shape[0]):
        d[(int(coords[r, 0]), slice(None)) + tuple(int(v) for v in coords[r, 1:])] = feats[r]
    return d


def _case(rng, extent, batch, c_in, c_out, ksize, density=0.25, gdensity=0.4, fdens=0.6, zero_frac=0.25):
    coords = random_sparse_sites(rng, extent, batch, density)
    feats = rng.normal(size=(coords.shape[0], c_in)).astype(np.float32)
    feats *= rng.random(feats.shape) >= zero_frac          # explicit zeros inside stored rows
    w = make_filter(rng, ksize, c_in, c_out, fdens, 0.5)
    g_coords = random_sparse_sites(rng, extent, batch, gdensity)
    g_feats = rng.normal(size=(g_coords.shape[0], c_out)).astype(np.float32)
    g_feats *= rng.random(g_feats.shape) >= zero_frac
    return coords, feats.astype(np.float32), w, g_coords, g_feats.astype(np.float32)


CASES = [((9, 7), 2, 3, 4, (3, 5)), ((6, 6), 1, 1, 1, (3, 3)), ((8, 5), 3, 2, 5, (1, 3)),
         ((6, 7, 5), 2, 3, 4, (3, 3, 5)), ((5, 5, 5), 1, 2, 2, (3, 3, 3)), ((4, 6, 7), 2, 1, 3, (5, 1, 3))]


# ---------------------------------------------------------------- B1: autograd of the library convolution, masked
@pytest.mark.parametrize("case", CASES)
def test_backward_equals_masked_autograd_of_library_convolution(case):
    extent, batch, c_in, c_out, ksize = case
    ndim = len(extent)
    rng = np.random.default_rng(100 + hash(case) % 1000)
    coords, feats, w, g_coords, g_feats = _case(rng, extent, batch, c_in, c_out, ksize)
    x = torch.tensor(_dense(extent, batch, coords, feats), requires_grad=True)
    wt = torch.from_numpy(w.astype(np.float64)).reshape(*ksize, c_in, c_out)
    wt = wt.permute(ndim + 1, ndim, *range(ndim)).contiguous().requires_grad_(True)  # [oc, ic, taps...]
    conv = torch.nn.functional.conv2d if ndim == 2 else torch.nn.functional.conv3d
    y = conv(x, wt, padding=[(s - 1) // 2 for s in ksize])
    gy = torch.from_numpy(_dense(extent, batch, g_coords, g_feats))
    (y * gy).sum().backward()
    dx = x.grad.numpy()
    dw = wt.grad.permute(*range(2, 2 + ndim), 1, 0).reshape(-1, c_in, c_out).numpy()
    want_data = np.stack([dx[(int(c[0]), slice(None)) + tuple(int(v) for v in c[1:])] for c in coords]) \
        if coords.shape[0] else np.zeros((0, c_in))
    want_data = want_data * (feats != 0)           # Eq. 3, first line
    want_filter = dw * (w != 0)                    # Eq. 3, second line
    bp_data, bp_filter = oracle.sparse_conv_bwd(extent, batch, coords, feats, ksize, w, g_coords, g_feats)
    assert bp_data.shape == feats.shape and bp_filter.shape == w.shape      # fixed shapes
    np.testing.assert_allclose(bp_data, want_data, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(bp_filter, want_filter, rtol=1e-6, atol=1e-6)
    assert np.array_equal(bp_data[feats == 0], np.zeros_like(bp_data[feats == 0]))
    assert np.array_equal(bp_filter[w == 0], np.zeros_like(bp_filter[w == 0]))


# ---------------------------------------------------------------- B2: a hand-worked example
def test_hand_worked_example_2d():
    # 3x3 grid, one sample, one channel in and out.  Inputs: x(0,0) = 2, x(1,1) = 3, and a stored zero at (2,2).
    # Filter (3x3, taps row-major over (d1, d2) in -1..1): w(-1,-1) = 5 [tap 0], w(0,0) = 7 [tap 4],
    # w(0,+1) = 11 [tap 5], everything else pruned (0).
    # Forward convention: an input at q seen through tap delta feeds output p = q - delta.
    # Gradient rows: g(0,0) = 1, g(1,0) = 10, g(1,1) = 100, g(2,2) = 1000.
    #   input (0,0): tap 0 -> p = (1,1): g = 100; tap 4 -> p = (0,0): g = 1; tap 5 -> p = (0,-1): outside.
    #     bp_data = 100*5 + 1*7 = 507
    #   input (1,1): tap 0 -> p = (2,2): g = 1000; tap 4 -> p = (1,1): g = 100; tap 5 -> p = (1,0): g = 10.
    #     bp_data = 1000*5 + 100*7 + 10*11 = 5810
    #   input (2,2) is a stored zero: no gradient.
    #   bp_filter: tap 0 = 100*2 + 1000*3 = 3200; tap 4 = 1*2 + 100*3 = 302; tap 5 = 10*3 = 30; pruned taps stay 0
    #   (tap 8 = delta (+1,+1) would otherwise collect g(0,0)*x(1,1) = 3).
    extent = (3, 3)
    coords = np.array([[0, 0, 0], [0, 1, 1], [0, 2, 2]], dtype=np.int32)
    feats = np.array([[2.0], [3.0], [0.0]], dtype=np.float32)
    w = np.zeros((9, 1, 1), dtype=np.float32)
    w[0], w[4], w[5] = 5.0, 7.0, 11.0
    g_coords = np.array([[0, 0, 0], [0, 1, 0], [0, 1, 1], [0, 2, 2]], dtype=np.int32)
    g_feats = np.array([[1.0], [10.0], [100.0], [1000.0]], dtype=np.float32)
    bp_data, bp_filter, info = oracle.sparse_conv_bwd(extent, 1, coords, feats, (3, 3), w, g_coords, g_feats,
                                                      return_info=True)
    assert bp_data.ravel().tolist() == [507.0, 5810.0, 0.0]
    assert bp_filter.ravel().tolist() == [3200.0, 0.0, 0.0, 0.0, 302.0, 30.0, 0.0, 0.0, 0.0]
    assert info["visits"] == 5  # (0,0): taps 0, 4; (1,1): taps 0, 4, 5


# ---------------------------------------------------------------- B3: adjoint identities with the forward oracle
@pytest.mark.parametrize("case", CASES)
def test_adjoint_identities_with_forward_pass(case):
    # y is bilinear in (x, w): <g, y> = <x, dL/dx> = <w, dL/dw>; the masked entries multiply zeros on the left.
    extent, batch, c_in, c_out, ksize = case
    rng = np.random.default_rng(200 + hash(case) % 1000)
    coords, feats, w, g_coords, g_feats = _case(rng, extent, batch, c_in, c_out, ksize)
    yc, yf = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, resp_only=True)
    gd = _dense(extent, batch, g_coords, g_feats)
    lhs = float((_dense(extent, batch, yc, yf) * gd).sum())
    bp_data, bp_filter = oracle.sparse_conv_bwd(extent, batch, coords, feats, ksize, w, g_coords, g_feats)
    scale = float(np.abs(_dense(extent, batch, yc, yf) * gd).sum()) + 1.0
    assert abs(float((feats.astype(np.float64) * bp_data).sum()) - lhs) <= 1e-5 * scale
    assert abs(float((w.astype(np.float64) * bp_filter).sum()) - lhs) <= 1e-5 * scale


# ---------------------------------------------------------------- B4: a single gradient entry reads the filter back
def test_single_gradient_entry_reads_filter_and_inputs_back():
    rng = np.random.default_rng(5)
    extent, ksize = (5, 6, 7), (3, 3, 3)
    occ = np.ones((1, *extent), dtype=bool)
    coords = np.argwhere(occ).astype(np.int32)                       # every site stored, all values non-zero
    feats = (rng.random((coords.shape[0], 2)) + 0.5).astype(np.float32)
    w = rng.normal(size=(27, 2, 3)).astype(np.float32)
    for site in [(2, 3, 3), (0, 0, 0), (4, 5, 6)]:
        for oc in range(3):
            g_coords = np.array([[0, *site]], dtype=np.int32)
            g_feats = np.zeros((1, 3), dtype=np.float32)
            g_feats[0, oc] = 1.0
            bp_data, bp_filter = oracle.sparse_conv_bwd(extent, 1, coords, feats, ksize, w, g_coords, g_feats)
            lin = {tuple(c[1:]): r for r, c in enumerate(coords)}
            want_data = np.zeros_like(feats)
            want_filter = np.zeros_like(w)
            for t, off in enumerate(itertools.product(range(3), range(3), range(3))):
                q = tuple(site[a] + off[a] - 1 for a in range(3))    # the input that feeds `site` through tap t
                if all(0 <= q[a] < extent[a] for a in range(3)):
                    want_data[lin[q]] = w[t, :, oc]
                    want_filter[t, :, oc] = feats[lin[q]]
            assert np.array_equal(bp_data, want_data)
            assert np.array_equal(bp_filter, want_filter)


# ---------------------------------------------------------------- B5: structure
def test_linearity_in_gradient_and_independence_of_samples():
    rng = np.random.default_rng(9)
    extent, ksize = (6, 5, 4), (3, 3, 3)
    coords, feats, w, g_coords, g_feats = _case(rng, extent, 2, 2, 3, ksize)
    d1, f1 = oracle.sparse_conv_bwd(extent, 2, coords, feats, ksize, w, g_coords, g_feats)
    d2, f2 = oracle.sparse_conv_bwd(extent, 2, coords, feats, ksize, w, g_coords, 2.0 * g_feats)
    assert np.array_equal(d2, 2.0 * d1) and np.array_equal(f2, 2.0 * f1)
    # bp_data of a sample depends on that sample's gradient rows only; bp_filter adds over samples
    parts = []
    for b in range(2):
        sel, gsel = coords[:, 0] == b, g_coords[:, 0] == b
        cb, gb = coords[sel].copy(), g_coords[gsel].copy()
        cb[:, 0] = 0
        gb[:, 0] = 0
        db, fb = oracle.sparse_conv_bwd(extent, 1, cb, feats[sel], ksize, w, gb, g_feats[gsel])
        assert np.array_equal(db, d1[sel])
        parts.append(fb.astype(np.float64))
    np.testing.assert_allclose(f1, parts[0] + parts[1], rtol=1e-6, atol=1e-6)


def test_empty_inputs_and_empty_gradient():
    extent, ksize = (4, 4), (3, 3)
    w = np.ones((9, 2, 3), dtype=np.float32)
    e_c, e_f = np.zeros((0, 3), np.int32), np.zeros((0, 2), np.float32)
    g_c, g_f = np.array([[0, 1, 1]], np.int32), np.ones((1, 3), np.float32)
    d, f = oracle.sparse_conv_bwd(extent, 1, e_c, e_f, ksize, w, g_c, g_f)
    assert d.shape == (0, 2) and not f.any()
    c, x = np.array([[0, 1, 1]], np.int32), np.ones((1, 2), np.float32)
    d, f = oracle.sparse_conv_bwd(extent, 1, c, x, ksize, w, np.zeros((0, 3), np.int32), np.zeros((0, 3), np.float32))
    assert d.shape == (1, 2) and not d.any() and not f.any()
