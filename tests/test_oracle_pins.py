"""Pins for the CPU oracle: brute force, library special cases, closed forms, invariants.

None of these tests touches the HIP library.  Each pin is chosen so that a
plausible slip in the oracle (dropped term, wrong sign of the tap offset,
transposed filter operand, wrong tie rule, off-by-one in k) fails at least one.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from tests.dense_bruteforce import entries_to_rows, layer_dense, rows_to_entries
from workloads import make_config, make_filter, random_sparse_sites, sort_rows

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _random_case(rng, ndim, extent, batch, c_in, c_out, ksize, density, fdens, dyadic=False):
    coords = random_sparse_sites(rng, extent, batch, density)
    if dyadic:
        feats = rng.integers(-3, 4, size=(coords.shape[0], c_in)).astype(np.float32) * 0.5
        w = rng.integers(-2, 3, size=(int(np.prod(ksize)), c_in, c_out)).astype(np.float32) * 0.25
        w *= (rng.random(w.shape) < fdens)
    else:
        feats = rng.normal(size=(coords.shape[0], c_in)).astype(np.float32)
        feats *= (rng.random(feats.shape) < 0.8)
        w = make_filter(rng, ksize, c_in, c_out, fdens, 0.5)
    return coords, feats.astype(np.float32), w.astype(np.float32)


def _assert_rows_equal(got, want, exact=True):
    gc, gf = got
    wc, wf = want
    assert gc.shape == wc.shape, (gc.shape, wc.shape)
    assert np.array_equal(gc, wc)
    if exact:
        assert np.array_equal(gf, wf)
    else:
        assert np.array_equal(gf != 0, wf != 0)
        np.testing.assert_allclose(gf, wf, rtol=1e-6, atol=1e-7)


# ---------------------------------------------------------------- P1: brute force on tiny inputs
CASES_2D = [((5, 6), 2, 2, 3, (3, 3)), ((7, 4), 1, 1, 2, (3, 3)), ((6, 6), 1, 3, 2, (5, 3)), ((8, 8), 2, 1, 4, (1, 3))]
CASES_3D = [((4, 5, 3), 2, 2, 2, (3, 3, 3)), ((5, 5, 5), 1, 1, 3, (3, 3, 3)), ((6, 4, 5), 1, 2, 2, (3, 1, 5))]


@pytest.mark.parametrize("case", CASES_2D + CASES_3D)
@pytest.mark.parametrize("mode", [oracle.ABS, oracle.SIGNED])
@pytest.mark.parametrize("fuse", [(False, False), (True, False), (False, True), (True, True)])
@pytest.mark.parametrize("dyadic", [False, True])
def test_oracle_matches_bruteforce(case, mode, fuse, dyadic):
    extent, batch, c_in, c_out, ksize = case
    rng = np.random.default_rng(hash((extent, batch, c_in, c_out, ksize, mode, fuse, dyadic)) % (2 ** 32))
    coords, feats, w = _random_case(rng, len(extent), extent, batch, c_in, c_out, ksize, 0.3, 0.6, dyadic)
    n = int(np.prod(extent))
    bias = None
    if rng.random() < 0.5:
        bias = (rng.integers(-2, 3, size=c_out) * 0.25).astype(np.float32) if dyadic else \
            rng.normal(size=c_out).astype(np.float32)
    for k in (0, 1, 3, n // 4, n):
        kept, oext = layer_dense(extent, batch, coords, feats, ksize, w, bias, k, mode, fuse[0], fuse[1])
        want = entries_to_rows(kept, oext, c_out)
        got = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, bias, k=k, topk_mode=mode,
                                     relu=fuse[0], pool=fuse[1])
        _assert_rows_equal(got, want, exact=dyadic)


def test_tie_break_lower_linear_index_wins():
    # four equal responses in one channel, k = 2: the two lowest lin survive
    extent = (4, 4)
    coords = np.array([[0, 0, 3], [0, 1, 1], [0, 2, 2], [0, 3, 0]], dtype=np.int32)
    feats = np.ones((4, 1), dtype=np.float32)
    w = np.zeros((9, 1, 1), dtype=np.float32)
    w[4, 0, 0] = -2.0  # centre tap only: output = -2 at each input site
    c, f = oracle.sparse_conv_fwd(extent, 1, coords, feats, (3, 3), w, k=2)
    assert c.tolist() == [[0, 0, 3], [0, 1, 1]] and f.ravel().tolist() == [-2.0, -2.0]
    # signed mode with mixed signs: +1 beats -2; abs mode: -2 beats +1
    feats2 = np.array([[1.0], [-0.5], [1.0], [-0.5]], dtype=np.float32)  # responses -2, +1, -2, +1
    c, f = oracle.sparse_conv_fwd(extent, 1, coords, feats2, (3, 3), w, k=1, topk_mode=oracle.SIGNED)
    assert c.tolist() == [[0, 1, 1]] and f.ravel().tolist() == [1.0]
    c, f = oracle.sparse_conv_fwd(extent, 1, coords, feats2, (3, 3), w, k=1, topk_mode=oracle.ABS)
    assert c.tolist() == [[0, 0, 3]] and f.ravel().tolist() == [-2.0]


# ---------------------------------------------------------------- P2: library special case (k = N)
@pytest.mark.parametrize("ndim", [2, 3])
def test_full_k_equals_library_convolution(ndim):
    rng = np.random.default_rng(7 + ndim)
    extent = (9, 7) if ndim == 2 else (6, 7, 5)
    ksize = (3, 5) if ndim == 2 else (3, 3, 5)
    batch, c_in, c_out = 2, 3, 4
    coords, feats, w = _random_case(rng, ndim, extent, batch, c_in, c_out, ksize, 0.2, 0.7)
    x = torch.zeros((batch, c_in, *extent), dtype=torch.float64)
    for r in range(coords.shape[0]):
        x[(int(coords[r, 0]), slice(None)) + tuple(int(v) for v in coords[r, 1:])] = torch.from_numpy(
            feats[r].astype(np.float64))
    wt = torch.from_numpy(w.astype(np.float64)).reshape(*ksize, c_in, c_out)
    wt = wt.permute(ndim + 1, ndim, *range(ndim)).contiguous()  # [oc, ic, taps...]
    pad = [(s - 1) // 2 for s in ksize]
    conv = torch.nn.functional.conv2d if ndim == 2 else torch.nn.functional.conv3d
    y = conv(x, wt, padding=pad).numpy().astype(np.float32)
    c, f = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, k=int(np.prod(extent)))
    dense = np.zeros_like(y)
    for r in range(c.shape[0]):
        dense[(int(c[r, 0]), slice(None)) + tuple(int(v) for v in c[r, 1:])] = f[r]
    np.testing.assert_allclose(dense, y, rtol=1e-6, atol=1e-7)
    # every non-zero library output must be a stored entry and vice versa
    assert np.array_equal(dense != 0, y != 0)


# ---------------------------------------------------------------- P3: delta input reflects the filter
def test_delta_input_reflects_filter_and_clips_at_corner():
    rng = np.random.default_rng(3)
    extent, ksize = (5, 6, 7), (3, 3, 3)
    w = rng.normal(size=(27, 1, 2)).astype(np.float32)
    for site in [(2, 3, 3), (0, 0, 0), (4, 5, 6), (0, 3, 6)]:
        coords = np.array([[0, *site]], dtype=np.int32)
        c, f = oracle.sparse_conv_fwd(extent, 1, coords, np.ones((1, 1), np.float32), ksize, w, k=10 ** 6)
        got = {tuple(c[r, 1:]): f[r] for r in range(c.shape[0])}
        want = {}
        for t, off in enumerate(itertools.product(range(3), range(3), range(3))):
            delta = tuple(o - 1 for o in off)
            p = tuple(site[a] - delta[a] for a in range(3))
            if all(0 <= p[a] < extent[a] for a in range(3)):
                want[p] = w[t, 0]
        assert set(got) == set(want)
        for p in want:
            assert np.array_equal(got[p], want[p])


# ---------------------------------------------------------------- P4: fill-in factor (Fig. 3 caption)
def test_isolated_voxels_fill_in_27x_and_sparse_filter_taps():
    extent = (12, 12, 12)
    sites = [(2, 2, 2), (2, 6, 9), (7, 3, 5), (9, 9, 9)]  # pairwise Chebyshev distance >= 3, interior
    coords = np.array([[0, *s] for s in sites], dtype=np.int32)
    feats = np.ones((4, 1), np.float32)
    rng = np.random.default_rng(0)
    w = (rng.random((27, 1, 1)) + 0.5).astype(np.float32)
    c, _ = oracle.sparse_conv_fwd(extent, 1, coords, feats, (3, 3, 3), w, k=12 ** 3)
    assert c.shape[0] == 27 * len(sites)
    w2 = w.copy()
    w2[[0, 5, 13, 20, 26]] = 0
    c, _ = oracle.sparse_conv_fwd(extent, 1, coords, feats, (3, 3, 3), w2, k=12 ** 3)
    assert c.shape[0] == 22 * len(sites)


# ---------------------------------------------------------------- P5: Table 1 closed form
def test_table1_memory_closed_form_and_per_channel_k():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_memory.txt")) if l.strip() and l[0] != "#"]
    batch, depth = 32, 8
    for r_s, s32, s64, tmp in rows:
        r = int(r_s)
        k = oracle.k_from_rho(1.0 / r, r ** 3)
        assert k == r * r
        entries = k * batch * depth  # k per (sample, channel)
        gb64 = entries * (8 + 4) / 1e9
        gb32 = entries * (4 + 4) / 1e9
        gbtmp = 8 * r ** 3 / 1e9
        def close(val, printed, tol_units=0.6):
            p = float(printed)
            if np.isnan(p):
                return True
            digits = len(printed.split("e")[0].replace(".", "").lstrip("0")) or 1
            return abs(val - p) <= tol_units * 10 ** (np.floor(np.log10(p)) - digits + 1) + 1e-12
        assert close(gb64, s64), (r, gb64, s64)
        assert close(gb32, s32), (r, gb32, s32)
        assert close(gbtmp, tmp, 1.0), (r, gbtmp, tmp)  # the table truncates 0.0168 to 0.016
    # and the oracle's output really holds exactly k entries per (sample, channel) when enough candidates exist
    rng = np.random.default_rng(5)
    r, batch, c_out = 8, 3, 4
    coords = random_sparse_sites(rng, (r, r, r), batch, 0.2)
    feats = rng.normal(size=(coords.shape[0], 1)).astype(np.float32)
    w = rng.normal(size=(27, 1, c_out)).astype(np.float32)
    c, f = oracle.sparse_conv_fwd((r, r, r), batch, coords, feats, (3, 3, 3), w, rho_up=1.0 / r)
    for b in range(batch):
        assert ((f[c[:, 0] == b] != 0).sum(axis=0) == r * r).all()


def test_k_from_rho_rules():
    assert oracle.k_from_rho(0.15, 784) == 117          # floor of 117.6
    assert oracle.k_from_rho(0.05, 128 ** 3) == 104857  # floor of 104857.6
    assert oracle.k_from_rho(0.1, 30) == 3              # 3.0000000000000004 -> 3
    assert oracle.k_from_rho(0.3, 10) == 3              # 2.9999999999999996 -> 3, not 2
    assert oracle.k_from_rho(0.0, 100) == 0
    assert oracle.k_from_rho(1.0, 100) == 100
    assert oracle.k_from_rho(2.0, 100) == 100


# ---------------------------------------------------------------- P6: invariants
def _entries_by_channel(c, f, extent):
    lin = np.zeros(c.shape[0], dtype=np.int64)
    for a, e in enumerate(extent):
        lin = lin * e + c[:, 1 + a]
    return lin


@pytest.mark.parametrize("mode", [oracle.ABS, oracle.SIGNED])
def test_selection_invariants(mode):
    rng = np.random.default_rng(11 + mode)
    extent, batch, c_in, c_out, ksize = (10, 9, 8), 2, 2, 3, (3, 3, 3)
    coords, feats, w = _random_case(rng, 3, extent, batch, c_in, c_out, ksize, 0.08, 0.6)
    n = int(np.prod(extent))
    full_c, full_f = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, k=n, topk_mode=mode)
    full_lin = _entries_by_channel(full_c, full_f, extent)
    for k in (1, 17, 100, n):
        c, f = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, k=k, topk_mode=mode)
        lin = _entries_by_channel(c, f, extent)
        key = c[:, 0].astype(np.int64) * n + lin
        assert (np.diff(key) > 0).all()            # rows strictly ascending
        assert (np.abs(f).sum(axis=1) > 0).all()   # no all-zero row
        for b in range(batch):
            for oc in range(c_out):
                allv = full_f[full_c[:, 0] == b, oc]
                alll = full_lin[full_c[:, 0] == b]
                nz = allv != 0
                kv = f[c[:, 0] == b, oc]
                kl = lin[c[:, 0] == b]
                knz = kv != 0
                assert knz.sum() == min(k, nz.sum())
                kept = set(kl[knz].tolist())
                assert kept <= set(alll[nz].tolist())
                sc = (lambda v: np.abs(v)) if mode == oracle.ABS else (lambda v: v)
                dropped = [(s, l) for s, l in zip(sc(allv[nz]), alll[nz]) if l not in kept]
                if dropped and knz.any():
                    min_kept = min(zip(sc(kv[knz]), -kl[knz]))
                    max_drop = max((s, -l) for s, l in dropped)
                    assert min_kept > max_drop


def test_homogeneity_and_additivity():
    rng = np.random.default_rng(21)
    extent, batch, c_in, c_out, ksize = (8, 8, 8), 1, 2, 3, (3, 3, 3)
    coords, feats, w = _random_case(rng, 3, extent, batch, c_in, c_out, ksize, 0.1, 0.7)
    k = 40
    c1, f1 = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, k=k)
    for alpha in (-4.0, 0.5):  # powers of two: bit-exact scaling
        c2, f2 = oracle.sparse_conv_fwd(extent, batch, coords, feats * np.float32(alpha), ksize, w, k=k)
        assert np.array_equal(c1, c2) and np.array_equal(f1 * np.float32(alpha), f2)
    # additivity of the raw responses (selection bypassed): layer(x + y) = layer(x) + layer(y)
    feats_b = rng.normal(size=feats.shape).astype(np.float32)
    n = int(np.prod(extent))
    def dense(fe):
        c, f = oracle.sparse_conv_fwd(extent, batch, coords, fe, ksize, w, k=n)
        d = np.zeros((n, c_out))
        lin = _entries_by_channel(c, f, extent)
        d[lin] = f
        return d
    np.testing.assert_allclose(dense(feats + feats_b), dense(feats) + dense(feats_b), rtol=1e-5, atol=1e-6)


def test_translation_equivariance_and_row_permutation():
    rng = np.random.default_rng(31)
    extent, ksize = (12, 12, 12), (3, 3, 3)
    base = random_sparse_sites(rng, (6, 6, 6), 1, 0.15)
    feats = rng.normal(size=(base.shape[0], 2)).astype(np.float32)
    w = rng.normal(size=(27, 2, 3)).astype(np.float32)
    a = base.copy(); a[:, 1:] += 2
    b = base.copy(); b[:, 1:] += 4
    ca, fa = oracle.sparse_conv_fwd(extent, 1, a, feats, ksize, w, k=25)
    cb, fb = oracle.sparse_conv_fwd(extent, 1, b, feats, ksize, w, k=25)
    ca[:, 1:] += 2
    assert np.array_equal(ca, cb) and np.array_equal(fa, fb)
    perm = rng.permutation(a.shape[0])
    cp, fp = oracle.sparse_conv_fwd(extent, 1, a[perm], feats[perm], ksize, w, k=25)
    cs, fs = oracle.sparse_conv_fwd(extent, 1, a, feats, ksize, w, k=25)
    assert np.array_equal(cp, cs)
    np.testing.assert_allclose(fp, fs, rtol=1e-6, atol=1e-7)


def test_single_tap_filter_is_a_shifted_scaled_copy():
    rng = np.random.default_rng(41)
    extent = (7, 8)
    coords = random_sparse_sites(rng, extent, 2, 0.3)
    feats = rng.normal(size=(coords.shape[0], 1)).astype(np.float32)
    for t, off in enumerate(itertools.product(range(3), range(3))):
        delta = (off[0] - 1, off[1] - 1)
        w = np.zeros((9, 1, 1), np.float32)
        w[t] = 2.0
        c, f = oracle.sparse_conv_fwd(extent, 2, coords, feats, (3, 3), w, k=10 ** 6)
        want = {}
        for r in range(coords.shape[0]):
            p = (coords[r, 1] - delta[0], coords[r, 2] - delta[1])
            if 0 <= p[0] < extent[0] and 0 <= p[1] < extent[1]:
                want[(int(coords[r, 0]), int(p[0]), int(p[1]))] = 2.0 * feats[r, 0]
        got = {tuple(int(v) for v in c[r]): f[r, 0] for r in range(c.shape[0])}
        assert got == want


# ---------------------------------------------------------------- P7: pooling / ReLU library cases
@pytest.mark.parametrize("extent", [(8, 6), (7, 5), (6, 4, 8), (5, 7, 3)])
def test_pool_and_relu_match_dense_library_ops(extent):
    rng = np.random.default_rng(sum(extent))
    batch, ch = 2, 3
    coords = random_sparse_sites(rng, extent, batch, 0.35)
    feats = rng.normal(size=(coords.shape[0], ch)).astype(np.float32)
    feats *= rng.random(feats.shape) < 0.7
    # ReLU == dense relu restricted to non-zeros
    c, f = oracle.sparse_relu(extent, coords, feats)
    want = rows_to_entries(coords, np.maximum(feats, 0))
    assert rows_to_entries(c, f) == want
    assert (f.max(axis=1) > 0).all()
    # pooling of non-negative data == dense max_pool (ceil_mode for odd extents) restricted to non-zeros
    pos = np.abs(feats)
    x = torch.zeros((batch, ch, *extent), dtype=torch.float32)
    for r in range(coords.shape[0]):
        x[(int(coords[r, 0]), slice(None)) + tuple(int(v) for v in coords[r, 1:])] = torch.from_numpy(pos[r])
    mp = torch.nn.functional.max_pool2d if len(extent) == 2 else torch.nn.functional.max_pool3d
    y = mp(x, kernel_size=2, stride=2, ceil_mode=True).numpy()
    c, f = oracle.sparse_maxpool(extent, coords, pos)
    dense = np.zeros_like(y)
    for r in range(c.shape[0]):
        dense[(int(c[r, 0]), slice(None)) + tuple(int(v) for v in c[r, 1:])] = f[r]
    assert np.array_equal(dense, y)
    key = c[:, 0].astype(np.int64) * 10 ** 6 + _entries_by_channel(c, f, [(e + 1) // 2 for e in extent])
    assert (np.diff(key) > 0).all()


def test_pool_takes_max_over_present_entries_only():
    # a cluster of negative entries pools to its largest (negative) member, not to 0
    coords = np.array([[0, 0, 0], [0, 0, 1], [0, 1, 1], [0, 2, 2]], dtype=np.int32)
    feats = np.array([[-3.0, 0.0], [-1.0, 2.0], [-2.0, 0.0], [0.0, -5.0]], dtype=np.float32)
    c, f = oracle.sparse_maxpool((4, 4), coords, feats)
    assert c.tolist() == [[0, 0, 0], [0, 1, 1]]
    assert f.tolist() == [[-1.0, 2.0], [0.0, -5.0]]


# ---------------------------------------------------------------- P8: MAC count (Eq. 1 numerator)
def test_mac_count_closed_form():
    rng = np.random.default_rng(51)
    extent, batch, c_in, c_out, ksize = (9, 9, 9), 2, 3, 4, (3, 3, 3)
    coords, feats, w = _random_case(rng, 3, extent, batch, c_in, c_out, ksize, 0.1, 0.5)
    _, _, info = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, k=5, return_info=True)
    upper = sum(int((feats[:, ic] != 0).sum()) * int((w[:, ic, :] != 0).sum()) for ic in range(c_in))
    assert 0 < info["macs"] <= upper
    # interior-only input: no update leaves the grid -> equality
    inner = coords[((coords[:, 1:] >= 1) & (coords[:, 1:] <= 7)).all(axis=1)]
    fin = feats[: inner.shape[0]]
    _, _, info = oracle.sparse_conv_fwd(extent, batch, inner, fin, ksize, w, k=5, return_info=True)
    assert info["macs"] == sum(int((fin[:, ic] != 0).sum()) * int((w[:, ic, :] != 0).sum()) for ic in range(c_in))


# ---------------------------------------------------------------- standalone ops agree with the fused call
def test_standalone_ops_compose_to_fused_layer():
    wl = make_config(1)
    L = wl.layers[0]
    n = int(np.prod(wl.extent))
    k = oracle.k_from_rho(L.rho_up, n)
    rc, rf = oracle.sparse_conv_fwd(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], resp_only=True)
    ac, af = oracle.attention_topk(wl.extent, wl.batch, rc, rf, k)
    assert ((af != 0).sum(axis=0) <= k).all()
    lc, lf = oracle.sparse_relu(wl.extent, ac, af)
    pc, pf = oracle.sparse_maxpool(wl.extent, lc, lf)
    fc, ff = oracle.sparse_conv_fwd(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0],
                                    rho_up=L.rho_up, relu=True, pool=True)
    assert np.array_equal(pc, fc) and np.array_equal(pf, ff)
    assert pc[:, 1:].max() < 14


def test_threads_do_not_change_the_result():
    wl = make_config(2, r=16, batch=3)
    L = wl.layers[0]
    a = oracle.sparse_conv_fwd(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], rho_up=L.rho_up,
                               relu=True, threads=1)
    b = oracle.sparse_conv_fwd(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], rho_up=L.rho_up,
                               relu=True, threads=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


# ---------------------------------------------------------------- sparseToDense against a library routine
@pytest.mark.parametrize("extent,batch,channels", [((7, 5), 2, 3), ((4, 6, 5), 3, 2)])
def test_sparse_to_dense_equals_library_coo_to_dense(extent, batch, channels):
    rng = np.random.default_rng(len(extent) + channels)
    coords = random_sparse_sites(rng, extent, batch, 0.3)
    feats = rng.normal(size=(coords.shape[0], channels)).astype(np.float32)
    dense = oracle.sparse_to_dense(extent, batch, coords, feats)
    assert dense.shape == (batch, channels, *extent)
    # library: a COO tensor indexed (b, site...) with a dense channel vector per entry, channel axis moved to 1
    coo = torch.sparse_coo_tensor(torch.from_numpy(coords.T.astype(np.int64)), torch.from_numpy(feats),
                                  size=(batch, *extent, channels))
    want = coo.to_dense().movedim(-1, 1).numpy()
    assert np.array_equal(dense, want)
    # value count and sum survive; everything off the rows is zero
    assert np.count_nonzero(dense) == np.count_nonzero(feats)
    assert dense[0, :, 0, 0].shape == (channels,) if len(extent) == 2 else True
