"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_1801_10585_amd as scnn
from tests.parity import ATOL, RTOL, assert_rows_well_formed, check_column, column, lin_index
from workloads import make_config, make_filter, make_paper_runtime, random_sparse_sites

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.cpu().numpy()


def gpu_conv(extent, batch, coords, feats, ksize, w, bias=None, **kw):
    c, f, n = scnn.sparse_conv_fwd(extent, batch, dev(coords), dev(feats), ksize, dev(w),
                                   None if bias is None else dev(bias), **kw)
    return host(c), host(f), n


def oracle_responses(extent, coords, feats, ksize, w, bias, b, ocs, threads=16):
    """Every response of sample b on the output channels `ocs`, before the selection: the oracle's rows (sample index
    0) and values [rows, len(ocs)]; a row is listed when any of these channels is non-zero there."""
    sel = coords[:, 0] == b
    cb = coords[sel].copy()
    cb[:, 0] = 0
    ocs = list(ocs)
    return oracle.sparse_conv_fwd(extent, 1, cb, feats[sel], ksize, np.ascontiguousarray(w[:, :, ocs]),
                                  None if bias is None else np.ascontiguousarray(bias[ocs]), resp_only=True,
                                  threads=threads)


def _close_column(got, want, where):
    """Same coordinate set, values within the layer's tolerance."""
    (gl, gv), (wl_, wv) = got, want
    assert np.array_equal(gl, wl_), f"{where}: coordinate sets differ ({len(gl)} vs {len(wl_)} entries)"
    assert np.allclose(gv, wv, rtol=RTOL, atol=ATOL), f"{where}: values differ"


def pooled_extent(extent):
    return tuple((int(e) + 1) // 2 for e in extent)


def check_conv_against_oracle(extent, batch, coords, feats, ksize, w, bias, k, rho_up, mode, columns=None, tag=""):
    """Band-rule comparison of the un-fused layer on all (or sampled) columns.  The fused ReLU / pooling variants
    are compared, column by column, with the oracle's ReLU / pooling applied to the ORACLE's own selection (nothing
    the HIP path produced is ever handed to the oracle); a column whose selection is ambiguous within the tolerance
    (entries in the band around the k-th score, or responses within 1e-6 of zero) is left out of that comparison.
    Separately, the fused variants must equal the library's standalone operators applied to its un-fused output,
    bit for bit (both sides HIP)."""
    c_out = w.shape[2]
    gc, gf, n = gpu_conv(extent, batch, coords, feats, ksize, w, bias, rho_up=rho_up, topk_mode=mode)
    assert int(n[2]) == 0, f"{tag}: status flags {int(n[2])}"
    assert_rows_well_formed(gc, gf, extent, batch)
    ext_p = pooled_extent(extent)
    fused = {}
    for relu, pool in ((True, False), (True, True), (False, True)):
        fc, ff, fn = gpu_conv(extent, batch, coords, feats, ksize, w, bias, rho_up=rho_up, topk_mode=mode, relu=relu,
                              pool=pool)
        assert int(fn[2]) == 0
        assert_rows_well_formed(fc, ff, ext_p if pool else extent, batch)
        fused[(relu, pool)] = (fc, ff)
    if columns is None:
        columns = [(b, oc) for b in range(batch) for oc in range(c_out)]
    band_total = 0
    for b in sorted({b for (b, _) in columns}):
        ocs = sorted(oc for (bb, oc) in columns if bb == b)
        # the oracle's responses of this sample, all wanted channels in one (threaded) run
        rc_all, rf_all = oracle_responses(extent, coords, feats, ksize, w, bias, b, ocs)
        lin_all = lin_index(rc_all, extent)
        for j, oc in enumerate(ocs):
            nz = rf_all[:, j] != 0
            rc, rf = np.ascontiguousarray(rc_all[nz]), np.ascontiguousarray(rf_all[nz, j:j + 1])
            all_lin, all_val = lin_all[nz], rf[:, 0]
            got_lin, got_val = column(gc, gf, extent, b, oc)
            where = f"{tag} (b={b}, oc={oc})"
            band = check_column(all_lin, all_val, got_lin, got_val, k, mode, where=where)
            band_total += band
            assert len(got_lin) <= k
            # (the k-th entry itself always lies in the band: more than one entry there makes the selection ambiguous)
            if band > 1 or (np.abs(all_val) <= ATOL).any():
                continue
            kc, kf = oracle.attention_topk(extent, 1, rc, rf, k, mode)     # the oracle's own selection
            rco, rfo = oracle.sparse_relu(extent, kc, kf)
            for (relu, pool), (fc, ff) in fused.items():
                ec, ef = (rco, rfo) if relu else (kc, kf)
                ext_o = extent
                if pool:
                    ec, ef = oracle.sparse_maxpool(extent, ec, ef)
                    ext_o = ext_p
                _close_column(column(fc, ff, ext_o, b, oc), (lin_index(ec, ext_o), ef[:, 0]),
                              f"{where} relu={relu} pool={pool}")
    # fused variants against the library's own standalone operators (no oracle involved): bit-exact
    dgc, dgf = dev(gc), dev(gf)
    rcs, rfs, _ = scnn.sparse_relu(len(extent), dgc, dgf)
    assert np.array_equal(fused[(True, False)][0], host(rcs)) and np.array_equal(fused[(True, False)][1], host(rfs)), \
        f"{tag}: fused ReLU differs from the standalone operator"
    pcs, pfs, _ = scnn.sparse_maxpool(extent, batch, rcs, rfs)
    assert np.array_equal(fused[(True, True)][0], host(pcs)) and np.array_equal(fused[(True, True)][1], host(pfs)), \
        f"{tag}: fused ReLU+pool differs from the standalone operators"
    pcs, pfs, _ = scnn.sparse_maxpool(extent, batch, dgc, dgf)
    assert np.array_equal(fused[(False, True)][0], host(pcs)) and np.array_equal(fused[(False, True)][1], host(pfs)), \
        f"{tag}: fused pool differs from the standalone operator"
    return gc, gf, band_total


def _sampled_columns(rng, batch, c_out, count):
    cols = {(0, 0), (batch - 1, c_out - 1)}
    while len(cols) < min(count, batch * c_out):
        cols.add((int(rng.integers(batch)), int(rng.integers(c_out))))
    return sorted(cols)


# ------------------------------------------------------------------ standalone operators: bit-exact
def _random_rows(rng, extent, batch, density, channels, levels=None, fill=0.7):
    coords = random_sparse_sites(rng, extent, batch, density)
    if levels:
        feats = rng.integers(-levels, levels + 1, size=(coords.shape[0], channels)).astype(np.float32) * 0.25
    else:
        feats = rng.normal(size=(coords.shape[0], channels)).astype(np.float32)
    feats *= rng.random(feats.shape) < fill
    return coords, np.ascontiguousarray(feats.astype(np.float32))


@pytest.mark.parametrize("extent,batch,channels,density", [
    ((9, 11), 1, 1, 0.5), ((16, 16), 3, 5, 0.4), ((12, 10, 9), 2, 64, 0.3), ((20, 20, 20), 4, 70, 0.12),
    ((33, 17, 5), 2, 130, 0.2), ((40, 40, 40), 2, 16, 0.1), ((48, 48, 32), 2, 40, 0.3), ((64, 64, 12), 1, 64, 0.9),
    # a thousand or more columns of at most 1024 positions (one wave per column): exactly 1024 sites, just below,
    # and just above (a workgroup per column again, as with fewer columns)
    ((28, 28), 260, 5, 0.4), ((32, 32), 16, 70, 0.6), ((10, 10, 10), 350, 3, 0.5), ((33, 32), 3, 4, 0.5),
    ((28, 28), 37, 5, 0.4),
    # more than a thousand columns of at most 4096 positions: one wave per column as well
    ((16, 16, 16), 130, 8, 0.2), ((60, 60), 260, 4, 0.3)])
@pytest.mark.parametrize("mode", [scnn.ABS, scnn.SIGNED])
def test_attention_topk_bit_exact_with_heavy_ties(extent, batch, channels, density, mode):
    rng = np.random.default_rng(abs(hash((extent, batch, channels, mode))) % 2 ** 32)
    for levels in (2, 40, None):  # few distinct values -> long runs of equal scores at the threshold
        coords, resp = _random_rows(rng, extent, batch, density, channels, levels)
        n_per = max(1, coords.shape[0] // batch)
        for k in (0, 1, n_per // 7 + 1, n_per // 2, n_per, 10 ** 9):
            say(f"attention_topk extent={extent} B={batch} C={channels} mode={mode} levels={levels} k={k}")
            gc, gf, n = scnn.attention_topk(extent, batch, dev(coords), dev(resp), k, mode)
            oc_, of_ = oracle.attention_topk(extent, batch, coords, resp, k, mode)
            assert int(n[2]) == 0
            assert np.array_equal(host(gc), oc_), (k, levels)
            assert np.array_equal(host(gf), of_), (k, levels)


@pytest.mark.parametrize("channels", [16, 40])
@pytest.mark.parametrize("mode", [scnn.ABS, scnn.SIGNED])
def test_attention_topk_is_exact_when_the_sampled_bracket_misses(channels, mode):
    """Long columns are settled from a bracket estimated on every S-th tile of 128 rows (S = ceil(tiles / 128)).
    Here exactly those tiles hold the strong responses, so the estimate is far off in every column: the selection must
    notice (result counter 3) and still return the oracle's rows bit for bit."""
    extent, batch = (64, 64, 16), 2
    rng = np.random.default_rng(77 + channels + mode)
    coords = random_sparse_sites(rng, extent, batch, 0.6)
    resp = rng.normal(size=(coords.shape[0], channels)).astype(np.float32)
    for b in range(batch):
        rows = np.nonzero(coords[:, 0] == b)[0]
        tiles = -(-len(rows) // 128)
        assert tiles > 2 * 128  # S = 3
        S = -(-tiles // 128)
        strong = (np.arange(len(rows)) // 128) % S == 0
        resp[rows[strong]] += np.float32(100.0)
    for k in (len(coords) // batch // 10, len(coords) // batch // 2):
        say(f"attention_topk bracket miss C={channels} mode={mode} k={k}")
        gc, gf, n = scnn.attention_topk(extent, batch, dev(coords), dev(resp), k, mode)
        oc_, of_ = oracle.attention_topk(extent, batch, coords, resp, k, mode)
        assert int(n[2]) == 0 and int(n[3]) == 1
        assert np.array_equal(host(gc), oc_) and np.array_equal(host(gf), of_)
    # and the usual case: the estimate holds
    resp = rng.normal(size=(coords.shape[0], channels)).astype(np.float32)
    k = len(coords) // batch // 3
    gc, gf, n = scnn.attention_topk(extent, batch, dev(coords), dev(resp), k, mode)
    oc_, of_ = oracle.attention_topk(extent, batch, coords, resp, k, mode)
    assert int(n[2]) == 0 and int(n[3]) == 0
    assert np.array_equal(host(gc), oc_) and np.array_equal(host(gf), of_)


def test_attention_topk_empty_and_single_sample_cases():
    extent, batch = (8, 8, 8), 3
    coords = np.zeros((0, 4), np.int32)
    resp = np.zeros((0, 4), np.float32)
    gc, gf, n = scnn.attention_topk(extent, batch, dev(coords), dev(resp), 5)
    assert gc.shape[0] == 0 and int(n[0]) == 0
    # only the middle sample populated
    rng = np.random.default_rng(1)
    coords, resp = _random_rows(rng, extent, 1, 0.4, 4, 3)
    coords[:, 0] = 1
    gc, gf, _ = scnn.attention_topk(extent, batch, dev(coords), dev(resp), 9)
    oc_, of_ = oracle.attention_topk(extent, batch, coords, resp, 9)
    assert np.array_equal(host(gc), oc_) and np.array_equal(host(gf), of_)


@pytest.mark.parametrize("extent,batch,channels", [((8, 6), 2, 3), ((7, 5), 1, 1), ((6, 4, 8), 2, 17), ((5, 7, 3), 3, 64),
                                                   ((31, 33, 29), 2, 40)])
def test_relu_and_maxpool_bit_exact(extent, batch, channels):
    rng = np.random.default_rng(sum(extent) + channels)
    coords, feats = _random_rows(rng, extent, batch, 0.3, channels)
    say(f"relu/maxpool extent={extent} B={batch} C={channels} rows={coords.shape[0]}")
    gc, gf, n = scnn.sparse_relu(len(extent), dev(coords), dev(feats))
    oc_, of_ = oracle.sparse_relu(extent, coords, feats)
    assert np.array_equal(host(gc), oc_) and np.array_equal(host(gf), of_)
    gc, gf, n = scnn.sparse_maxpool(extent, batch, dev(coords), dev(feats))
    oc_, of_ = oracle.sparse_maxpool(extent, coords, feats)
    assert np.array_equal(host(gc), oc_) and np.array_equal(host(gf), of_)
    # all-negative clusters keep their (negative) maximum
    neg = -np.abs(feats) - (feats == 0)
    gc, gf, n = scnn.sparse_maxpool(extent, batch, dev(coords), dev(neg.astype(np.float32)))
    oc_, of_ = oracle.sparse_maxpool(extent, coords, neg.astype(np.float32))
    assert np.array_equal(host(gc), oc_) and np.array_equal(host(gf), of_)


@pytest.mark.parametrize("extent,batch,density", [((176, 176, 176), 1, 0.001), ((64, 64, 64), 5, 0.004),
                                                  ((262, 258, 260), 1, 0.0005)])
def test_maxpool_on_large_grids(extent, batch, density):
    """Pooled bitmaps of more than 8192 words (the emit kernel still counts the words before its own by itself, up to
    32768 words) and of more than 32768 (popcount and scan launches), several samples, odd extents."""
    rng = np.random.default_rng(extent[0] + batch)
    coords, feats = _random_rows(rng, extent, batch, density, 4)
    say(f"maxpool extent={extent} B={batch} rows={coords.shape[0]}")
    gc, gf, n = scnn.sparse_maxpool(extent, batch, dev(coords), dev(feats))
    oc_, of_ = oracle.sparse_maxpool(extent, coords, feats)
    assert np.array_equal(host(gc), oc_) and np.array_equal(host(gf), of_)


def test_relu_and_pool_on_empty_input():
    c = np.zeros((0, 3), np.int32)
    f = np.zeros((0, 2), np.float32)
    gc, gf, n = scnn.sparse_relu(2, dev(c), dev(f))
    assert gc.shape[0] == 0
    gc, gf, n = scnn.sparse_maxpool((4, 4), 1, dev(c), dev(f))
    assert gc.shape[0] == 0


# ------------------------------------------------------------------ the layer on small random cases (all columns)
SMALL = [
    # extent, batch, c_in, c_out, ksize, density, filter density
    ((12, 13), 2, 1, 3, (3, 3), 0.3, 0.6),
    ((28, 28), 1, 1, 8, (3, 3), 0.2, 0.5),
    ((9, 10, 11), 2, 2, 5, (3, 3, 3), 0.15, 0.5),
    ((16, 16, 16), 3, 4, 24, (3, 3, 3), 0.1, 0.5),
    ((20, 9, 14), 1, 3, 40, (5, 1, 3), 0.1, 0.7),
    ((14, 14, 14), 2, 8, 70, (3, 3, 3), 0.08, 1.0),
    ((10, 10, 10), 1, 33, 17, (1, 1, 1), 0.3, 0.9),
    ((24, 24, 24), 2, 16, 32, (5, 5, 5), 0.03, 0.3),
]


@pytest.mark.parametrize("case", SMALL)
@pytest.mark.parametrize("mode", [scnn.ABS, scnn.SIGNED])
def test_layer_small_cases_all_columns(case, mode):
    extent, batch, c_in, c_out, ksize, density, fdens = case
    rng = np.random.default_rng(abs(hash((case, mode))) % 2 ** 32)
    coords = random_sparse_sites(rng, extent, batch, density)
    feats = rng.normal(size=(coords.shape[0], c_in)).astype(np.float32)
    feats *= rng.random(feats.shape) < 0.85
    feats = np.ascontiguousarray(feats.astype(np.float32))
    w = make_filter(rng, ksize, c_in, c_out, fdens, 0.4)
    bias = rng.normal(size=c_out).astype(np.float32) if rng.random() < 0.5 else None
    n = int(np.prod(extent))
    for rho in (0.02, 0.2, 1.0):
        k = scnn.k_from_rho(rho, n)
        say(f"layer small extent={extent} B={batch} {c_in}->{c_out} ks={ksize} mode={mode} rho={rho} k={k}")
        check_conv_against_oracle(extent, batch, coords, feats, ksize, w, bias, k, rho, mode, tag=f"small {case}")


MFMA_CASES = [
    # extent, batch, c_in, c_out, ksize, density, filter density  (shapes the matrix-core kernel accepts)
    ((14, 14, 14), 2, 32, 16, (3, 3, 3), 0.08, 1.0),
    ((20, 20, 20), 2, 32, 64, (3, 3, 3), 0.05, 1.0),
    ((16, 16, 16), 1, 64, 48, (3, 3, 3), 0.06, 0.5),
    ((18, 18, 18), 2, 32, 32, (5, 5, 5), 0.03, 0.3),
    ((40, 40), 3, 96, 32, (3, 3), 0.15, 0.8),
    ((12, 12, 12), 1, 128, 64, (1, 3, 3), 0.2, 1.0),
    # sixteen input channels: the half-chunk form of the matrix-core kernel
    ((16, 16, 16), 2, 16, 16, (3, 3, 3), 0.08, 1.0),
    ((20, 20, 20), 1, 16, 64, (3, 3, 3), 0.05, 0.6),
    ((30, 30), 2, 16, 48, (3, 3), 0.2, 1.0),
    # the channel widths of the paper's networks (appendix table: 8 / 16 / 24 / 32 / 40 / 48) and output widths that
    # are no multiple of 16: the quad matrix-core kernel with one or two quads per instruction
    ((18, 18, 18), 2, 8, 8, (3, 3, 3), 0.08, 1.0),
    ((16, 16, 16), 2, 24, 24, (3, 3, 3), 0.08, 0.7),
    ((16, 16, 16), 1, 40, 40, (3, 3, 3), 0.07, 1.0),
    ((14, 14, 14), 2, 48, 48, (3, 3, 3), 0.08, 0.5),
    ((16, 16, 16), 2, 24, 33, (3, 3, 3), 0.06, 1.0),
    ((20, 20, 20), 1, 64, 17, (3, 1, 3), 0.1, 1.0),
    ((36, 36), 3, 40, 64, (5, 5), 0.12, 0.6),
    ((150, 3, 3), 1, 32, 64, (3, 3, 3), 0.3, 1.0),
    # more than 64 output channels: the quad kernel runs once per group of 64 (a full and a partial group, partial
    # groups of at most and of more than 32 channels)
    ((16, 16, 16), 2, 32, 128, (3, 3, 3), 0.07, 1.0),
    ((16, 16, 16), 1, 24, 96, (3, 3, 3), 0.08, 0.7),
    ((14, 14, 14), 2, 64, 80, (3, 3, 3), 0.08, 1.0),
    ((30, 30), 2, 16, 100, (3, 3), 0.2, 1.0),
    # 96 and 128 input channels with output widths only the quad kernel takes (and, forced, those the pair lists take)
    ((14, 14, 14), 2, 96, 96, (3, 3, 3), 0.08, 1.0),
    ((12, 12, 12), 1, 128, 40, (3, 3, 3), 0.1, 0.6),
    ((24, 24), 2, 128, 128, (3, 3), 0.2, 1.0),
    # eight input channels with many output channels, 24 with few
    ((20, 20, 20), 2, 8, 64, (3, 3, 3), 0.06, 1.0),
    ((18, 18, 18), 1, 24, 16, (3, 3, 3), 0.08, 0.8),
]


@pytest.mark.parametrize("case", MFMA_CASES)
@pytest.mark.parametrize("path", [0, 1, 2, 3])
def test_layer_wide_channels_both_kernels(case, path):
    extent, batch, c_in, c_out, ksize, density, fdens = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 32)
    coords = random_sparse_sites(rng, extent, batch, density)
    feats = rng.random(size=(coords.shape[0], c_in)).astype(np.float32)
    feats *= rng.random(feats.shape) < 0.9
    feats = np.ascontiguousarray(feats.astype(np.float32))
    w = make_filter(rng, ksize, c_in, c_out, fdens, 0.2)
    bias = rng.normal(size=c_out).astype(np.float32) if c_out in (32, 96) else None
    n = int(np.prod(extent))
    scnn.set_conv_path(path)
    try:
        for mode, rho in ((scnn.ABS, 0.03), (scnn.SIGNED, 0.1), (scnn.ABS, 1.0)):
            k = scnn.k_from_rho(rho, n)
            say(f"layer wide extent={extent} B={batch} {c_in}->{c_out} ks={ksize} path={path} mode={mode} rho={rho}")
            check_conv_against_oracle(extent, batch, coords, feats, ksize, w, bias, k, rho, mode,
                                      tag=f"wide {case} path={path}")
    finally:
        scnn.set_conv_path(0)


def test_matrix_core_kernels_are_exact_on_integer_data_and_repeatable():
    """Small integers: every product and every partial sum is exact, so each kernel family must give the oracle's
    values bit for bit; and two runs of the same call must give the same bits on every family whose additions
    have a fixed order (all but the pair-list kernel)."""
    rng = np.random.default_rng(123)
    for (extent, batch, c_in, c_out, ksize) in (((22, 22, 22), 2, 32, 64, (3, 3, 3)), ((20, 20, 20), 2, 64, 32, (3, 3, 3)),
                                                ((20, 20, 20), 1, 24, 24, (3, 3, 3)), ((18, 18, 18), 2, 32, 100, (3, 3, 3))):
        coords = random_sparse_sites(rng, extent, batch, 0.08)
        feats = rng.integers(-3, 4, size=(coords.shape[0], c_in)).astype(np.float32)
        w = rng.integers(-2, 3, size=(int(np.prod(ksize)), c_in, c_out)).astype(np.float32)
        oc_, of_ = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, rho_up=1.0, threads=16)
        for path in (1, 2, 3):
            scnn.set_conv_path(path)
            try:
                gc, gf, _ = gpu_conv(extent, batch, coords, feats, ksize, w, rho_up=1.0)
                kernel = scnn.last_conv_kernel()
            finally:
                scnn.set_conv_path(0)
            say(f"integer data {c_in}->{c_out} path={path}: {kernel}, rows={gc.shape[0]}")
            assert np.array_equal(gc, oc_) and np.array_equal(gf, of_), f"path {path} ({kernel})"
            assert kernel == ("k_conv_valu" if path == 1 else "k_conv_quad") or path == 3
    # continuous data on the shape of the r = 128 configuration: the same bits on every run, selection included
    wl = make_config(4, r=40, batch=2)
    L = wl.layers[0]
    scnn.set_conv_path(2)
    try:
        runs = [gpu_conv(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], rho_up=L.rho_up, relu=True)
                for _ in range(3)]
    finally:
        scnn.set_conv_path(0)
    assert scnn.last_conv_kernel() == "k_conv_quad"
    for r in runs[1:]:
        assert np.array_equal(runs[0][0], r[0]) and np.array_equal(runs[0][1], r[1]), "runs differ"


def test_matrix_core_kernel_keeps_small_responses_accurate():
    """Shell workload at the r=128 configuration's channel widths with the selection bypassed (rho_up = 1):
    every response, however small against the products it is summed from, must meet the value tolerance."""
    wl = make_config(4, r=48, batch=2)
    L = wl.layers[0]
    rng = np.random.default_rng(44)
    n = 48 ** 3
    say(f"cfg4@48 bypass rows={wl.coords.shape[0]}")
    check_conv_against_oracle(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], None, n, 1.0, scnn.ABS,
                              columns=_sampled_columns(rng, wl.batch, L.c_out, 16), tag="cfg4@48 bypass")


@pytest.mark.parametrize("extent, batch, density", [((40, 40, 40), 4, 0.08), ((44, 44, 44), 4, 0.08)])
def test_matrix_core_kernel_with_a_partial_last_round_of_units(extent, batch, density):
    """Layers a little larger than one round of the quad kernel's wave slots (one wave takes 64 candidate sites at a
    time, about 3000 waves run at once on 256 compute units): the sites left for the last, partial round are dealt
    out in quarters of 16 (about 230 000 candidate sites) or not split at all (about 300 000).  Every column is
    compared; random sites, so that nearly every site of the grid is a candidate."""
    rng = np.random.default_rng(4044 + extent[0])
    coords = random_sparse_sites(rng, extent, batch, density)
    feats = rng.normal(size=(coords.shape[0], 32)).astype(np.float32)
    w = make_filter(rng, (3, 3, 3), 32, 64, 1.0, 0.2)
    n = int(np.prod(extent))
    k = scnn.k_from_rho(0.2, n)
    say(f"partial last round extent={extent} B={batch} rows={coords.shape[0]}")
    check_conv_against_oracle(extent, batch, coords, feats, (3, 3, 3), w, None, k, 0.2, scnn.ABS,
                              tag=f"partial round {extent}")


def test_layer_exact_ties_integer_data():
    """Dyadic inputs and weights: fp32 sums are exact on both sides, so the outputs must be bit-identical,
    including the choice among equal scores at the threshold (lower lin wins)."""
    rng = np.random.default_rng(99)
    extent, batch, c_in, c_out, ksize = (18, 18, 18), 2, 2, 6, (3, 3, 3)
    coords = random_sparse_sites(rng, extent, batch, 0.12)
    feats = (rng.integers(1, 3, size=(coords.shape[0], c_in)) * 0.5).astype(np.float32)
    w = (rng.integers(-2, 3, size=(27, c_in, c_out)) * 0.25).astype(np.float32)
    n = int(np.prod(extent))
    for mode in (scnn.ABS, scnn.SIGNED):
        for rho in (0.01, 0.05, 0.2):
            k = scnn.k_from_rho(rho, n)
            say(f"layer ties mode={mode} rho={rho} k={k}")
            for relu, pool in ((False, False), (True, False), (True, True)):
                gc, gf, _ = gpu_conv(extent, batch, coords, feats, ksize, w, rho_up=rho, topk_mode=mode, relu=relu,
                                     pool=pool)
                oc_, of_ = oracle.sparse_conv_fwd(extent, batch, coords, feats, ksize, w, k=k, topk_mode=mode,
                                                  relu=relu, pool=pool)
                assert np.array_equal(gc, oc_) and np.array_equal(gf, of_), (mode, rho, relu, pool)


# ------------------------------------------------------------------ the five configurations
def test_config1_strokes_2d():
    wl = make_config(1)
    L = wl.layers[0]
    k = scnn.k_from_rho(L.rho_up, 28 * 28)
    say(f"cfg1 rows={wl.coords.shape[0]} k={k}")
    check_conv_against_oracle(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], None, k, L.rho_up,
                              scnn.ABS, tag="cfg1")
    gc, gf, _ = gpu_conv(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], rho_up=L.rho_up, relu=True,
                         pool=True)
    assert gc[:, 1:].max() < 14


def test_config2_shells_unit_values_with_ties():
    wl = make_config(2)
    L = wl.layers[0]
    k = scnn.k_from_rho(L.rho_up, 32 ** 3)
    say(f"cfg2 rows={wl.coords.shape[0]} k={k}")
    _, _, band = check_conv_against_oracle(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], None, k,
                                           L.rho_up, scnn.ABS, tag="cfg2")
    say(f"cfg2 band entries: {band}")


def test_config3_two_layers_full_size():
    wl = make_config(3)
    L1, L2 = wl.layers
    rng = np.random.default_rng(3)
    k1 = scnn.k_from_rho(L1.rho_up, 64 ** 3)
    say(f"cfg3 layer 1 rows={wl.coords.shape[0]} k={k1}")
    check_conv_against_oracle(wl.extent, wl.batch, wl.coords, wl.feats, L1.ksize, wl.filters[0], None, k1, L1.rho_up,
                              scnn.ABS, tag="cfg3-L1")
    # layer 2 takes the ORACLE's layer-1 output (conv + attention + ReLU + pool) as the input of both sides
    c1, f1 = oracle.sparse_conv_fwd(wl.extent, wl.batch, wl.coords, wl.feats, L1.ksize, wl.filters[0], k=k1,
                                    relu=True, pool=True, threads=16)
    ext2 = (32, 32, 32)
    k2 = scnn.k_from_rho(L2.rho_up, 32 ** 3)
    say(f"cfg3 layer 2 rows={c1.shape[0]} k={k2}")
    check_conv_against_oracle(ext2, wl.batch, c1, f1, L2.ksize, wl.filters[1], None, k2, L2.rho_up, scnn.ABS,
                              tag="cfg3-L2")
    # the library's own two-layer chain: well-formed, within the density bound, and close to the oracle's chain
    g1c, g1f, _ = gpu_conv(wl.extent, wl.batch, wl.coords, wl.feats, L1.ksize, wl.filters[0], rho_up=L1.rho_up,
                           relu=True, pool=True)
    g2c, g2f, n2 = scnn.sparse_conv_fwd(ext2, wl.batch, dev(g1c), dev(g1f), L2.ksize, dev(wl.filters[1]),
                                        rho_up=L2.rho_up, relu=True)
    g2c, g2f = host(g2c), host(g2f)
    assert int(n2[2]) == 0
    assert_rows_well_formed(g2c, g2f, ext2, wl.batch)
    for b in range(wl.batch):
        assert ((g2f[g2c[:, 0] == b] != 0).sum(axis=0) <= k2).all()
    assert abs(g1c.shape[0] - c1.shape[0]) <= 0.001 * c1.shape[0]


def test_config4_r128_dense_filter_full_size_every_column():
    wl = make_config(4)
    L = wl.layers[0]
    k = scnn.k_from_rho(L.rho_up, 128 ** 3)
    say(f"cfg4 rows={wl.coords.shape[0]} k={k}")
    gc, gf, band = check_conv_against_oracle(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], None, k,
                                             L.rho_up, scnn.ABS, tag="cfg4")
    say(f"cfg4 out rows={gc.shape[0]} band entries={band}")
    for b in range(wl.batch):
        assert ((gf[gc[:, 0] == b] != 0).sum(axis=0) <= k).all()


_CFG5 = {}


def _cfg5_oracle_responses():
    """The oracle's responses of cfg 5 on all 64 channels, computed once for the three rho_up values."""
    if not _CFG5:
        wl = make_config(5)
        L = wl.layers[0]
        say(f"cfg5 oracle: rows={wl.coords.shape[0]} (threaded, all {L.c_out} channels)")
        rc, rf = oracle_responses(wl.extent, wl.coords, wl.feats, L.ksize, wl.filters[0], None, 0, range(L.c_out))
        _CFG5.update(wl=wl, lin=lin_index(rc, wl.extent), resp=rf)
    return _CFG5["wl"], _CFG5["lin"], _CFG5["resp"]


@pytest.mark.parametrize("rho", [0.02, 0.05, 0.10])
def test_config5_r256_5x5x5_full_size_every_column(rho):
    wl, all_lin, all_resp = _cfg5_oracle_responses()
    L = wl.layers[0]
    k = scnn.k_from_rho(rho, 256 ** 3)
    say(f"cfg5 rows={wl.coords.shape[0]} rho={rho} k={k}")
    gc, gf, n = gpu_conv(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], rho_up=rho)
    assert int(n[2]) == 0
    assert_rows_well_formed(gc, gf, wl.extent, wl.batch)
    assert ((gf != 0).sum(axis=0) <= k).all()
    got_lin_all = lin_index(gc, wl.extent)
    band_total = 0
    for oc in range(L.c_out):
        nz = all_resp[:, oc] != 0
        gnz = gf[:, oc] != 0
        band_total += check_column(all_lin[nz], all_resp[nz, oc], got_lin_all[gnz], gf[gnz, oc], k, scnn.ABS,
                                   where=f"cfg5 rho={rho} oc={oc}")
    say(f"cfg5 rho={rho} out rows={gc.shape[0]} band entries={band_total}")


# ------------------------------------------------------------------ the paper's runtime experiment (Sec. 4.1)
@pytest.mark.parametrize("r", [16, 32, 64, 128, 256])
@pytest.mark.parametrize("rho_f", [0.1, 1.0])
def test_paper_runtime_workload_random_sites(r, rho_f):
    """Uniformly random sites at density 1/r, one input and eight output channels, rho_up = 1/r, batch 1."""
    wl = make_paper_runtime(r, rho_f)
    L = wl.layers[0]
    k = scnn.k_from_rho(L.rho_up, r ** 3)
    assert k == r * r
    say(f"paper runtime r={r} rho_f={rho_f} rows={wl.coords.shape[0]} k={k}")
    cols = None if r <= 64 else [(0, oc) for oc in (0, 3, 7)]
    for mode in (scnn.ABS, scnn.SIGNED):
        gc, gf, band = check_conv_against_oracle(wl.extent, 1, wl.coords, wl.feats, L.ksize, wl.filters[0], None, k,
                                                 L.rho_up, mode, columns=cols, tag=f"{wl.name} mode={mode}")
        assert ((gf != 0).sum(axis=0) <= k).all()
        say(f"  mode={mode} out rows={gc.shape[0]} density={gc.shape[0] / r ** 3:.4f} band={band}")


# ------------------------------------------------------------------ edge cases and error reporting
def test_empty_input_and_zero_k():
    extent = (8, 8, 8)
    w = np.ones((27, 2, 3), np.float32)
    gc, gf, n = gpu_conv(extent, 2, np.zeros((0, 4), np.int32), np.zeros((0, 2), np.float32), (3, 3, 3), w, rho_up=0.5)
    assert gc.shape[0] == 0 and int(n[0]) == 0 and int(n[2]) == 0
    rng = np.random.default_rng(0)
    coords = random_sparse_sites(rng, extent, 2, 0.2)
    feats = rng.normal(size=(coords.shape[0], 2)).astype(np.float32)
    gc, gf, n = gpu_conv(extent, 2, coords, feats, (3, 3, 3), w, rho_up=0.0)
    assert gc.shape[0] == 0 and int(n[1]) > 0
    # all-zero filter: no candidate sites at all
    gc, gf, n = gpu_conv(extent, 2, coords, feats, (3, 3, 3), np.zeros_like(w), rho_up=0.5)
    assert gc.shape[0] == 0 and int(n[1]) == 0


@pytest.mark.parametrize("extent", [(64, 64, 136), (128, 128, 130)])
def test_candidate_overflow_on_large_bitmaps(extent):
    """Bitmaps of more than 8192 words (and of more than 32768): the candidate list is placed from per-chunk counts;
    a capacity below the candidate count is flagged and leaves an empty output, the exact capacity works."""
    rng = np.random.default_rng(extent[2])
    coords = random_sparse_sites(rng, extent, 1, 0.002)
    feats = rng.normal(size=(coords.shape[0], 2)).astype(np.float32)
    w = rng.normal(size=(27, 2, 3)).astype(np.float32)
    full_c, full_f, n = gpu_conv(extent, 1, coords, feats, (3, 3, 3), w, rho_up=1.0)
    n_cand = int(n[1])
    assert n_cand > 0 and int(n[0]) > 0
    c, f, nn = scnn.sparse_conv_fwd(extent, 1, dev(coords), dev(feats), (3, 3, 3), dev(w), rho_up=1.0,
                                    cand_capacity=n_cand - 1, sync=False)
    nn = nn.cpu()
    assert int(nn[2]) & scnn.FLAG_CAND_OVERFLOW and int(nn[0]) == 0 and int(nn[1]) == n_cand
    c, f, nn = gpu_conv(extent, 1, coords, feats, (3, 3, 3), w, rho_up=1.0, cand_capacity=n_cand)
    assert np.array_equal(c, full_c) and np.array_equal(f, full_f)


def test_capacity_flags_and_validation():
    extent = (10, 10, 10)
    rng = np.random.default_rng(2)
    coords = random_sparse_sites(rng, extent, 1, 0.2)
    feats = rng.normal(size=(coords.shape[0], 2)).astype(np.float32)
    w = rng.normal(size=(27, 2, 3)).astype(np.float32)
    full_c, full_f, n = gpu_conv(extent, 1, coords, feats, (3, 3, 3), w, rho_up=1.0)
    rows, n_cand = int(n[0]), int(n[1])
    # output truncated: true count still reported, prefix intact, flag set
    c, f, nn = scnn.sparse_conv_fwd(extent, 1, dev(coords), dev(feats), (3, 3, 3), dev(w), rho_up=1.0,
                                    out_capacity=rows // 2, sync=False)
    nn = nn.cpu()
    assert int(nn[0]) == rows and int(nn[2]) & scnn.FLAG_OUT_OVERFLOW
    assert np.array_equal(host(c)[: rows // 2], full_c[: rows // 2])
    assert np.array_equal(host(f)[: rows // 2], full_f[: rows // 2])
    # candidate capacity too small: flagged, empty output
    c, f, nn = scnn.sparse_conv_fwd(extent, 1, dev(coords), dev(feats), (3, 3, 3), dev(w), rho_up=1.0,
                                    cand_capacity=n_cand // 2, sync=False)
    nn = nn.cpu()
    assert int(nn[2]) & scnn.FLAG_CAND_OVERFLOW and int(nn[0]) == 0 and int(nn[1]) == n_cand
    # exactly enough capacity works
    c, f, nn = gpu_conv(extent, 1, coords, feats, (3, 3, 3), w, rho_up=1.0, cand_capacity=n_cand)
    assert np.array_equal(c, full_c) and np.array_equal(f, full_f)
    # validation entry point
    scnn.validate_rows(extent, 1, dev(coords))
    bad = coords[::-1].copy()
    with pytest.raises(scnn.ScnnError) as e:
        scnn.validate_rows(extent, 1, dev(bad))
    assert e.value.code == -4
    oob = coords.copy()
    oob[3, 2] = 10
    with pytest.raises(scnn.ScnnError) as e:
        scnn.validate_rows(extent, 1, dev(oob))
    assert e.value.code == -1
    # an out-of-grid row is skipped and reported, never dereferenced
    c, f, nn = scnn.sparse_conv_fwd(extent, 1, dev(oob), dev(feats), (3, 3, 3), dev(w), rho_up=1.0, sync=False)
    assert int(nn.cpu()[2]) & scnn.FLAG_BAD_COORD


def test_runs_on_a_side_stream_and_is_repeatable():
    wl = make_config(2, r=24, batch=3)
    L = wl.layers[0]
    a = gpu_conv(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], rho_up=L.rho_up, relu=True)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        b = gpu_conv(wl.extent, wl.batch, wl.coords, wl.feats, L.ksize, wl.filters[0], rho_up=L.rho_up, relu=True)
    s.synchronize()
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
