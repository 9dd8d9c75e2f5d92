"""GPU parity over a seeded sweep of small layer shapes, chosen to cross the points at which the library changes
kernels: channel counts around the 16- and 32-channel blocks of the vector convolution, odd and even C_in (vector
width of the gathers), row counts around the 32- and 128-row work items, filters with more than 32 taps, grids on both
sides of the single-workgroup selection (32768 sites per sample), item counts on both sides of the small / latency /
streaming forms of the vector convolution, a sample without rows.  Every case goes through the same band-rule
comparison with the oracle as the fixed cases (un-fused layer on sampled columns, fused variants, standalone
operators)."""
import numpy as np
import pytest

import paper_1801_10585_amd as scnn
from tests.test_gpu_parity import _sampled_columns, check_conv_against_oracle, say
from workloads import make_filter, random_sparse_sites

pytestmark = pytest.mark.gpu

KSIZES_3D = [(3, 3, 3), (1, 3, 3), (3, 1, 1), (5, 5, 5), (3, 5, 1), (1, 1, 1)]
KSIZES_2D = [(3, 3), (5, 3), (7, 7), (1, 5)]
C_IN = [1, 2, 3, 4, 6, 8, 12, 16, 24]
C_OUT = [1, 3, 8, 15, 16, 17, 24, 31, 32, 33, 40]


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    if seed % 4 == 3:
        extent = tuple(int(x) for x in rng.integers(6, 40, size=2))
        ksize = KSIZES_2D[int(rng.integers(len(KSIZES_2D)))]
    else:
        extent = tuple(int(x) for x in rng.integers(4, 18, size=3))
        ksize = KSIZES_3D[int(rng.integers(len(KSIZES_3D)))]
    batch = int(rng.integers(1, 4))
    c_in = C_IN[int(rng.integers(len(C_IN)))]
    c_out = C_OUT[int(rng.integers(len(C_OUT)))]
    density = float(rng.choice([0.03, 0.1, 0.3, 0.6]))
    fdens = float(rng.choice([0.3, 0.7, 1.0]))
    return rng, extent, batch, c_in, c_out, ksize, density, fdens


@pytest.mark.parametrize("seed", range(36))
def test_random_small_layers(seed):
    rng, extent, batch, c_in, c_out, ksize, density, fdens = _case(seed)
    coords = random_sparse_sites(rng, extent, batch, density)
    if batch > 1 and seed % 5 == 0:  # one sample without rows
        coords = np.ascontiguousarray(coords[coords[:, 0] != batch // 2])
    feats = rng.normal(size=(coords.shape[0], c_in)).astype(np.float32)
    feats *= rng.random(feats.shape) < 0.9
    feats = np.ascontiguousarray(feats.astype(np.float32))
    w = make_filter(rng, ksize, c_in, c_out, fdens, 0.4)
    bias = rng.normal(size=c_out).astype(np.float32) if seed % 3 == 0 else None
    n = int(np.prod(extent))
    mode = scnn.ABS if seed % 2 == 0 else scnn.SIGNED
    for rho in (0.05, 0.4):
        k = scnn.k_from_rho(rho, n)
        say(f"sweep seed={seed} extent={extent} B={batch} {c_in}->{c_out} ksize={ksize} rows={coords.shape[0]} "
            f"fdens={fdens} rho={rho} k={k} mode={mode}")
        check_conv_against_oracle(extent, batch, coords, feats, ksize, w, bias, k, rho, mode,
                                  columns=_sampled_columns(rng, batch, c_out, 5), tag=f"sweep {seed} rho={rho}")


# item counts (tiles x 32-channel blocks) on both sides of the vector convolution's three forms, and grids on both
# sides of the single-workgroup selection
REGIMES = [
    # extent, batch, c_in, c_out, density
    ((30, 30, 30), 1, 4, 8, 0.04),     # 27000 sites: about 200 tiles -> 32-row items
    ((36, 36, 36), 1, 8, 16, 0.03),    # 46656 sites: about 360 tiles -> 128-row items, generic selection
    ((32, 32, 32), 2, 2, 40, 0.05),    # up to 514 tiles x 2 channel blocks: the device-side count picks the form
    ((48, 48, 48), 2, 6, 12, 0.08),    # most of 221184 sites are candidates: over 1024 tiles -> streaming form
    ((48, 48, 48), 2, 8, 8, 0.08),     # the same with at most 8 output channels: 8 accumulators per thread
    ((64, 64, 128), 1, 2, 4, 0.003),   # exactly 8192 bitmap words: the emit kernels still find their own offsets
    ((64, 64, 136), 1, 2, 4, 0.003),   # more than 8192 words: candidate list from per-chunk counts (16-word chunks)
    ((100, 90, 61), 2, 2, 4, 0.002),   # ... 8579 words per sample: a sample starts inside a chunk
    ((150, 130, 111), 2, 2, 4, 0.0005),  # ... over 32768 words: 256-word chunks, 33821 words per sample
    ((33, 32, 32), 2, 4, 8, 0.05),     # just over 32768 sites per sample: three-launch selection
    ((176, 176, 176), 1, 2, 4, 0.0004),  # pooled grid 88^3: more than 8192 words in the pooling's bitmap
    ((9, 8, 7), 37, 4, 24, 0.2),       # many small samples, some of them empty
    ((28, 28), 300, 1, 8, 0.19),       # a batch of small images: per-sample ranges by a scan over the samples
    ((28, 28), 1100, 1, 3, 0.1),       # ... more than 8192 bitmap words of 13-word samples (a sample starts inside a chunk)
    ((28, 28), 2600, 1, 2, 0.05),      # ... more than 32768 words, still 16-word chunks because the samples are short
]


@pytest.mark.parametrize("case", REGIMES)
def test_vector_convolution_regimes(case):
    extent, batch, c_in, c_out, density = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 32)
    coords = random_sparse_sites(rng, extent, batch, density)
    if batch > 8:  # every fifth sample without rows
        coords = np.ascontiguousarray(coords[coords[:, 0] % 5 != 2])
    feats = np.ascontiguousarray(rng.normal(size=(coords.shape[0], c_in)).astype(np.float32))
    ksize = (3,) * len(extent)
    w = make_filter(rng, ksize, c_in, c_out, 0.8, 0.3)
    n = int(np.prod(extent))
    k = scnn.k_from_rho(0.1, n)
    say(f"regime extent={extent} B={batch} {c_in}->{c_out} rows={coords.shape[0]} k={k}")
    check_conv_against_oracle(extent, batch, coords, feats, ksize, w, None, k, 0.1, scnn.ABS,
                              columns=_sampled_columns(rng, batch, c_out, 4), tag=f"regime {extent}")


# Long columns (more than 32768 sites per sample): the selection brackets the k-th key from every S-th tile of 128
# rows, S = ceil(tiles / 128); the compaction streams for 17..64 channels and looks back otherwise; the settling pass
# holds up to 20480 bracket entries of a column in registers.  Row counts on both sides of S = 1 / 2, channel counts
# on both sides of 17, 33 and 64, and few distinct values, which put far more than 20480 equal scores into the bracket.
SELECTION_REGIMES = [
    # rows per sample, channels, levels (None: normal values)
    (128 * 128, 40, None), (128 * 128 + 1, 40, None), (129 * 128, 33, 40), (300 * 128 + 77, 32, None),
    (300 * 128 + 77, 64, 2), (300 * 128 + 77, 65, None), (40000, 48, 2), (40000, 8, 2),
    (129 * 128, 16, None), (40000, 17, 2), (129 * 128 + 5, 24, 3),
    # more than 256 columns: the settling pass with the small caches (two workgroups per compute unit), on brackets
    # that fit them and, with few distinct values, on brackets that do not
    (129 * 128, 150, None), (40000, 140, 2),
]


@pytest.mark.parametrize("case", SELECTION_REGIMES)
@pytest.mark.parametrize("mode", [scnn.ABS, scnn.SIGNED])
def test_selection_regimes_bit_exact(case, mode):
    import oracle
    from tests.test_gpu_parity import dev, host
    rows_per_sample, channels, levels = case
    extent, batch = (64, 64, 16), 2
    rng = np.random.default_rng(abs(hash((case, mode))) % 2 ** 32)
    full = random_sparse_sites(rng, extent, batch, 0.8)
    keep = np.concatenate([np.nonzero(full[:, 0] == b)[0][:rows_per_sample] for b in range(batch)])
    coords = np.ascontiguousarray(full[keep])
    assert (np.bincount(coords[:, 0], minlength=batch) == rows_per_sample).all()
    if levels:
        resp = rng.integers(-levels, levels + 1, size=(coords.shape[0], channels)).astype(np.float32) * 0.25
    else:
        resp = rng.normal(size=(coords.shape[0], channels)).astype(np.float32)
    resp = np.ascontiguousarray(resp * (rng.random(resp.shape) < 0.9), dtype=np.float32)
    for k in (1, rows_per_sample // 20, rows_per_sample // 2, rows_per_sample):
        say(f"selection regime rows={rows_per_sample} C={channels} levels={levels} mode={mode} k={k}")
        gc, gf, n = scnn.attention_topk(extent, batch, dev(coords), dev(resp), k, mode)
        oc_, of_ = oracle.attention_topk(extent, batch, coords, resp, k, mode)
        assert int(n[2]) == 0
        assert np.array_equal(host(gc), oc_), (case, k)
        assert np.array_equal(host(gf), of_), (case, k)


@pytest.mark.parametrize("channels,levels", [(3, None), (33, None), (20, 3)])
def test_selection_very_long_columns(channels, levels):
    """Columns of about 700 000 entries: the bracket holds more entries than the settling pass caches (32768), so
    it is read twice -- leading digit, then the k-th key's bin into LDS -- or, with few distinct values (a bin longer
    than LDS), once per digit.  With and without row marks (33 / 3 and 20 channels)."""
    import oracle
    from tests.test_gpu_parity import dev, host
    extent, batch = (128, 128, 64), 1
    rng = np.random.default_rng(channels)
    coords = random_sparse_sites(rng, extent, batch, 0.7)
    if levels:
        resp = rng.integers(-levels, levels + 1, size=(coords.shape[0], channels)).astype(np.float32) * 0.5
    else:
        resp = rng.normal(size=(coords.shape[0], channels)).astype(np.float32)
    resp = np.ascontiguousarray(resp * (rng.random(resp.shape) < 0.9), dtype=np.float32)
    rows = coords.shape[0]
    for mode, k in ((scnn.ABS, rows // 20), (scnn.SIGNED, rows // 3), (scnn.ABS, rows // 2)):
        say(f"selection very long rows={rows} C={channels} levels={levels} mode={mode} k={k}")
        gc, gf, n = scnn.attention_topk(extent, batch, dev(coords), dev(resp), k, mode)
        oc_, of_ = oracle.attention_topk(extent, batch, coords, resp, k, mode)
        assert int(n[2]) == 0
        assert np.array_equal(host(gc), oc_), (channels, k)
        assert np.array_equal(host(gf), of_), (channels, k)


@pytest.mark.parametrize("seed", range(12))
def test_selection_random_long_columns(seed):
    """Samples of very different sizes in one batch (one of them may be empty or tiny), channels that are all zero
    or hold a single entry, k above and below the samples' entry counts: attention_topk bit for bit."""
    import oracle
    from tests.test_gpu_parity import dev, host
    rng = np.random.default_rng(5000 + seed)
    extent = [(64, 64, 16), (40, 40, 40), (256, 300)][seed % 3]
    batch = int(rng.integers(2, 5))
    channels = int(rng.choice([1, 5, 16, 33, 40, 64, 70]))
    full = random_sparse_sites(rng, extent, batch, 0.7)
    keep = []
    for b in range(batch):
        rows = np.nonzero(full[:, 0] == b)[0]
        frac = float(rng.choice([0.0, 0.001, 0.3, 1.0]))
        keep.append(rows[: int(len(rows) * frac)])
    coords = np.ascontiguousarray(full[np.concatenate(keep)])
    levels = [None, 3, 1][seed % 3]
    if levels:
        resp = rng.integers(-levels, levels + 1, size=(coords.shape[0], channels)).astype(np.float32)
    else:
        resp = rng.standard_cauchy(size=(coords.shape[0], channels)).astype(np.float32)  # heavy tails: wide key range
    resp *= rng.random(resp.shape) < float(rng.choice([0.05, 0.5, 1.0]))
    if channels > 2:
        resp[:, 0] = 0.0                      # a channel without entries
        resp[:, 1] = 0.0
        if len(resp):
            resp[len(resp) // 2, 1] = 2.5     # a channel with one entry
    resp = np.ascontiguousarray(resp, dtype=np.float32)
    n_max = int(np.bincount(coords[:, 0], minlength=batch).max()) if len(coords) else 0
    mode = scnn.ABS if seed % 2 == 0 else scnn.SIGNED
    for k in sorted({0, 1, max(1, n_max // 50), max(1, n_max // 3), n_max, n_max + 5}):
        say(f"selection random seed={seed} extent={extent} B={batch} C={channels} rows={len(coords)} k={k} mode={mode}")
        gc, gf, n = scnn.attention_topk(extent, batch, dev(coords), dev(resp), k, mode)
        oc_, of_ = oracle.attention_topk(extent, batch, coords, resp, k, mode)
        assert int(n[2]) == 0
        assert np.array_equal(host(gc), oc_), (seed, k)
        assert np.array_equal(host(gf), of_), (seed, k)


# Whole layers whose columns are long and whose channel counts take the row-marking selection with the streaming
# compaction (17..64 output channels), with the quad, the pair-list and the vector convolution in front of it.
WIDE_LONG = [
    ((40, 40, 40), 2, 32, 40, 0.08), ((36, 36, 36), 1, 16, 64, 0.10), ((48, 40, 36), 2, 8, 33, 0.06),
    ((40, 40, 40), 1, 64, 48, 0.05), ((40, 40, 40), 2, 8, 17, 0.08), ((36, 40, 44), 1, 24, 24, 0.10),
    ((64, 64, 40), 1, 8, 32, 0.08),  # (more than 1024 tiles: the library picks the quad kernel for 8 -> 32 itself)
]


@pytest.mark.parametrize("case", WIDE_LONG)
def test_wide_layers_with_long_columns(case):
    extent, batch, c_in, c_out, density = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 32)
    coords = random_sparse_sites(rng, extent, batch, density)
    feats = np.ascontiguousarray(rng.normal(size=(coords.shape[0], c_in)).astype(np.float32))
    w = make_filter(rng, (3, 3, 3), c_in, c_out, 0.9, 0.3)
    bias = rng.normal(size=c_out).astype(np.float32) * 0.1
    n = int(np.prod(extent))
    for rho in (0.02, 0.3):
        k = scnn.k_from_rho(rho, n)
        say(f"wide/long extent={extent} B={batch} {c_in}->{c_out} rows={coords.shape[0]} rho={rho} k={k}")
        check_conv_against_oracle(extent, batch, coords, feats, (3, 3, 3), w, bias, k, rho, scnn.ABS,
                                  columns=_sampled_columns(rng, batch, c_out, 6), tag=f"wide/long {extent} rho={rho}")


@pytest.mark.parametrize("seed", range(12))
def test_matrix_core_and_vector_kernels_agree_over_layer_sizes(seed):
    """Layer sizes from a hundred to several thousand groups of 64 candidate sites, i.e. on both sides of every point
    at which the quad kernel changes how it deals its work out (wave tiles in quarters, in halves, whole; an XCD's
    tiles in one span or in chunks; one or two groups of 64 output channels).  The oracle needs minutes for the
    larger ones, so this sweep compares the library's two kernel families with each other instead: the vector
    kernels (fp64 sums; compared with the oracle by every other test here) and the quad kernel, selection bypassed
    (rho_up = 1), every response within the value tolerance and the same sites.  The oracle comparisons of the quad
    kernel at full size are the configuration tests."""
    import torch
    from tests.parity import ATOL, RTOL
    rng = np.random.default_rng(7000 + seed)
    c_in, c_out = [(32, 64), (16, 24), (32, 96), (8, 32), (24, 24), (32, 32)][seed % 6]
    e = int(rng.integers(20, 72))
    extent = (e, e, int(rng.integers(8, e + 1)))
    batch = int(rng.integers(1, 6))
    coords = random_sparse_sites(rng, extent, batch, float(rng.choice([0.02, 0.05, 0.1, 0.3])))
    feats = rng.normal(size=(coords.shape[0], c_in)).astype(np.float32)
    w = (rng.normal(size=(27, c_in, c_out)) * 0.04).astype(np.float32)
    dev = torch.device("cuda:0")
    ct, ft, wt = (torch.from_numpy(a).to(dev) for a in (coords, feats, w))
    out = {}
    try:
        for path in (1, 2):
            scnn.set_conv_path(path)
            oc, of, n = scnn.sparse_conv_fwd(extent, batch, ct, ft, (3, 3, 3), wt, rho_up=1.0, relu=False, pool=False)
            assert int(n[2]) == 0
            out[path] = (oc.cpu().numpy(), of.cpu().numpy(), scnn.last_conv_kernel())
    finally:
        scnn.set_conv_path(0)
    say(f"families seed={seed} extent={extent} B={batch} {c_in}->{c_out} rows={coords.shape[0]} "
        f"sites out={out[1][0].shape[0]} kernels={out[1][2]}, {out[2][2]}")
    assert out[1][2] == "k_conv_valu" and out[2][2] == "k_conv_quad"
    assert np.array_equal(out[1][0], out[2][0]), "the two kernel families disagree on the output sites"
    ref, got = out[1][1], out[2][1]
    assert np.all(np.abs(got - ref) <= RTOL * np.abs(ref) + ATOL), "the two kernel families disagree on a value"
