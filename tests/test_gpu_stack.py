"""GPU parity of a multi-layer chain: the sparse part of the paper's OctNet3 networks (appendix table of
architectures) with random weights, and sparseToDense.

Each layer is checked "teacher-forced": both sides take the ORACLE's output of the previous layer as input, so that a
difference cannot hide behind an earlier one (and nothing the HIP path produced is ever an oracle input).  The
library's own end-to-end chain is then compared with the oracle's chain on row counts and on the final dense tensor."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_1801_10585_amd as scnn
from tests.test_gpu_parity import _sampled_columns, check_conv_against_oracle, dev, host, pooled_extent, say
from workloads import make_octnet3_stack, random_sparse_sites

pytestmark = pytest.mark.gpu


def oracle_chain(wl, threads=16):
    """[(extent, coords, feats)] before every layer, plus the final output."""
    ext, c, f = wl.extent, wl.coords, wl.feats
    states = []
    for L, w in zip(wl.layers, wl.filters):
        states.append((ext, c, f))
        k = oracle.k_from_rho(L.rho_up, int(np.prod(ext)))
        c, f = oracle.sparse_conv_fwd(ext, wl.batch, c, f, L.ksize, w, k=k, relu=L.relu, pool=L.pool, threads=threads)
        if L.pool:
            ext = pooled_extent(ext)
    states.append((ext, c, f))
    return states


@pytest.mark.parametrize("r", [32, 64])
def test_octnet3_sparse_part_layer_by_layer_and_end_to_end(r):
    wl = make_octnet3_stack(r)
    states = oracle_chain(wl)
    rng = np.random.default_rng(r)
    for i, (L, w) in enumerate(zip(wl.layers, wl.filters)):
        ext, c, f = states[i]
        k = scnn.k_from_rho(L.rho_up, int(np.prod(ext)))
        say(f"octnet3-{r} layer {i}: {L.c_in}->{L.c_out} extent={ext} rows={c.shape[0]} k={k}")
        check_conv_against_oracle(ext, wl.batch, c, f, L.ksize, w, None, k, L.rho_up, scnn.ABS,
                                  columns=_sampled_columns(rng, wl.batch, L.c_out, 6), tag=f"octnet3-{r} L{i}")
    # the library's own chain, end to end
    ext, c, f = wl.extent, dev(wl.coords), dev(wl.feats)
    for i, (L, w) in enumerate(zip(wl.layers, wl.filters)):
        c, f, n = scnn.sparse_conv_fwd(ext, wl.batch, c, f, L.ksize, dev(w), rho_up=L.rho_up, relu=L.relu, pool=L.pool)
        assert int(n[2]) == 0
        if L.pool:
            ext = pooled_extent(ext)
        want_rows = states[i + 1][1].shape[0]
        assert abs(int(c.shape[0]) - want_rows) <= max(2, 0.002 * want_rows), (i, int(c.shape[0]), want_rows)
    dense = host(scnn.sparse_to_dense(ext, wl.batch, c, f))
    want = oracle.sparse_to_dense(ext, wl.batch, states[-1][1], states[-1][2])
    assert dense.shape == want.shape == (wl.batch, 24, *ext)
    bad = ~np.isclose(dense, want, rtol=1e-4, atol=1e-5)
    say(f"octnet3-{r} end to end: {int(bad.sum())} of {bad.size} dense elements differ beyond 1e-4")
    assert bad.mean() <= 1e-3


@pytest.mark.parametrize("extent,batch,channels", [((7, 5), 1, 1), ((9, 11), 3, 5), ((6, 5, 7), 2, 3), ((16, 16, 16), 2, 24),
                                                   ((33, 17, 5), 1, 70)])
def test_sparse_to_dense_is_exact(extent, batch, channels):
    rng = np.random.default_rng(sum(extent) + channels)
    coords = random_sparse_sites(rng, extent, batch, 0.3)
    feats = rng.normal(size=(coords.shape[0], channels)).astype(np.float32)
    feats *= rng.random(feats.shape) < 0.7
    got = host(scnn.sparse_to_dense(extent, batch, dev(coords), dev(feats)))
    assert np.array_equal(got, oracle.sparse_to_dense(extent, batch, coords, feats))
    # a buffer that held other data is overwritten entirely; an empty row list gives all zeros
    out = torch.full((batch, channels, *extent), 7.0, dtype=torch.float32, device="cuda:0")
    scnn.sparse_to_dense(extent, batch, dev(coords[:0]), dev(feats[:0]), out=out)
    assert not host(out).any()


def _eager_chain(wl):
    ext, c, f = wl.extent, dev(wl.coords), dev(wl.feats)
    for L, w in zip(wl.layers, wl.filters):
        c, f, n = scnn.sparse_conv_fwd(ext, wl.batch, c, f, L.ksize, dev(w), rho_up=L.rho_up, relu=L.relu, pool=L.pool)
        if L.pool:
            ext = pooled_extent(ext)
    return ext, host(c), host(f), host(scnn.sparse_to_dense(ext, wl.batch, c, f))


def _build_chain(wl):
    layers, ext, cap = [], wl.extent, wl.coords.shape[0]
    for L, w in zip(wl.layers, wl.filters):
        lay = scnn.ChainedLayer(ext, wl.batch, cap, L.c_in, L.ksize, dev(w), rho_up=L.rho_up, relu=L.relu, pool=L.pool)
        layers.append(lay)
        ext, cap = lay.out_extent, lay.out_capacity
    dense = torch.empty((wl.batch, wl.layers[-1].c_out, *ext), dtype=torch.float32, device="cuda:0")
    return layers, ext, dense


def _run_chain(layers, ext, dense, c, f, n_dev, batch):
    for lay in layers:
        c, f, nnz = lay(c, f, n_dev)
        n_dev = nnz[:1]
    scnn.sparse_to_dense(ext, batch, c, f, rows_dev=n_dev, out=dense)
    return c, f, nnz


@pytest.mark.parametrize("r", [32, 64])
def test_chain_without_host_reads_equals_the_call_by_call_chain(r):
    """The same nine layers enqueued back to back with device-resident row counts (buffers at their capacities):
    these channel widths run the vector kernels, whose sums have a fixed order, so the results must be identical."""
    wl = make_octnet3_stack(r)
    ext_e, c_e, f_e, dense_e = _eager_chain(wl)
    layers, ext, dense = _build_chain(wl)
    assert ext == ext_e
    n0 = torch.tensor([wl.coords.shape[0]], dtype=torch.int64, device="cuda:0")
    c, f, nnz = _run_chain(layers, ext, dense, dev(wl.coords), dev(wl.feats), n0, wl.batch)
    nnz = host(nnz)
    assert int(nnz[2]) == 0 and int(nnz[0]) == c_e.shape[0]
    assert np.array_equal(host(c)[:c_e.shape[0]], c_e) and np.array_equal(host(f)[:c_e.shape[0]], f_e)
    assert np.array_equal(host(dense), dense_e)
    say(f"octnet3-{r} chained: {int(nnz[0])} final rows, identical to the call-by-call chain")


def test_chain_captured_in_a_graph_replays_correctly():
    """The chain contains no allocation, host synchronisation or memset, so it can be captured; every replay is
    checked against the eager result, with eager work and synchronisations between the replays and a changed input
    before the last one."""
    wl = make_octnet3_stack(32)
    _, c_e, f_e, dense_e = _eager_chain(wl)
    layers, ext, dense = _build_chain(wl)
    cap = wl.coords.shape[0]
    cin, fin = dev(wl.coords).clone(), dev(wl.feats).clone()
    n0 = torch.tensor([cap], dtype=torch.int64, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up outside the capture
        _run_chain(layers, ext, dense, cin, fin, n0, wl.batch)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _run_chain(layers, ext, dense, cin, fin, n0, wl.batch)
    for rep in range(3):
        dense.fill_(-1.0)                               # eager work between replays
        scnn.sparse_relu(3, dev(wl.coords), dev(np.ones((cap, 2), np.float32)))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(host(dense), dense_e), f"replay {rep}"
        assert int(host(layers[-1].nnz)[0]) == c_e.shape[0]
    # a different input through the same graph: half of the rows (device-resident count), same buffers
    half = cap // 2
    n0.fill_(half)
    graph.replay()
    torch.cuda.synchronize()
    wl2_c, wl2_f = wl.coords[:half], wl.feats[:half]
    ext2, c2 = wl.extent, None
    cc, ff = dev(wl2_c), dev(wl2_f)
    for L, w in zip(wl.layers, wl.filters):
        cc, ff, _ = scnn.sparse_conv_fwd(ext2, wl.batch, cc, ff, L.ksize, dev(w), rho_up=L.rho_up, relu=L.relu,
                                         pool=L.pool)
        if L.pool:
            ext2 = pooled_extent(ext2)
    want = host(scnn.sparse_to_dense(ext2, wl.batch, cc, ff))
    assert np.array_equal(host(dense), want), "replay with a new device-resident row count"


def test_chained_layer_ignores_rows_past_the_device_count_on_the_matrix_core_path():
    """Wide channels (matrix-core kernels) through the chained entry point, with input arrays twice as long as the
    device-resident row count says and garbage behind it: the result must be the plain call's."""
    from workloads import make_config
    wl = make_config(4, r=48, batch=2)
    L = wl.layers[0]
    rows = wl.coords.shape[0]
    rng = np.random.default_rng(5)
    pad_c = np.full((rows, 4), 7, dtype=np.int32)                    # same site over and over: never indexed
    pad_f = rng.normal(size=(rows, L.c_in)).astype(np.float32)
    cin, fin = dev(np.concatenate([wl.coords, pad_c])), dev(np.concatenate([wl.feats, pad_f]))
    lay = scnn.ChainedLayer(wl.extent, wl.batch, 2 * rows, L.c_in, L.ksize, dev(wl.filters[0]), rho_up=L.rho_up,
                            relu=True)
    n_dev = torch.tensor([rows], dtype=torch.int64, device="cuda:0")
    oc, of, nnz = lay(cin, fin, n_dev)
    nnz = host(nnz)
    assert int(nnz[2]) == 0
    rc, rf, rn = scnn.sparse_conv_fwd(wl.extent, wl.batch, dev(wl.coords), dev(wl.feats), L.ksize, dev(wl.filters[0]),
                                      rho_up=L.rho_up, relu=True)
    n = int(nnz[0])
    assert n == rc.shape[0] and int(nnz[1]) == int(rn[1])
    assert np.array_equal(host(oc)[:n], host(rc))
    # the matrix-core kernel adds its fp64 partial sums in no fixed order: values agree to the last bits only
    assert np.allclose(host(of)[:n], host(rf), rtol=1e-6, atol=1e-7)
    # a count larger than the arrays is clamped to their capacity (here: the garbage rows then take part, flagged)
    n_dev.fill_(10 * rows)
    _, _, nnz2 = lay(cin, fin, n_dev)
    assert int(host(nnz2)[2]) & (scnn.FLAG_UNSORTED | scnn.FLAG_BAD_COORD)


def test_chained_narrow_layer_with_a_workspace_far_larger_than_its_data():
    """Narrow channels (vector kernels) through the chained entry point with input arrays sixty times as long as the
    device-resident row count: the workspace holds thousands of tiles, so only the streaming kernel is launched, and
    it runs on a layer of a few hundred tiles.  The result must be the plain call's, bit for bit."""
    from workloads import make_filter, random_sparse_sites
    rng = np.random.default_rng(17)
    extent, batch, c_in, c_out = (96, 96, 96), 2, 4, 12
    coords = random_sparse_sites(rng, extent, batch, 0.0006)
    rows = coords.shape[0]
    feats = rng.normal(size=(rows, c_in)).astype(np.float32)
    w = make_filter(rng, (3, 3, 3), c_in, c_out, 0.8, 0.3)
    cap = 60 * rows
    pad_c = np.full((cap - rows, 4), 5, dtype=np.int32)
    pad_f = rng.normal(size=(cap - rows, c_in)).astype(np.float32)
    cin, fin = dev(np.concatenate([coords, pad_c])), dev(np.concatenate([feats, pad_f]))
    lay = scnn.ChainedLayer(extent, batch, cap, c_in, (3, 3, 3), dev(w), rho_up=0.01, relu=True)
    n_dev = torch.tensor([rows], dtype=torch.int64, device="cuda:0")
    oc, of, nnz = lay(cin, fin, n_dev)
    nnz = host(nnz)
    assert int(nnz[2]) == 0
    rc, rf, rn = scnn.sparse_conv_fwd(extent, batch, dev(coords), dev(feats), (3, 3, 3), dev(w), rho_up=0.01, relu=True)
    n = int(nnz[0])
    say(f"chained narrow layer: {rows} of {cap} rows, {int(nnz[1])} candidate sites, {n} rows out")
    assert n == rc.shape[0] and int(nnz[1]) == int(rn[1]) and n > 0
    assert np.array_equal(host(oc)[:n], host(rc)) and np.array_equal(host(of)[:n], host(rf))
