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
