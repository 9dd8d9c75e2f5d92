"""sparse_relu_static (the entry point that allocates nothing) against sparse_relu, through the C ABI.

Two calls in a row on the same GPU, the second with a smaller input: the library's own scratch array keeps the
first call's contents, so the second call shows that everything that must start from zero is cleared.
"""
import ctypes
import sys

import numpy as np
import pytest
import torch

import paper_1801_10585_amd as scnn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rows(rng, extent, batch, density, channels):
    occ = rng.random((batch, *extent)) < density
    coords = np.ascontiguousarray(np.argwhere(occ).astype(np.int32))
    feats = rng.standard_normal((coords.shape[0], channels)).astype(np.float32)
    feats[rng.random(feats.shape) < 0.4] = 0.0
    drop = rng.random(coords.shape[0]) < 0.2   # rows without a positive entry disappear
    feats[drop] = -np.abs(feats[drop]) - 1.0
    return coords, feats


def _static_call(L, ndim, coords, feats, out_coords, out_feats, nnz):
    rows, ch = feats.shape
    stream = torch.cuda.current_stream().cuda_stream
    rc = L.sparse_relu_static(ndim, ctypes.c_void_p(coords.data_ptr()), ctypes.c_void_p(feats.data_ptr()), rows, ch,
                              ctypes.c_void_p(out_coords.data_ptr()), ctypes.c_void_p(out_feats.data_ptr()),
                              out_feats.shape[0], ctypes.c_void_p(nnz.data_ptr()), ctypes.c_void_p(stream))
    assert rc == 0, L.scnn_last_error()


def test_static_relu_matches_workspace_relu_twice():
    L = scnn.load_library()
    rng = np.random.default_rng(77)
    cases = [((40, 40, 40), 2, 0.25, 24), ((17, 9, 12), 1, 0.3, 5)]   # 32 000 rows (several scan blocks), then 550
    for extent, batch, density, ch in cases:
        coords, feats = _rows(rng, extent, batch, density, ch)
        print(f"static relu extent={extent} B={batch} C={ch} rows={coords.shape[0]}", flush=True)
        sys.stdout.flush()
        c = torch.from_numpy(coords).to(DEV)
        f = torch.from_numpy(feats).to(DEV)
        want_c, want_f, want_n = scnn.sparse_relu(len(extent), c, f)
        out_c = torch.full((coords.shape[0], 1 + len(extent)), -7, dtype=torch.int32, device=DEV)
        out_f = torch.full((coords.shape[0], ch), -7.0, dtype=torch.float32, device=DEV)
        nnz = torch.full((4,), -1, dtype=torch.int64, device=DEV)
        _static_call(L, len(extent), c, f, out_c, out_f, nnz)
        torch.cuda.synchronize()
        n = nnz.cpu().numpy()
        assert np.array_equal(n, want_n.numpy()), (n, want_n)
        rows = int(n[0])
        assert 0 < rows < coords.shape[0]
        assert torch.equal(out_c[:rows], want_c) and torch.equal(out_f[:rows], want_f)
        # nothing is written past the rows produced
        assert bool((out_c[rows:] == -7).all()) and bool((out_f[rows:] == -7.0).all())


def test_static_relu_rejects_too_many_rows_on_the_host():
    L = scnn.load_library()
    limit = L.sparse_relu_static_max_rows()
    assert limit == 1 << 20
    fake = ctypes.c_void_p(256)
    rc = L.sparse_relu_static(3, fake, fake, limit + 1, 4, fake, fake, 16, fake, None)
    assert rc == -2 and b"at most" in L.scnn_last_error()
