"""CPU-only checks of the C-ABI library: it loads, exports what the header declares,
and rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1801_10585_amd as scnn
import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "scnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", "".join(
        l for l in text.splitlines(True) if not l.lstrip().startswith("#")))))


def test_library_exports_every_declared_symbol():
    L = scnn.load_library()
    declared = _declared_functions()
    assert set(declared) == set(scnn.EXPORTED_SYMBOLS), declared
    for name in declared:
        assert hasattr(L, name), name
    assert L.scnn_version() >= 1


@pytest.mark.parametrize("rho,n", [(0.15, 784), (0.05, 128 ** 3), (0.1, 30), (0.3, 10), (0.0, 5), (1.0, 7), (0.02, 256 ** 3),
                                   (1 / 32, 32 ** 3), (0.10, 64 ** 3), (0.15, 32 ** 3)])
def test_k_from_rho_matches_oracle(rho, n):
    assert scnn.k_from_rho(rho, n) == oracle.k_from_rho(rho, n)


def _i32(v):
    return (ctypes.c_int32 * len(v))(*v)


def test_host_argument_checks():
    L = scnn.load_library()
    ext3, ks3 = _i32([8, 8, 8]), _i32([3, 3, 3])
    assert L.sparse_conv_fwd_max_rows(3, ext3, 2, 10, ks3) == 270
    assert L.sparse_conv_fwd_max_rows(3, ext3, 2, 1000, ks3) == 1024
    assert L.sparse_conv_fwd_max_rows(4, ext3, 2, 10, ks3) == -1
    assert L.sparse_conv_fwd_max_rows(3, ext3, 2, 10, _i32([3, 2, 3])) == -1
    assert b"odd" in L.scnn_last_error()
    assert L.sparse_conv_fwd_workspace(3, ext3, 2, 10, 4, 4, ks3, 0, 0) > 0
    assert L.sparse_conv_fwd_workspace(3, ext3, 2, 10, 0, 4, ks3, 0, 0) == 0
    assert L.sparse_conv_fwd_workspace(3, ext3, 2, 10, 4, 4, ks3, 3, 0) > L.sparse_conv_fwd_workspace(
        3, ext3, 2, 10, 4, 4, ks3, 0, 0)
    # a call with bad arguments returns before touching the device
    fake = ctypes.c_void_p(256)
    rc = L.sparse_conv_fwd(3, ext3, 2, fake, fake, 10, 4, ks3, fake, None, 4, 1.5, 0, 0, fake, fake, 10, 0, fake, fake,
                           1 << 30, None)
    assert rc == -1 and b"rho_up" in L.scnn_last_error()
    rc = L.sparse_conv_fwd(3, ext3, 2, fake, fake, 10, 4, ks3, fake, None, 4, 0.5, 7, 0, fake, fake, 10, 0, fake, fake,
                           1 << 30, None)
    assert rc == -1
    rc = L.sparse_conv_fwd(3, ext3, 2, fake, fake, 10, 4, ks3, fake, None, 4, 0.5, 0, 0, fake, fake, 10, 0, fake, fake,
                           16, None)
    assert rc == -3 and b"workspace" in L.scnn_last_error()
    rc = L.sparse_conv_fwd(3, ext3, 2, fake, fake, 10, 4, ks3, fake, None, 4, 0.5, 0, 0, fake, fake, 10, 0, fake,
                           ctypes.c_void_p(8), 1 << 30, None)
    assert rc == -3
    rc = L.attention_topk(3, ext3, 2, fake, fake, 10, 4, -1, 0, fake, fake, 10, fake, fake, 1 << 30, None)
    assert rc == -1
    rc = L.sparse_maxpool(3, ext3, 2, 3, fake, fake, 10, 4, fake, fake, 10, fake, fake, 1 << 30, None)
    assert rc == -1 and b"window" in L.scnn_last_error()
    rc = L.sparse_relu(5, fake, fake, 10, 4, fake, fake, 10, fake, fake, 1 << 30, None)
    assert rc == -1
    big = _i32([2048, 2048, 2048])
    assert L.sparse_conv_fwd_max_rows(3, big, 1, 10, ks3) == -2


def test_host_argument_checks_of_the_widening_entry_points():
    L = scnn.load_library()
    ext3, ks3 = _i32([8, 8, 8]), _i32([3, 3, 3])
    fake = ctypes.c_void_p(256)
    f64 = ctypes.c_double
    # backward pass
    assert L.sparse_conv_bwd_workspace(3, ext3, 2, 10, 4, 4, ks3, 20) > 0
    assert L.sparse_conv_bwd_workspace(3, ext3, 2, 10, 0, 4, ks3, 20) == 0
    assert L.sparse_conv_bwd_workspace(3, ext3, 2, 10, 4, 4, _i32([3, 4, 3]), 20) == 0
    rc = L.sparse_conv_bwd(3, ext3, 2, fake, fake, 10, 4, ks3, fake, 4, fake, fake, 20, fake, fake, fake, fake, 16, None)
    assert rc == -3 and b"workspace" in L.scnn_last_error()
    rc = L.sparse_conv_bwd(3, ext3, 2, fake, fake, 10, 4, ks3, None, 4, fake, fake, 20, fake, fake, fake, fake, 1 << 30,
                           None)
    assert rc == -1
    rc = L.sparse_conv_bwd(3, ext3, 2, fake, fake, 10, 4, ks3, fake, 4, None, fake, 20, fake, fake, fake, fake, 1 << 30,
                           None)
    assert rc == -1 and b"gradient" in L.scnn_last_error()
    # chained forward: the device-resident count is mandatory
    rc = L.sparse_conv_fwd_chained(3, ext3, 2, fake, fake, 10, None, 4, ks3, fake, None, 4, 0.5, 0, 0, fake, fake, 10, 0,
                                   fake, fake, 1 << 30, None)
    assert rc == -1 and b"nnz_in_dev" in L.scnn_last_error()
    rc = L.sparse_conv_fwd_chained(3, ext3, 2, fake, fake, 10, fake, 4, ks3, fake, None, 4, 1.5, 0, 0, fake, fake, 10, 0,
                                   fake, fake, 1 << 30, None)
    assert rc == -1 and b"rho_up" in L.scnn_last_error()
    # sparseToDense
    assert L.sparse_to_dense(3, ext3, 2, fake, fake, 10, None, 0, fake, None) == -1
    assert L.sparse_to_dense(3, ext3, 2, fake, fake, 10, None, 4, ctypes.c_void_p(260), None) == -1
    assert b"aligned" in L.scnn_last_error()
    assert L.sparse_to_dense(3, ext3, 2, fake, fake, 10, None, 4, None, None) == -1
    # regulariser and pruning
    assert L.density_regulariser_workspace() >= 256
    args = [fake, 10, None, 4, 1000]
    tail = [fake, 100, fake, fake, fake, ctypes.c_size_t(1 << 20), None]
    assert L.density_regulariser(*args, f64(1.5), f64(0.1), f64(1.0), f64(1.0), f64(1e-3), *tail) == -1
    assert L.density_regulariser(*args, f64(0.5), f64(-0.1), f64(1.0), f64(1.0), f64(1e-3), *tail) == -1
    assert L.density_regulariser(fake, 10, None, 4, 0, f64(0.5), f64(0.1), f64(1.0), f64(1.0), f64(1e-3), *tail) == -1
    assert L.density_regulariser(*args, f64(0.5), f64(0.1), f64(1.0), f64(1.0), f64(1e-3), fake, 100, fake, fake, fake,
                                 ctypes.c_size_t(8), None) == -3
    assert L.prune_weights(fake, fake, 10, ctypes.c_float(-1.0), fake, None) == -1
    assert L.prune_weights(None, fake, 10, ctypes.c_float(0.1), fake, None) == -1
    assert L.prune_weights(fake, fake, 10, ctypes.c_float(0.1), None, None) == -1


def test_measurement_switches_reject_unknown_modes():
    L = scnn.load_library()
    assert L.scnn_profile_enable(4) == -1 and b"profile mode" in L.scnn_last_error()
    assert L.scnn_profile_enable(2) == 0 and L.scnn_profile_enable(0) == 0
    assert L.scnn_set_conv_path(4) == -1 and b"conv path" in L.scnn_last_error()
    assert L.scnn_set_conv_path(2) == 0 and L.scnn_set_conv_path(0) == 0
    names = [L.scnn_profile_stage_name(i).decode() for i in range(L.scnn_profile_stage_count())]
    assert names[3] == "conv" and len(set(names)) == len(names)


def test_mac_count_matches_oracle_loop_count():
    from workloads import make_config
    wl = make_config(2, r=16, batch=2)
    w = wl.filters[0]
    macs = scnn.count_mac_nz(wl.extent, wl.coords, wl.feats, wl.layers[0].ksize, w)
    _, _, info = oracle.sparse_conv_fwd(wl.extent, wl.batch, wl.coords, wl.feats, wl.layers[0].ksize, w, k=1,
                                        return_info=True)
    assert macs == info["macs"]
    wl = make_config(1)
    macs = scnn.count_mac_nz(wl.extent, wl.coords, wl.feats, wl.layers[0].ksize, wl.filters[0])
    _, _, info = oracle.sparse_conv_fwd(wl.extent, wl.batch, wl.coords, wl.feats, wl.layers[0].ksize, wl.filters[0],
                                        k=1, return_info=True)
    assert macs == info["macs"]


def test_backward_visit_count_matches_oracle_loop_counter():
    import numpy as np
    import oracle
    from workloads import make_filter, random_sparse_sites
    rng = np.random.default_rng(0)
    for extent, batch, ci, co, ks in [((9, 7), 2, 3, 4, (3, 5)), ((6, 7, 5), 2, 2, 3, (3, 3, 3))]:
        c = random_sparse_sites(rng, extent, batch, 0.3)
        f = rng.normal(size=(c.shape[0], ci)).astype(np.float32)
        f *= rng.random(f.shape) > 0.3
        w = make_filter(rng, ks, ci, co, 0.5, 0.3)
        # the oracle's loop visits every in-grid site of its dense gradient buffer; with a gradient row on every
        # site the two counts must agree, and thinning the gradient rows can only lower the count of rows met
        full = random_sparse_sites(rng, extent, batch, 1.1)
        _, _, info = oracle.sparse_conv_bwd(extent, batch, c, f, ks, w, full, np.ones((full.shape[0], co), np.float32),
                                            return_info=True)
        assert scnn.count_bwd_visits(extent, batch, c, f, ks, w, full) == info["visits"]
        assert scnn.count_bwd_visits(extent, batch, c, f, ks, w, full) == scnn.count_mac_nz(extent, c, f, ks, w)
        thin = random_sparse_sites(rng, extent, batch, 0.4)
        assert 0 < scnn.count_bwd_visits(extent, batch, c, f, ks, w, thin) < info["visits"]


def test_operators_refuse_cpu_tensors():
    import torch
    c = torch.zeros((1, 4), dtype=torch.int32)
    f = torch.zeros((1, 2), dtype=torch.float32)
    with pytest.raises(ValueError):
        scnn.sparse_relu(3, c, f)
