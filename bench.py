#!/usr/bin/env python3
"""Benchmark of the forward sparse convolution layer with attention on one MI355X.

A step = one pass of the whole hot path (index build, candidate sites, convolution,
k-selection, ReLU, compaction and write) over one batch of the r = 128 workload:
3-D shell-surface voxel grid 128^3, batch 4, 32 -> 64 channels, dense 3x3x3 filter,
rho_up = 0.05, ReLU.  Inputs are synthetic (seeded) and resident in HBM before the
timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_FP32_TFLOPS = 157.3
PEAK_FP64_VECTOR_TFLOPS = 78.6


def cpu_baseline(wl, layer, w, mac_total):
    """The oracle, as it stands, on the host cores: the whole batch on all the cores the box gives us, and sample 0
    on one thread (the whole batch on one thread would take over a minute)."""
    import numpy as np
    import oracle
    k = oracle.k_from_rho(layer.rho_up, int(np.prod(wl.extent)))
    ws = np.ascontiguousarray(w)

    def run(batch, coords, feats, threads):
        t0 = time.perf_counter()
        _, _, info = oracle.sparse_conv_fwd(wl.extent, batch, coords, feats, layer.ksize, ws, k=k, relu=layer.relu,
                                            pool=layer.pool, threads=threads, return_info=True)
        return time.perf_counter() - t0, info

    threads = min(16, os.cpu_count() or 1)
    dt, info = run(wl.batch, wl.coords, wl.feats, threads)
    multi = {"value": info["macs"] / dt / 1e9, "unit": "GMAC/s (non-zero MACs)", "cores": info["threads"],
             "kind": "oracle", "seconds": dt,
             "sample": f"the whole batch of {wl.batch} samples, all {w.shape[2]} output channels "
                       f"({info['macs'] / 1e9:.3f} of {mac_total / 1e9:.3f} GMAC), full layer incl. selection + ReLU"}
    sel = wl.coords[:, 0] == 0
    dt1, info1 = run(1, wl.coords[sel].copy(), wl.feats[sel], 1)
    single = {"value": info1["macs"] / dt1 / 1e9, "unit": "GMAC/s (non-zero MACs)", "cores": info1["threads"],
              "kind": "oracle", "seconds": dt1,
              "sample": f"sample 0 of {wl.batch}, all {w.shape[2]} output channels "
                        f"({info1['macs'] / 1e9:.3f} of {mac_total / 1e9:.3f} GMAC), full layer incl. selection + ReLU"}
    return multi, single


def copy_ceiling(scnn, torch, dev):
    """GB/s (read + write) of a plain 1 GiB device-to-device copy kernel: what streaming reaches on this machine."""
    src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    scnn.calibration_copy(dst, src)
    best = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        scnn.calibration_copy(dst, src)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, 2.0 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del src, dst
    return best


def bench_stack(args):
    """A step = the nine-layer sparse part of OctNet3-R^3 + sparseToDense on one batch; each layer's row count is read
    back on the host (the boundary takes it as a host integer), so the timed region includes those nine round trips."""
    import numpy as np
    import torch
    import paper_1801_10585_amd as scnn
    from workloads import make_octnet3_stack
    dev = torch.device("cuda:0")
    wl = make_octnet3_stack(args.stack, batch=4)
    c0, f0 = torch.from_numpy(wl.coords).to(dev), torch.from_numpy(wl.feats).to(dev)
    ws = [torch.from_numpy(w).to(dev) for w in wl.filters]
    macs, rows_log, dens_log = 0, [], []
    ext, c, f = wl.extent, wl.coords, wl.feats
    # sizing pass (untimed): work count and per-layer densities
    cd, fd = c0, f0
    for L, w, wd in zip(wl.layers, wl.filters, ws):
        macs += scnn.count_mac_nz(ext, cd.cpu().numpy(), fd.cpu().numpy(), L.ksize, w)
        cd, fd, _ = scnn.sparse_conv_fwd(ext, wl.batch, cd, fd, L.ksize, wd, rho_up=L.rho_up, relu=L.relu, pool=L.pool)
        if L.pool:
            ext = tuple((e + 1) // 2 for e in ext)
        n_sites = wl.batch * int(np.prod(ext))
        rows_log.append(int(cd.shape[0]))
        dens_log.append(float((fd != 0).sum().item()) / (n_sites * L.c_out))

    def step():
        e, cc, ff = wl.extent, c0, f0
        for L, wd in zip(wl.layers, ws):
            cc, ff, _ = scnn.sparse_conv_fwd(e, wl.batch, cc, ff, L.ksize, wd, rho_up=L.rho_up, relu=L.relu,
                                             pool=L.pool)
            if L.pool:
                e = tuple((x + 1) // 2 for x in e)
        return scnn.sparse_to_dense(e, wl.batch, cc, ff)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps * 1e3

    ms_calls = timed(step)
    # the same chain enqueued without host reads (device-resident row counts, buffers at their capacities) ...
    layers, e, cap = [], wl.extent, wl.coords.shape[0]
    for L, wd in zip(wl.layers, ws):
        lay = scnn.ChainedLayer(e, wl.batch, cap, L.c_in, L.ksize, wd, rho_up=L.rho_up, relu=L.relu, pool=L.pool)
        layers.append(lay)
        e, cap = lay.out_extent, lay.out_capacity
    dense = torch.empty((wl.batch, wl.layers[-1].c_out, *e), dtype=torch.float32, device=dev)
    n0 = torch.tensor([wl.coords.shape[0]], dtype=torch.int64, device=dev)

    def chain():
        cc, ff, nd = c0, f0, n0
        for lay in layers:
            cc, ff, nnz = lay(cc, ff, nd)
            nd = nnz[:1]
        scnn.sparse_to_dense(e, wl.batch, cc, ff, rows_dev=nd, out=dense)

    ms_chain = timed(chain)
    # ... and captured once in a HIP graph, replayed per step
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    ms_graph = timed(graph.replay)
    rows_final = int(layers[-1].nnz.cpu()[0])
    assert rows_final == rows_log[-1], "the graph's result disagrees with the call-by-call chain"
    line = {
        "metric": "effective non-zero GMAC/s of a nine-layer sparse conv+attention stack, end to end",
        "value": macs / (ms_graph * 1e-3) / 1e9, "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_graph, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "ms_per_step_by_mode": {"call_by_call_with_host_reads": ms_calls, "chained_device_counts": ms_chain,
                                "hip_graph_replay": ms_graph},
        "config": {"workload": wl.name, "grid": list(wl.extent), "batch": wl.batch, "rows_in": int(wl.coords.shape[0]),
                   "layers": [[L.c_in, L.c_out, L.rho_up, bool(L.pool)] for L in wl.layers], "mac_nz": int(macs),
                   "rows_after_layer": rows_log, "entry_density_after_layer": dens_log, "seed": wl.seed},
    }
    print(json.dumps(line))


def bench_backward(args, wl, layer, w, coords, feats, wd):
    """Backward pass of the same layer: gradient rows with the sparsity pattern of the layer's own output (taken
    from one untimed forward call), random values.  A step = one sparse_conv_bwd call."""
    import numpy as np
    import torch
    import paper_1801_10585_amd as scnn
    dev = coords.device
    nnz_in, c_in = wl.feats.shape
    c_out = w.shape[2]
    yc, yf, _ = scnn.sparse_conv_fwd(wl.extent, wl.batch, coords, feats, layer.ksize, wd, rho_up=layer.rho_up,
                                     relu=layer.relu, pool=False)
    gen = torch.Generator(device="cpu").manual_seed(wl.seed)
    g_feats = (torch.randn(yf.shape, generator=gen).to(dev) * (yf != 0)).contiguous()
    g_coords = yc.contiguous()
    g_rows = int(g_coords.shape[0])
    visits = scnn.count_bwd_visits(wl.extent, wl.batch, wl.coords, wl.feats, layer.ksize, w, g_coords.cpu().numpy())
    ws_bytes = scnn.sparse_conv_bwd_workspace(wl.extent, wl.batch, nnz_in, c_in, c_out, layer.ksize, g_rows)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    out = (torch.empty((nnz_in, c_in), dtype=torch.float32, device=dev),
           torch.empty(w.shape, dtype=torch.float32, device=dev), torch.zeros(4, dtype=torch.int64, device=dev))

    def step():
        scnn.sparse_conv_bwd(wl.extent, wl.batch, coords, feats, layer.ksize, wd, g_coords, g_feats,
                             workspace=workspace, out=out, sync=False)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    scnn.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    scnn.profile_enable(False)
    stage_ms, calls = scnn.profile_collect()
    assert int(out[2].cpu()[2]) == 0
    stage = {k: v / max(calls, 1) for k, v in stage_ms.items() if k.startswith("bwd_")}
    ms_per_step = dt / args.steps * 1e3
    mfma = c_out % 32 == 0 and c_out <= 128 and c_in % 16 == 0 and c_in <= 64
    peak = PEAK_MFMA_FP32_TFLOPS if mfma else PEAK_FP64_VECTOR_TFLOPS
    # the two contractions (bp_data and bp_filter) do one multiply-add per visit each
    dominant = "bwd_filter" if stage["bwd_filter"] >= stage["bwd_data_conv"] else "bwd_data_conv"
    tflops = 2.0 * visits / (stage[dominant] * 1e-3) / 1e12
    # HBM bytes of the dominant kernel per launch, from the committed counter runs of this command (see main())
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"bwd_cfg{args.config}_traffic.json")
    if not args.paper_runtime and os.path.exists(tpath):
        try:
            rec = json.load(open(tpath)).get(dominant)
            if rec:
                traffic = rec.get("hbm_bytes_per_launch")
                traffic_source = "profiles/" + os.path.basename(tpath) + ": " + rec.get("source", "")
        except Exception:
            traffic = None
    line = {
        "metric": "effective non-zero GMAC/s of the sparse conv backward pass (two multiply-adds per visit)",
        "value": 2.0 * visits * args.steps / dt / 1e9, "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name + "_backward", "grid": list(wl.extent), "batch": wl.batch, "c_in": c_in,
                   "c_out": c_out, "ksize": list(layer.ksize), "filter_density": layer.filter_density,
                   "rho_up": layer.rho_up, "rows_in": int(nnz_in), "gradient_rows": g_rows, "visits": int(visits),
                   "seed": wl.seed},
        "roofline": {"bound": "mfma" if mfma else "alu", "kernel": dominant, "achieved": tflops, "peak": peak,
                     "unit": "TFLOP/s", "frac": tflops / peak, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel_ms": stage[dominant],
                     "flops_per_launch": 2 * int(visits)},
        "stage_ms": stage,
    }
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload index (1..5); 4 is the headline")
    ap.add_argument("--paper-runtime", type=int, default=0, metavar="R",
                    help="instead of --config: the paper's runtime experiment (Sec. 4.1) at resolution R "
                         "(random sites, density = rho_up = 1/R, 1 -> 8 channels, batch 1); not the headline")
    ap.add_argument("--rho-f", type=float, default=1.0, help="filter density of --paper-runtime")
    ap.add_argument("--stack", type=int, default=0, metavar="R", choices=[0, 32, 64, 128],
                    help="instead of --config: the sparse part of the paper's OctNet3-R^3 network (nine convolutions, "
                         "two poolings, sparseToDense) with random weights, end to end; not the headline")
    ap.add_argument("--backward", action="store_true",
                    help="time the backward pass (Algorithm 2) of the same layer instead; not the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rho-up", type=float, default=None, help="override the configuration's rho_up (not the headline)")
    ap.add_argument("--layer", type=int, default=1,
                    help="which layer of a multi-layer configuration to time (1-based; its input is produced by the "
                         "library from the layers before it, untimed); not the headline")
    ap.add_argument("--conv-path", type=int, default=0, choices=[0, 1, 2, 3],
                    help="convolution kernel family (scnn_set_conv_path): 0 the library's choice (the headline), "
                         "1 vector kernels, 2 matrix cores wherever possible, 3 the pair-list matrix-core kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the layer shards by sample with no exchange; "
              "no multi-GPU path exists) -- use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_1801_10585_amd as scnn
    from workloads import make_config, make_paper_runtime

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    scnn.set_conv_path(args.conv_path)
    if args.stack:
        return bench_stack(args)
    wl = make_paper_runtime(args.paper_runtime, args.rho_f) if args.paper_runtime else make_config(args.config)
    if not 1 <= args.layer <= len(wl.layers):
        print(f"bench.py: configuration {args.config} has {len(wl.layers)} layer(s)", file=sys.stderr)
        sys.exit(2)
    if args.layer > 1:
        # the timed layer's input: the output of the layers before it (and their pooling), computed here, untimed
        import dataclasses
        cc, ff, ext = torch.from_numpy(wl.coords).to(dev), torch.from_numpy(wl.feats).to(dev), wl.extent
        for L, wprev in zip(wl.layers[:args.layer - 1], wl.filters):
            cc, ff, _ = scnn.sparse_conv_fwd(ext, wl.batch, cc, ff, L.ksize, torch.from_numpy(wprev).to(dev),
                                             rho_up=L.rho_up, relu=L.relu, pool=L.pool)
            if L.pool:
                ext = tuple((e + 1) // 2 for e in ext)
        wl = dataclasses.replace(wl, name=f"{wl.name}_layer{args.layer}", extent=ext, coords=cc.cpu().numpy(),
                                 feats=ff.cpu().numpy(), layers=wl.layers[args.layer - 1:],
                                 filters=wl.filters[args.layer - 1:])
    layer = wl.layers[0]
    if args.rho_up is not None:
        import dataclasses
        layer = dataclasses.replace(layer, rho_up=args.rho_up)
    w = wl.filters[0]
    ndim = wl.ndim
    mac_nz = scnn.count_mac_nz(wl.extent, wl.coords, wl.feats, layer.ksize, w)

    coords = torch.from_numpy(wl.coords).to(dev)
    feats = torch.from_numpy(wl.feats).to(dev)
    wd = torch.from_numpy(w).to(dev)
    nnz_in, c_in = wl.feats.shape
    c_out = w.shape[2]
    copy_gbs = copy_ceiling(scnn, torch, dev)  # (also the known-size copy that scales the profiler's byte counters)
    if args.backward:
        return bench_backward(args, wl, layer, w, coords, feats, wd)
    # size the buffers from a first (untimed) run: candidate count is data dependent
    oc0, of0, n0 = scnn.sparse_conv_fwd(wl.extent, wl.batch, coords, feats, layer.ksize, wd, rho_up=layer.rho_up,
                                        relu=layer.relu, pool=layer.pool)
    rows_out, n_cand = int(n0[0]), int(n0[1])
    del oc0, of0
    cand_cap = n_cand
    fuse = (1 if layer.relu else 0) | (2 if layer.pool else 0)
    ws_bytes = scnn.sparse_conv_fwd_workspace(wl.extent, wl.batch, nnz_in, c_in, c_out, layer.ksize, fuse, cand_cap)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    out = (torch.empty((cand_cap, 1 + ndim), dtype=torch.int32, device=dev),
           torch.empty((cand_cap, c_out), dtype=torch.float32, device=dev),
           torch.zeros(4, dtype=torch.int64, device=dev))

    def step():
        scnn.sparse_conv_fwd(wl.extent, wl.batch, coords, feats, layer.ksize, wd, rho_up=layer.rho_up,
                             relu=layer.relu, pool=layer.pool, out_capacity=cand_cap, cand_capacity=cand_cap,
                             workspace=workspace, out=out, sync=False)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # untimed: the same number of calls with the timed region's event mode, so that the library's events exist before
    # the clock starts (creating them costs about 10 us each)
    scnn.profile_enable(3)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    scnn.profile_collect()
    # timed region: on every fourth call the library records two HIP events on the launch stream, around the
    # convolution kernel (the dominant one, whose duration the roofline object needs from this very region)
    scnn.profile_enable(3)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    scnn.profile_enable(False)
    conv_only, conv_calls = scnn.profile_collect()
    n_chk = out[2].cpu()
    assert int(n_chk[0]) == rows_out and int(n_chk[2]) == 0, "timed runs disagree with the sizing run"

    # the same region once more with events at every stage boundary (the per-stage breakdown; eight events per call
    # cost about 0.03 ms), and once without any, to state what the events cost
    scnn.profile_enable(1)
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_stages = time.perf_counter() - t1
    scnn.profile_enable(False)
    stage_ms, calls = scnn.profile_collect()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_plain = time.perf_counter() - t1

    ms_per_step = dt / args.steps * 1e3
    gmacs = mac_nz * args.steps / dt / 1e9
    conv_ms = conv_only["conv"] / max(conv_calls, 1)
    conv_tflops = 2.0 * mac_nz / (conv_ms * 1e-3) / 1e12
    bytes_alg = scnn.algorithmic_bytes(ndim, nnz_in, c_in, w.shape[0], c_out, n_cand, rows_out)
    conv_kernel = scnn.last_conv_kernel()   # what the library launched, by its own rule
    # HBM bytes of the dominant kernel per launch: hardware counters cannot be read from inside this process, so the
    # figure is the one committed from two counter runs of this same command under the profiler (and only used if it
    # was taken for the kernel that ran here)
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"conv_cfg{args.config}_traffic.json")
    if not args.paper_runtime and args.layer == 1 and os.path.exists(tpath):
        try:
            rec = json.load(open(tpath))
            if rec.get("kernel", "").startswith(conv_kernel):
                traffic = rec.get("hbm_bytes_per_launch")
                traffic_source = "profiles/" + os.path.basename(tpath) + ": " + rec.get("source", "")
        except Exception:
            traffic = None
    on_matrix_cores = conv_kernel in ("k_conv_quad", "k_conv_mfma")
    # the matrix-core kernel is priced against the fp32 MFMA peak, the vector kernel (fp64 FMA) against the fp64
    # vector peak
    conv_peak = PEAK_MFMA_FP32_TFLOPS if on_matrix_cores else PEAK_FP64_VECTOR_TFLOPS
    line = {
        "metric": "effective non-zero GMAC/s of sparse conv+attention; % of HBM roofline",
        "value": gmacs, "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "grid": list(wl.extent), "batch": wl.batch, "c_in": c_in, "c_out": c_out,
                   "ksize": list(layer.ksize), "filter_density": layer.filter_density, "rho_up": layer.rho_up,
                   "relu": layer.relu, "pool": layer.pool, "rows_in": int(nnz_in), "candidate_sites": n_cand,
                   "rows_out": rows_out, "mac_nz": int(mac_nz), "input_density": wl.density, "seed": wl.seed},
        "roofline": {"bound": "mfma" if on_matrix_cores else "alu", "kernel": conv_kernel,
                     "achieved": conv_tflops, "peak": conv_peak, "unit": "TFLOP/s", "frac": conv_tflops / conv_peak,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel_ms": conv_ms, "kernel_launches_timed": conv_calls, "flops_per_launch": 2 * int(mac_nz),
                     # the whole layer against its own bound: max(algorithmic bytes / 8 TB/s, flops / fp32 MFMA peak)
                     # over the step time
                     "layer_frac": max(bytes_alg["alg"] / (PEAK_HBM_GBS * 1e9),
                                       2.0 * mac_nz / (PEAK_MFMA_FP32_TFLOPS * 1e12)) / (ms_per_step * 1e-3)},
        "hbm": {"algorithmic_bytes": bytes_alg["alg"], "achieved_GBs": bytes_alg["alg"] / (ms_per_step * 1e-3) / 1e9,
                "frac_of_8TBs": bytes_alg["alg"] / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "copy_kernel_GBs": copy_gbs,
                "whole_layer_roofline_frac": max(bytes_alg["alg"] / (PEAK_HBM_GBS * 1e9),
                                                 2.0 * mac_nz / (PEAK_MFMA_FP32_TFLOPS * 1e12)) / (ms_per_step * 1e-3)},
        "stage_ms": {k: v / max(calls, 1) for k, v in stage_ms.items() if not k.startswith("bwd_")},
        "ms_per_step_with_stage_events": dt_stages / args.steps * 1e3,
        "ms_per_step_without_events": dt_plain / args.steps * 1e3,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"], line["cpu_baseline_1thread"] = cpu_baseline(wl, layer, w, mac_nz)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
