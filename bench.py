#!/usr/bin/env python3
"""Benchmark of the Insum SpMM hot path on one MI355X.

A step is one SpMM launch of the library (all kernels of the call) on a synthetic
workload already resident in HBM; conversion to the fixed-length format happens once
before the timed region and is reported separately.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--no-extra]

The headline workload is cfg3 (GroupCOO, graph-aggregation shape, fp32, N = 128): the only
configuration whose dense operand exceeds the on-chip caches, i.e. the one the HBM
roofline applies to.  Unless --no-extra is given the line also carries the
BlockGroupCOO result on cfg5 (MFMA roofline) and short results for the other configs.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0      # dense bf16 / fp16
SIZEOF = {"f32": 4, "f16": 2, "bf16": 2}


def _torch_dtype(torch, name):
    return {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[name]


def _to_device(torch, x_f32, dtype):
    import synth
    st = synth.storage_array(x_f32, dtype)
    if dtype == "bf16":
        return torch.from_numpy(st.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(st).cuda()


def _time_launches(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / steps      # ms per step


def _time_graph_replay(torch, fn, launches=20, replays=10):
    """ms per launch when `launches` calls are captured once in a HIP graph and the graph is
    replayed: what a launch-bound workload costs without the host's per-launch work."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fn()                                   # warm (also: nothing is allocated during capture)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(launches):
                fn()
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(replays):
        graph.replay()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / (replays * launches)


def _per_launch_times(torch, fn, launches, flush=None):
    """Each launch timed on its own (HIP events around it); `flush`, when given, runs before
    every launch outside its timed window.  Returns (median, min) in ms."""
    times = []
    for _ in range(launches):
        if flush is not None:
            flush()
        start = torch.cuda.Event(enable_timing=True)
        stop = torch.cuda.Event(enable_timing=True)
        start.record()
        fn()
        stop.record()
        torch.cuda.synchronize()
        times.append(start.elapsed_time(stop))
    times.sort()
    return times[len(times) // 2], times[0]


def launch_statistics(torch, fn, launches=50):
    """Warm (back to back) and cold (a 1 GiB buffer is rewritten before every launch, which
    evicts the 8 x 4 MiB L2 and the 256 MB Infinity Cache) per-launch times of the headline."""
    for _ in range(5):
        fn()
    warm = _per_launch_times(torch, fn, launches)
    junk = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    cold = _per_launch_times(torch, fn, launches, flush=lambda: junk.add_(1.0))
    del junk
    return {"launches": launches, "warm_median_ms": warm[0], "warm_min_ms": warm[1],
            "cold_median_ms": cold[0], "cold_min_ms": cold[1],
            "note": "single launches between their own events (includes ~launch latency); ms_per_step is the "
                    "mean over back-to-back launches"}


def prepare(torch, I, name):
    """Generate a workload, move it to the device and convert it with the library."""
    import synth
    cfg = synth.make_config(name)
    row = torch.from_numpy(cfg["row"]).cuda()
    col = torch.from_numpy(cfg["col"]).cuda()
    val = _to_device(torch, cfg["val"], cfg["a_dtype"])
    B = _to_device(torch, cfg["B"], cfg["b_dtype"])
    conv_ms = None
    for _ in range(2):      # the second call sees a warm allocator: that one is reported
        A = None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if cfg["kind"] == "group":
            A = I.insum_coo_to_groupcoo(cfg["M"], cfg["K"], row, col, val, g=0)
        else:
            A = I.insum_coo_to_blockgroupcoo(cfg["M"], cfg["K"], row, col, val, cfg["bM"], cfg["bK"], g=0)
        torch.cuda.synchronize()
        conv_ms = (time.perf_counter() - t0) * 1e3
    nnz = int(cfg["row"].shape[0])
    del row, col, val
    return cfg, A, B, nnz, conv_ms


def _kernel_source_hashes():
    """sha256 of the kernel sources, by file name: a stored counter figure is only quoted for the
    sources it was measured on."""
    import hashlib
    out = {}
    csrc = os.path.join(ROOT, "paper_2510_17505_amd", "csrc")
    for fn in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, fn), "rb") as f:
            out[fn] = hashlib.sha256(f.read()).hexdigest()
    return out


def _traffic(name):
    """Counter-measured bytes per launch between L2 and the memory fabric (FETCH_SIZE + WRITE_SIZE,
    rocprofv3) from profiles/hbm_traffic.json, or None when that figure was taken on other kernel
    sources than the ones in the tree."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            entry = json.load(f).get(name)
    except (OSError, ValueError):
        return None
    if not entry:
        return None
    now = _kernel_source_hashes()
    for fn, sha in entry.get("source_sha256", {"?": "?"}).items():
        if now.get(fn) != sha:
            return None
    return entry.get("hbm_bytes_per_launch")


def run_workload(torch, I, name, steps, warmup, peaks=None):
    cfg, A, B, nnz, conv_ms = prepare(torch, I, name)
    M, N = cfg["M"], cfg["N"]
    sA, sB, sC = SIZEOF[cfg["a_dtype"]], SIZEOF[cfg["b_dtype"]], SIZEOF[cfg["c_dtype"]]
    C = torch.empty((M, N), dtype=_torch_dtype(torch, cfg["c_dtype"]), device="cuda")
    plan_ms = None
    if cfg["kind"] == "group":
        ws = torch.empty(I.insum_spmm_groupcoo_workspace_bytes(M, N, A.G, A.g), dtype=torch.uint8,
                         device="cuda")
        fn = lambda: I.insum_spmm_groupcoo(A, B, C_out=C, workspace=ws)
        slots = A.G * A.g
        # Bytes that have to come from beyond the caches when B does not fit them: every real
        # entry gathers a row of B; a padding slot repeats the row just fetched and adds only
        # its own column index and value; AM, and C written once.
        real_bytes = nnz * (N * sB + 4 + sA) + (slots - nnz) * (4 + sA) + 4 * A.G + M * N * sC
        # The same with every slot counted as a gather (what the kernel requests from L1/L2).
        model_bytes = slots * (N * sB + 4 + sA) + 4 * A.G + M * N * sC
        stored = slots
    else:
        for _ in range(2):                      # once per matrix and N, like the conversion
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            plan = I.insum_spmm_blockgroupcoo_plan(A, N)
            torch.cuda.synchronize()
            plan_ms = (time.perf_counter() - t0) * 1e3
        A.plans[N] = plan
        fn = lambda: I.insum_spmm_blockgroupcoo(A, B, C_out=C)
        nblk = nnz // (cfg["bM"] * cfg["bK"])
        model_bytes = nblk * (cfg["bM"] * cfg["bK"] * sA + cfg["bK"] * N * sB) + 8 * A.G * A.g + M * N * sC
        real_bytes = model_bytes
        stored = nblk
    ms = _time_launches(torch, fn, steps, warmup)
    graph_ms = _time_graph_replay(torch, fn) if ms < 0.03 else None     # launch-bound sizes only
    flops = 2.0 * nnz * N
    res = {
        "workload": name, "format": "GroupCOO" if cfg["kind"] == "group" else "BlockGroupCOO",
        "M": M, "K": cfg["K"], "N": N, "nnz": nnz, "g": A.g, "groups": A.G, "stored_units": int(stored),
        "dtype": cfg["a_dtype"], "ms_per_step": ms, "gflops": flops / ms / 1e6,
        "model_bytes": int(model_bytes), "model_gbs": model_bytes / ms / 1e6,
        "conversion_ms": conv_ms,
    }
    if plan_ms is not None:
        res["plan_ms"] = plan_ms
    if graph_ms is not None:
        res["ms_per_step_in_a_hip_graph"] = graph_ms
    b_bytes = cfg["K"] * N * sB
    if cfg["kind"] == "group":
        gbs = real_bytes / ms / 1e6
        roof = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbs / HBM_PEAK_GBS, "traffic": _traffic(name),
                "bytes_per_launch": int(real_bytes),
                "bytes_rule": "nnz*(N*sB+4+sA) + padding_slots*(4+sA) + 4*G + M*N*sC (a padding slot's "
                              "gather repeats the row just fetched and is not counted)"}
        if peaks:
            row_bytes = N * sB
            key = ("2GiB" if b_bytes > (512 << 20) else "512MiB" if b_bytes > (128 << 20) else
                   "128MiB" if b_bytes > (32 << 20) else None)       # the measured set nearest to B's size
            mp = peaks.get("random_row_read_gbs", {}).get(str(row_bytes), {}).get(key) if key else None
            if mp:
                roof["measured_peak"] = mp
                roof["frac_of_measured_peak"] = gbs / mp
                roof["measured_peak_is"] = (f"random {row_bytes}-byte row reads over a {key} set "
                                            f"(csrc/peaks.hip), the access pattern of the gather; a "
                                            f"microbenchmark of this run, repeatable to 1-2 %, so a ratio "
                                            f"slightly above 1 is within its noise - `frac` is the roofline figure")
            mix = peaks.get("row_gather_with_stores_gbs", {}).get(str(row_bytes), {}).get(key) if key else None
            if mix:
                roof["measured_mix_peak"] = mix
                roof["frac_of_measured_mix_peak"] = gbs / mix
                roof["measured_mix_peak_is"] = ("the same reads with one row written (streaming, per lane group) "
                                                "per 16 rows read: the read/write mix of this workload")
            roof["frac_of_bound"] = gbs / HBM_PEAK_GBS      # min(HBM, ALU) = HBM for a 0.5 flop/byte path
        if b_bytes <= (32 << 20):
            roof["note"] = ("B fits the 8 x 4 MiB L2: the gathers are served by the caches; bytes are "
                            "counted as if they came from memory, so this figure can exceed the HBM "
                            "peak and HBM is not what bounds this workload")
        elif b_bytes <= (256 << 20):
            roof["note"] = ("B fits the 256 MB Infinity Cache: most of these bytes cross the fabric "
                            "between L2 and that cache, not the HBM interface")
        else:
            roof["note"] = (f"B is {b_bytes >> 20} MiB against a 256 MB Infinity Cache: up to "
                            f"{min(1.0, 256e6 / b_bytes):.2f} of the gathers can still be served by that "
                            f"cache rather than by HBM itself; `traffic` counts both")
        res["roofline"] = roof
    else:
        tf = flops / ms / 1e9
        roof = {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_PEAK_TFLOPS, "traffic": _traffic(name)}
        if peaks:
            # The format fixes bM flop per gathered byte of B (a gathered tile serves the bM rows of
            # one block); B tiles that miss L2 arrive at the measured rate of L2-missing reads.
            # The rate is the one measured for random 1 KiB reads over a working set of B's size class
            # (B decides how many of the gathers hit L2).
            key = ("1MiB" if b_bytes <= (1 << 20) else "16MiB" if b_bytes <= (16 << 20) else
                   "128MiB" if b_bytes <= (128 << 20) else "2GiB")
            rate = peaks.get("random_1kib_read_gbs", {}).get(key)
            if rate:
                bound = min(MFMA_PEAK_TFLOPS, cfg["bM"] * rate / 1e3)
                roof["bound_tflops"] = bound
                roof["bound_is"] = (f"min(MFMA peak, bM = {cfg['bM']} flop/byte x {rate:.0f} GB/s of random 1 KiB "
                                    f"reads over a {key} set measured on this chip; B is {b_bytes >> 20} MiB)")
                roof["frac_of_bound"] = tf / bound
            if peaks.get("mfma_bf16_tflops"):
                roof["measured_peak"] = peaks["mfma_bf16_tflops"]
                roof["frac_of_measured_peak"] = tf / peaks["mfma_bf16_tflops"]
        res["roofline"] = roof
    return res, (cfg, A, B, C)


SPCONV = {"grid": 96, "density": 0.3, "C": 128, "M": 128, "dtype": "f16"}


def run_spconv(torch, I, steps, warmup, cloud="volume"):
    """Point-cloud sparse convolution (Section 6.4) on a synthetic voxel kernel map: 3x3x3
    stencil, 128 -> 128 channels, fp16 features and weights, fp32 output.  Timed like the SpMM
    workloads (map already grouped).  cloud = "volume": a 96^3 grid with 30 % of the voxels
    occupied independently; "surfaces": 192^3 voxels, the ones on five planes and two sphere
    shells occupied, points numbered along the Z-curve (closer to a scanned room)."""
    import synth
    c = SPCONV
    if cloud == "volume":
        P, mx, my, mz, mv = synth.voxel_kernel_map(c["grid"], c["density"], seed=0, dtype=c["dtype"])
    else:
        P, mx, my, mz, mv = synth.surface_kernel_map(192, 5, 2, seed=0, dtype=c["dtype"])
    rng = np.random.default_rng(1)
    In = _to_device(torch, synth.round_to_dtype(rng.normal(size=(P, c["C"])).astype(np.float32), c["dtype"]),
                    c["dtype"])
    W = _to_device(torch, synth.round_to_dtype((rng.normal(size=(27, c["C"], c["M"])) / 8).astype(np.float32),
                                               c["dtype"]), c["dtype"])
    dmx, dmy, dmz = (torch.from_numpy(a).cuda() for a in (mx, my, mz))
    dmv = _to_device(torch, mv, c["dtype"])
    conv_ms = None
    for _ in range(2):
        Map = None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        Map = I.insum_map_to_groupcoo(P, P, 27, dmx, dmy, dmz, dmv, g=0)
        torch.cuda.synchronize()
        conv_ms = (time.perf_counter() - t0) * 1e3
    Out = torch.empty((P, c["M"]), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(1, I.insum_spconv_groupcoo_workspace_bytes(Map, c["C"], c["M"], In.dtype)),
                     dtype=torch.uint8, device="cuda")
    ms = _time_launches(torch, lambda: I.insum_spconv_groupcoo(Map, In, W, Out=Out, workspace=ws), steps, warmup)
    ms_reuse = _time_launches(torch, lambda: I.insum_spconv_groupcoo(Map, In, W, Out=Out, workspace=ws,
                                                                     reuse_map_tables=True), steps, warmup)
    S = int(mx.shape[0])
    slots = Map.G * Map.g
    flops = 2.0 * S * c["C"] * c["M"]
    # Useful work only: 2*S*C*M.  The output-stationary schedule also multiplies the (absent)
    # zero rows of every 32-point tile, so the matrix cores execute 2 * 32*ceil(P/32) * 27 * C * M.
    executed = 2.0 * 32 * ((P + 31) // 32) * 27 * c["C"] * c["M"]
    # algorithmic bytes: every map entry gathers one input row; Out is written once; map and weights
    model_bytes = S * c["C"] * 2 + P * c["M"] * 4 + slots * (4 + 4 + 2) + 4 * Map.G + 27 * c["C"] * c["M"] * 2
    tf = flops / ms / 1e9
    return {"format": "GroupCOO along the kernel offset", "cloud": cloud, "dtype": c["dtype"], "points": P, "nnz": S,
            "C": c["C"], "M": c["M"], "g": Map.g, "groups": Map.G, "ms_per_step": ms, "tflops": tf,
            "executed_tflops": executed / ms / 1e9,
            "ms_per_step_reusing_map_tables": ms_reuse,   # later layers over the same kernel map
            "model_bytes": int(model_bytes), "model_gbs": model_bytes / ms / 1e6, "conversion_ms": conv_ms,
            "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tf / MFMA_PEAK_TFLOPS, "traffic": _traffic("spconv"),
                         "note": "ms_per_step covers the whole call (table build, weight transpose, main "
                                 "kernel); the main kernel is limited by the L1 address path and LDS "
                                 "reads, not by HBM or the matrix cores"}}


def measured_peaks():
    """Achievable rates of this chip from the library's microbenchmarks (context for the
    datasheet peaks, and the denominators of frac_of_measured_peak / frac_of_bound)."""
    import ctypes
    from paper_2510_17505_amd import _build
    lib = ctypes.CDLL(_build.PEAKS_LIB)
    for name, args in (("insum_peak_copy_gbs", [ctypes.c_size_t, ctypes.c_int]),
                       ("insum_peak_read_gbs", [ctypes.c_size_t, ctypes.c_int]),
                       ("insum_peak_random_read_gbs", [ctypes.c_size_t, ctypes.c_int]),
                       ("insum_peak_random_rows_gbs", [ctypes.c_size_t, ctypes.c_int, ctypes.c_int]),
                       ("insum_peak_gather_store_gbs", [ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int]),
                       ("insum_peak_mfma_tflops", [ctypes.c_int])):
        getattr(lib, name).restype = ctypes.c_double
        getattr(lib, name).argtypes = args
    sets = (("128MiB", 128 << 20), ("512MiB", 512 << 20), ("2GiB", 2 << 30))
    return {
        "stream_copy_gbs": lib.insum_peak_copy_gbs(2 << 30, 3),
        "stream_read_gbs": lib.insum_peak_read_gbs(2 << 30, 3),
        "random_1kib_read_gbs": {"1MiB": lib.insum_peak_random_read_gbs(1 << 20, 2),
                                 "16MiB": lib.insum_peak_random_read_gbs(16 << 20, 2),
                                 "128MiB": lib.insum_peak_random_read_gbs(128 << 20, 2),
                                 "2GiB": lib.insum_peak_random_read_gbs(2 << 30, 2)},
        "random_row_read_gbs": {str(rb): {k: lib.insum_peak_random_rows_gbs(ws, rb, 2) for k, ws in sets}
                                for rb in (256, 512)},
        # the same reads with one row written per 16 read (cfg3: 16 entries per row of C)
        "row_gather_with_stores_gbs": {str(rb): {k: lib.insum_peak_gather_store_gbs(ws, rb, 16, 2) for k, ws in sets}
                                       for rb in (256, 512)},
        "mfma_bf16_tflops": lib.insum_peak_mfma_tflops(2),
    }


def group_size_sweep(torch, I, steps, warmup):
    """Section 4.2 / 6.5 experiment on the paper's two shapes - the ablation matrix (4096 x 4096,
    90 % sparsity in 32 x 32 blocks) and the matrix of the runtime-versus-F(g) figure of Section 4.2
    (the same at 80 % sparsity) - fp16, N = 4096: time both SpMM kernels for a range of group
    sizes and report the indirect-access count F(g) and the format size next to each time, then
    what insum_choose_group_size picks by timing the default and its neighbours."""
    import synth
    M = K = N = 4096
    out = {}
    B = _to_device(torch, synth.round_to_dtype(
        np.random.default_rng(1).standard_normal((K, N)).astype(np.float32), "f16"), "f16")
    C = torch.empty((M, N), dtype=torch.float16, device="cuda")
    for label, density in (("ablation_90pct_sparse", 0.10), ("fig_runtime_vs_F_80pct_sparse", 0.20)):
        row, col, val = synth.random_block_coo(M, K, 32, 32, seed=0, dtype="f16", block_density=density,
                                               sigma=0.02)
        rd, cd = torch.from_numpy(row).cuda(), torch.from_numpy(col).cuda()
        vd = _to_device(torch, val, "f16")
        flops = 2.0 * row.size * N
        occ = np.bincount(row, minlength=M)
        occ_b = np.bincount(np.unique((row // 32).astype(np.int64) * (K // 32) + col // 32) // (K // 32),
                            minlength=M // 32)
        res = {"shape": f"4096x4096 fp16, {density:.0%} of 32x32 blocks, N=4096", "nnz": int(row.size),
               "default_g_rows": I.insum_default_group_size(int(row.size), M),
               "default_g_block_rows": I.insum_default_group_size(int(occ_b.sum()), M // 32),
               "groupcoo": [], "blockgroupcoo": []}
        for g in (1, 2, 4, 8, 16, 32, 64, 128):
            A = I.insum_coo_to_groupcoo(M, K, rd, cd, vd, g=g)
            ws = torch.empty(I.insum_spmm_groupcoo_workspace_bytes(M, N, A.G, A.g), dtype=torch.uint8, device="cuda")
            ms = _time_launches(torch, lambda: I.insum_spmm_groupcoo(A, B, C_out=C, workspace=ws), steps, warmup)
            res["groupcoo"].append({"g": g, "ms": ms, "gflops": flops / ms / 1e6,
                                    "F": I.insum_indirect_access_cost(occ.tolist(), g),
                                    "format_bytes": int(A.AM.numel() * 4 + A.AK.numel() * 4 + A.AV.numel() * 2)})
        for g in (1, 2, 4, 8, 16, 32):
            A = I.insum_coo_to_blockgroupcoo(M, K, rd, cd, vd, 32, 32, g=g)
            ms = _time_launches(torch, lambda: I.insum_spmm_blockgroupcoo(A, B, C_out=C), steps, warmup)
            res["blockgroupcoo"].append({"g": g, "ms": ms, "gflops": flops / ms / 1e6,
                                         "F": I.insum_indirect_access_cost(occ_b.tolist(), g),
                                         "format_bytes": int(A.AM.numel() * 4 + A.AK.numel() * 4 + A.AV.numel() * 2)})
        best, times = I.insum_choose_group_size(M, K, rd, cd, vd, B, C_out=C, repeats=max(3, steps))
        res["chosen_by_timing"] = {"g": best, "ms_per_candidate": times}
        out[label] = res
        del rd, cd, vd
        torch.cuda.empty_cache()
    return out


def run_transposed(torch, I, name, steps, warmup):
    """D = A^T E over the stored GroupCOO format of workload `name` (E = the shape of that
    workload's C): the derivative of the SpMM with respect to its dense operand."""
    cfg, A, B, nnz, _ = prepare(torch, I, name)
    M, K, N = cfg["M"], cfg["K"], cfg["N"]
    dt = _torch_dtype(torch, cfg["c_dtype"])
    E = torch.randn((M, N), device="cuda").to(dt)
    D = torch.empty((K, N), dtype=dt, device="cuda")
    nws = max(1, int(I.api._sgt_ws(K, N, I.api._DTYPE[dt])))
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    ms = _time_launches(torch, lambda: I.insum_spmm_groupcoo_transposed(A, E, D_out=D, workspace=ws), steps, warmup)
    s = SIZEOF[cfg["a_dtype"]]
    # one row of E per group, one read-modify-write of a row of D (fp32 sums) per real entry
    nbytes = A.G * (N * s + 4) + A.G * A.g * (4 + s) + nnz * N * 4 * 2 + K * N * s
    out = {"format": "GroupCOO (transposed product)", "dtype": cfg["a_dtype"], "nnz": nnz, "N": N, "g": A.g,
           "ms_per_step": ms, "gflops": 2.0 * nnz * N / ms / 1e6, "model_gbs": nbytes / ms / 1e6,
           "atomic_adds_per_s": nnz * N / ms * 1e3,
           "note": "scatter with hardware fp32 atomic adds; bounded by the rate at which the L2 completes them"}
    # The other route to the same product, for a matrix that is used many times (training): a
    # second GroupCOO copy holding A^T (insum_groupcoo_transpose: built once from the format), then
    # the ordinary SpMM - no atomics, a fixed summation order.
    del ws
    conv_ms = None
    for _ in range(2):
        At = None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        At = I.insum_groupcoo_transpose(A)
        torch.cuda.synchronize()
        conv_ms = (time.perf_counter() - t0) * 1e3
    del A
    ws = torch.empty(max(1, I.insum_spmm_groupcoo_workspace_bytes(K, N, At.G, At.g)), dtype=torch.uint8, device="cuda")
    ms2 = _time_launches(torch, lambda: I.insum_spmm_groupcoo(At, E, C_out=D, workspace=ws), steps, warmup)
    out["via_second_copy_of_A_transposed"] = {"transpose_ms": conv_ms, "g": At.g, "ms_per_step": ms2,
                                              "gflops": 2.0 * nnz * N / ms2 / 1e6}
    return out


def tail_cases(torch, I, steps, warmup):
    """Two GroupCOO inputs that stress the parts of the SpMM outside its main loop, each timed
    next to the time its bytes would take at the rate the same run measures on cfg3:
    `hub`: rank-size row lengths (131072, 65536, ... entries: single rows span hundreds of work
    ranges, whose partial sums the second kernel adds); `gaps`: 2^20 rows, nonzeros only in the
    first and the last 1 % of them (98 % of C is zero-fill of rows without groups)."""
    N, out = 128, {}
    ref, _ = run_workload(torch, I, "cfg3", steps, warmup)
    rate = ref["roofline"]["achieved"]                       # GB/s of real-entry bytes on cfg3
    rng = np.random.default_rng(7)
    cases = {}
    M, K = 4096, 1 << 18
    occ = np.minimum((K // 2) // np.arange(1, M + 1), K // 2).astype(np.int64)
    occ[64:] = rng.integers(0, 4, M - 64)
    row = np.repeat(np.arange(M, dtype=np.int32), occ)
    col = np.concatenate([rng.choice(K, size=int(k), replace=False) for k in occ]).astype(np.int32)
    cases["hub"] = (M, K, row, col)
    M = K = 1 << 20
    n = 8_000_000
    r = rng.integers(0, M // 100, n)
    r[n // 2:] = M - 1 - r[n // 2:]
    cases["gaps"] = (M, K, r.astype(np.int32), rng.integers(0, K, n).astype(np.int32))
    for name, (M, K, row, col) in cases.items():
        val = torch.randn(row.size, device="cuda")
        A = I.insum_coo_to_groupcoo(M, K, torch.from_numpy(row).cuda(), torch.from_numpy(col).cuda(), val, g=4)
        B = torch.randn((K, N), device="cuda")
        C = torch.empty((M, N), device="cuda")
        ws = torch.empty(I.insum_spmm_groupcoo_workspace_bytes(M, N, A.G, A.g), dtype=torch.uint8, device="cuda")
        ms = _time_launches(torch, lambda: I.insum_spmm_groupcoo(A, B, C_out=C, workspace=ws), steps, warmup)
        nnz, slots = int(row.size), A.G * A.g
        nbytes = nnz * (N * 4 + 8) + (slots - nnz) * 8 + 4 * A.G + M * N * 4
        out[name] = {"M": M, "K": K, "N": N, "nnz": nnz, "ms": ms, "bytes": int(nbytes),
                     "ms_at_cfg3_rate": nbytes / rate / 1e6, "ratio": ms / (nbytes / rate / 1e6)}
        del A, B, C, ws
        torch.cuda.empty_cache()
    out["cfg3_rate_gbs"] = rate
    return out


def width_sweep(torch, I, steps, warmup):
    """GroupCOO SpMM on the cfg3 matrix for dense widths N = 8 ... 256 in fp32 and fp16: how the
    gather-bound kernel behaves from 16-byte to 1 KiB rows of B."""
    import synth
    cfg = synth.make_config("cfg3")
    M, K = cfg["M"], cfg["K"]
    A32 = I.insum_coo_to_groupcoo(M, K, torch.from_numpy(cfg["row"]).cuda(), torch.from_numpy(cfg["col"]).cuda(),
                                  torch.from_numpy(cfg["val"]).cuda(), g=0)
    nnz = int(cfg["row"].size)
    out = []
    for name, dt, es in (("f32", torch.float32, 4), ("f16", torch.float16, 2)):
        A = A32 if es == 4 else I.GroupCOO(A32.M, A32.K, A32.g, A32.AM, A32.AK, A32.AV.half())
        for N in (8, 16, 32, 64, 128, 256):
            B = torch.randn((K, N), device="cuda").to(dt)
            C = torch.empty((M, N), dtype=dt, device="cuda")
            ws = torch.empty(I.insum_spmm_groupcoo_workspace_bytes(M, N, A.G, A.g), dtype=torch.uint8,
                             device="cuda")
            ms = _time_launches(torch, lambda: I.insum_spmm_groupcoo(A, B, C_out=C, workspace=ws), steps, warmup)
            model = A.G * A.g * (N * es + 4 + es) + 4 * A.G + M * N * es
            out.append({"dtype": name, "N": N, "row_bytes": N * es, "ms": ms, "gflops": 2.0 * nnz * N / ms / 1e6,
                        "model_gbs": model / ms / 1e6, "gathers_per_s": A.G * A.g / ms * 1e3})
            del B, C, ws
    return out


def vendor_context(torch, I, steps, warmup):
    """Context only (not part of the library): the vendor SpMM that PyTorch dispatches to
    (rocSPARSE CSR) on cfg3 and cfg2, and the dense GEMM (hipBLASLt) on the sweep shape - the
    MI355X analogues of the cuSPARSE and dense-matmul comparisons in Section 6.2 / 6.3."""
    import synth
    out = {}
    for name in ("cfg3", "cfg2"):
        cfg = synth.make_config(name)
        M, K, N = cfg["M"], cfg["K"], cfg["N"]
        dt = _torch_dtype(torch, cfg["a_dtype"])
        order = np.lexsort((cfg["col"], cfg["row"]))
        crow = np.concatenate([[0], np.cumsum(np.bincount(cfg["row"], minlength=M))]).astype(np.int64)
        try:
            A = torch.sparse_csr_tensor(torch.from_numpy(crow).cuda(),
                                        torch.from_numpy(cfg["col"][order].astype(np.int64)).cuda(),
                                        _to_device(torch, cfg["val"][order], cfg["a_dtype"]), size=(M, K))
            B = _to_device(torch, cfg["B"], cfg["b_dtype"])
            ms = _time_launches(torch, lambda: torch.sparse.mm(A, B), steps, warmup)
            out[name] = {"library": "torch.sparse.mm on a CSR tensor (rocSPARSE)", "dtype": str(dt),
                         "ms": ms, "gflops": 2.0 * cfg["row"].size * N / ms / 1e6}
            del A, B
        except Exception as e:      # context only: report and go on
            out[name] = {"error": f"{type(e).__name__}: {e}"[:200]}
        torch.cuda.empty_cache()
    a = torch.randn((4096, 4096), dtype=torch.float16, device="cuda")
    b = torch.randn((4096, 4096), dtype=torch.float16, device="cuda")
    ms = _time_launches(torch, lambda: torch.matmul(a, b), steps, warmup)
    out["dense_4096_f16"] = {"library": "torch.matmul (hipBLASLt)", "ms": ms,
                             "tflops": 2.0 * 4096 ** 3 / ms / 1e9}
    # Section 6.2 asks at which sparsity the block-sparse product beats the dense one: the same
    # 4096^2 fp16 matrix in 32x32 blocks at several block densities, N = 4096.
    sweep = []
    for density in (0.05, 0.1, 0.2, 0.3, 0.4, 0.5, 0.75, 1.0):
        row, col, val = synth.random_block_coo(4096, 4096, 32, 32, seed=0, dtype="f16", block_density=density)
        A = I.insum_coo_to_blockgroupcoo(4096, 4096, torch.from_numpy(row).cuda(), torch.from_numpy(col).cuda(),
                                         _to_device(torch, val, "f16"), 32, 32, g=0)
        C = torch.empty((4096, 4096), dtype=torch.float16, device="cuda")
        t = _time_launches(torch, lambda: I.insum_spmm_blockgroupcoo(A, b, C_out=C), steps, warmup)
        sweep.append({"block_density": density, "g": A.g, "ms": t, "dense_ms_over_ms": ms / t})
        del A, C
    out["block_density_sweep_4096_f16"] = sweep
    return out


def cpu_baseline(cfg, A, nnz_total):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import oracle
    from oracle import bf16_bits_to_f32
    N = cfg["N"]
    budget_fma = 3.0e10                         # bounds the oracle run to some tens of seconds
    AM = A.AM.cpu().numpy()
    G = AM.shape[0]
    if cfg["kind"] == "group":
        per_group = A.g * N
    else:
        per_group = A.g * cfg["bM"] * cfg["bK"] * N
    Gs = int(min(G, max(1, budget_fma // per_group)))
    AMs = AM[:Gs]
    AKs = A.AK[:Gs].cpu().numpy()
    AVt = A.AV[:Gs].cpu()
    if cfg["a_dtype"] == "bf16":
        import torch
        AVs = bf16_bits_to_f32(AVt.view(torch.int16).numpy().view(np.uint16))
    else:
        AVs = AVt.numpy().astype(np.float32)
    B = cfg["B"]
    real = int(np.count_nonzero(AVs))           # padding holds exact zeros; values are nonzero
    dt = float("inf")
    for _ in range(4):                          # one warm-up, best of three
        t0 = time.perf_counter()
        if cfg["kind"] == "group":
            oracle.spmm_groupcoo(cfg["M"], cfg["K"], N, AMs, AKs, AVs, B)
        else:
            oracle.spmm_blockgroupcoo(cfg["M"], cfg["K"], N, cfg["bM"], cfg["bK"], AMs, AKs, AVs, B)
        dt = min(dt, time.perf_counter() - t0)
    return {"value": 2.0 * real * N / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": dt,
            "sample": f"first {Gs} of {G} groups of {cfg['name']} ({real} nonzeros of {nnz_total}), "
                      f"fp64 loops, best of 3 after a warm-up, includes zero-initialising the full C"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-peaks", action="store_true",
                    help="skip the achievable-peak microbenchmarks (and the fractions that use them)")
    ap.add_argument("--sweep", action="store_true",
                    help="only run the group-size sweep on the paper's ablation shape")
    ap.add_argument("--context", action="store_true",
                    help="only time the vendor libraries PyTorch dispatches to (context, not product)")
    ap.add_argument("--width-sweep", action="store_true",
                    help="only run the GroupCOO SpMM of cfg3 for N = 8 ... 256 in fp32 and fp16")
    ap.add_argument("--tails", action="store_true",
                    help="only time the hub-row and empty-row-gap inputs of the GroupCOO SpMM")
    ap.add_argument("--spconv", action="store_true",
                    help="only time the sparse-convolution workload (Section 6.4)")
    ap.add_argument("--spconv-surfaces", action="store_true",
                    help="only time the sparse convolution on the surface-like point cloud")
    ap.add_argument("--peaks", action="store_true", help="only run the achievable-peak microbenchmarks")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run a plain elementwise copy of MIB mebibytes (read MIB, write MIB) "
                         "--steps times: the known-size kernel that scales the HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.calibrate_copy:
        n = args.calibrate_copy * (1 << 20) // 4
        x = torch.ones(n, dtype=torch.float32, device="cuda")
        y = torch.empty_like(x)
        ms = _time_launches(torch, lambda: torch.mul(x, 1.0, out=y), args.steps, args.warmup)
        print(json.dumps({"calibrate_copy_mib": args.calibrate_copy, "ms_per_step": ms,
                          "copy_gbs": 2.0 * n * 4 / ms / 1e6}))
        return
    import paper_2510_17505_amd as I

    if args.peaks:
        print(json.dumps({"measured_peaks": measured_peaks()}))
        return
    if args.context:
        print(json.dumps({"vendor_context": vendor_context(torch, I, args.steps, args.warmup)}))
        return
    if args.tails:
        print(json.dumps({"tail_cases": tail_cases(torch, I, args.steps, args.warmup)}))
        return
    if args.width_sweep:
        print(json.dumps({"width_sweep": width_sweep(torch, I, args.steps, args.warmup)}))
        return
    if args.spconv:
        print(json.dumps({"spconv": run_spconv(torch, I, args.steps, args.warmup)}))
        return
    if args.spconv_surfaces:
        print(json.dumps({"spconv_surfaces": run_spconv(torch, I, args.steps, args.warmup, cloud="surfaces")}))
        return
    if args.sweep:
        print(json.dumps({"group_size_sweep": group_size_sweep(torch, I, args.steps, args.warmup)}))
        return
    peaks = None if args.no_peaks else measured_peaks()
    res, (cfg, A, B, C) = run_workload(torch, I, args.workload, args.steps, args.warmup, peaks)
    line = {
        "metric": "SpMM GFLOP/s (2*nnz*N)", "value": res["gflops"], "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["a_dtype"], "data": "synthetic",
        "config": {"workload": f"{args.workload}: {res['format']} SpMM, A {cfg['M']}x{cfg['K']} "
                               f"{cfg['a_dtype']} nnz={res['nnz']} g={res['g']}, B {cfg['K']}x{cfg['N']}",
                   "format": res["format"], "g": res["g"], "groups": res["groups"]},
        "roofline": res["roofline"],
        "model_bytes_per_launch": res["model_bytes"],
        "model_gbs": res["model_gbs"],
        "conversion_ms": res["conversion_ms"],
    }
    for key in ("plan_ms", "ms_per_step_in_a_hip_graph"):
        if key in res:
            line[key] = res[key]
    if cfg["kind"] == "group":
        ws = torch.empty(I.insum_spmm_groupcoo_workspace_bytes(cfg["M"], cfg["N"], A.G, A.g), dtype=torch.uint8,
                         device="cuda")
        line["launch_statistics"] = launch_statistics(
            torch, lambda: I.insum_spmm_groupcoo(A, B, C_out=C, workspace=ws))
        del ws
    else:
        line["launch_statistics"] = launch_statistics(torch, lambda: I.insum_spmm_blockgroupcoo(A, B, C_out=C))
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(cfg, A, res["nnz"])
    del A, B, C, cfg
    torch.cuda.empty_cache()
    if not args.no_extra:
        others = {}
        for name in ("cfg3_f16", "cfg5", "cfg4", "cfg2", "cfg1"):
            if name == args.workload:
                continue
            r, keep = run_workload(torch, I, name, args.steps, args.warmup, peaks)
            del keep
            torch.cuda.empty_cache()
            others[name] = {k: r[k] for k in ("format", "dtype", "nnz", "N", "g", "ms_per_step", "gflops",
                                              "model_gbs", "roofline", "conversion_ms", "plan_ms",
                                              "ms_per_step_in_a_hip_graph") if k in r}
        for name in ("cfg3", "cfg2"):
            others[name + "_transposed"] = run_transposed(torch, I, name, args.steps, args.warmup)
            torch.cuda.empty_cache()
        others["spconv"] = run_spconv(torch, I, args.steps, args.warmup)
        line["other_workloads"] = others
    if peaks is not None:
        line["measured_peaks"] = peaks
    print(json.dumps(line))


if __name__ == "__main__":
    main()
