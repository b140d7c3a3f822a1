#!/usr/bin/env python3
"""Benchmark of the sparse-convolution hot path on one MI355X.

One step = one whole layer on synthetic input already resident in HBM:
sc_hash_build -> sc_kmap_build -> sc_conv_fwd (kernel map construction included).
Prints ONE JSON line.  The headline (`value`, `ms_per_step`) is the largest single-GPU workload,
cfg5 (~10^6 voxels, 128 -> 128 channels, fp16): effective TFLOP/s over active MACs
(2*P*C_in*C_out / time per layer).  The same line carries, under "target64", the same
measurements for the ~110k-voxel 64 -> 64 layer; for each: the per-phase split, per-kernel
durations (HIP events stamped with every dispatch's begin and end, on the launch's stream) with
their fractions of the HBM and matrix-core peaks, the roofline of the convolution kernel, and the
cold first layer (table fill included).  The CPU oracle is timed on this host's cores on a sample
of the headline workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|target64|cfg4|cfg2|cfg3|cfg3k3|cfg1|cfg2-stage|cfg3-inverse] [--table hash|grid|fused]
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

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_MFMA_TFLOPS = 2500.0      # dense fp16 / bf16 MFMA
PEAK_FP32_TFLOPS = 157.3       # fp32 vector ALU


def algorithmic_bytes(kernel: str, st: dict) -> float | None:
    """Bytes one launch of `kernel` has to move by the method's own accounting: a per-unit figure
    (the comment on each case below) times the units one launch processes."""
    N, N_out, P, K3, cap = st["N"], st["N_out"], st["P"], st["K3"], st["cap"]
    C_in, C_out, e = st["C_in"], st["C_out"], st["elem_bytes"]
    if kernel == "k_table_fill":
        return 16.0 * cap                                  # every 16-byte slot written once
    if kernel == "k_hash_insert":
        return N * (16 + 8 + 8 + 4)                       # coords, key compare-and-swap (read + write), row index
    if kernel == "k_kmap_subm":
        # coords, one 8-byte key per neighbour probe, 4 bytes per hit, one 4-byte table cell per (row, offset)
        return N * 16 + N * (K3 - 1) * 8 + (P - N) * 4 + N * K3 * 4
    if kernel == "k_grid_insert":
        return N * (16 + 8 + 8)                           # coords, one 8-byte cell exchanged (read + write)
    if kernel == "k_kmap_subm_grid":
        # coords, one 8-byte cell per neighbour probe, one 4-byte table cell per (row, offset)
        return N * 16 + N * (K3 - 1) * 8 + N * K3 * 4
    if kernel in ("k_conv_mfma", "k_conv_f32"):
        # features in once, features out once, weights once, 8 bytes of map per pair
        return N * C_in * e + N_out * C_out * e + K3 * C_in * C_out * e + P * 8
    if kernel == "k_strided_fill":
        return 16.0 * cap + N * K3 * 4.0
    if kernel == "k_strided_insert":
        return N * (16 + 8 + 8 + 4 + 4)
    if kernel == "k_strided_pairs":
        return N * (16 + 4 + 16 + 4 + 4 + 8 + 4) + N_out * 16
    if kernel == "k_masks_from_table":
        return N_out * K3 * 4.0
    return None


def stage_bench(args, torch, sc, synth) -> int:
    """Three chained layers on the cfg2 voxel set, the way an encoder stage runs them: two
    submanifold 3x3x3 layers (32->32) that share ONE location table and ONE kernel map, then a
    strided 2x2x2 layer (32->64) with its own map.  One step = all three; reports the amortised
    time per layer."""
    dev = "cuda:0"
    cfg = synth.make_config("cfg2")
    coords = cfg["coords"]
    N = len(coords)
    d_coords = torch.from_numpy(coords).to(dev)
    d_feat = torch.from_numpy(cfg["feat"]).to(dev).half().contiguous()
    w1 = torch.from_numpy(synth.weights(27, 32, 32, "f16", 1)).to(dev).half()
    w2 = torch.from_numpy(synth.weights(27, 32, 32, "f16", 2)).to(dev).half()
    w3 = torch.from_numpy(synth.weights(8, 32, 64, "f16", 3)).to(dev).half()
    subm = sc.LayerBuffers(N, 3, 1, "subm", 32, 32, "f16", device=dev)
    down = sc.LayerBuffers(N, 2, 2, "strided", 32, 64, "f16", device=dev)
    mid = torch.empty((N, 32), dtype=torch.float16, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        subm.hash_build(d_coords, stream)
        subm.kmap_build(d_coords, stream)
        subm.conv_fwd(d_feat, w1, stream)                                   # layer 1 -> subm.feat_out
        sc.sc_conv_fwd(subm.feat_out, w2, mid, subm.kmap, subm.counts, 3, 1, "subm", subm.workspace, stream)
        down.kmap_build(d_coords, stream, standalone=True)                  # a strided layer needs no input table
        down.conv_fwd(mid, w3, stream)

    step()
    P1 = int(subm.read_counts().n_pairs)
    hd = down.read_counts()
    flops = 2.0 * (2 * P1 * 32 * 32 + int(hd.n_pairs) * 32 * 64)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    sc.sc_profile_enable(True)
    for _ in range(args.steps):
        step()
    prof = sc.sc_profile_read()
    sc.sc_profile_enable(False)
    print(json.dumps({
        "metric": "effective TFLOP/s over active MACs, three chained layers incl. their kernel maps",
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "ms_per_layer_amortised": ms / 3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "cfg2-stage: subm 32->32, subm 32->32 (shared table and map), strided K=2 32->64",
                   "N": N, "N_out_strided": int(hd.n_out), "P_subm": P1, "P_strided": int(hd.n_pairs)},
        "kernels": {k: {"launches_per_step": l / args.steps, "avg_us": round(1e3 * t / l, 3), "median_us": round(1e3 * m, 3)}
                    for k, (l, t, m) in prof.items()},
    }))
    return 0


def inverse_bench(args, torch, sc, synth) -> int:
    """The up-sampling layer that undoes cfg3's down-sampling (Section III-E): coarse rows with 64
    channels -> the cfg2 voxel set with 32 channels, K = stride = 2.  The strided map exists
    already (the encoder built it); one step = transposing it (sc_kmap_transpose) + the
    convolution over the transposed map."""
    dev = "cuda:0"
    cfg = synth.make_config("cfg3")
    coords = cfg["coords"]
    N = len(coords)
    d_coords = torch.from_numpy(coords).to(dev)
    down = sc.LayerBuffers(N, 2, 2, "strided", 32, 64, "f16", device=dev)
    down.kmap_build(d_coords, standalone=True)
    n_c = int(down.read_counts().n_out)
    feat_c = torch.from_numpy(synth.features(n_c, 64, "f16", 11)).to(dev).half().contiguous()
    w = torch.from_numpy(synth.weights(8, 64, 32, "f16", 11)).to(dev).half().contiguous()
    kmap_inv = torch.empty(sc.sc_kmap_bytes(N, 2, 2, "inverse"), dtype=torch.uint8, device=dev)
    out = torch.empty((N, 32), dtype=torch.float16, device=dev)
    ws = torch.empty(max(sc.sc_conv_workspace_bytes(2, 64, 32, "f16"), 16), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        sc.sc_kmap_transpose(down.kmap, N, 2, 2, down.counts, kmap_inv, stream)
        sc.sc_conv_fwd(feat_c, w, out, kmap_inv, down.counts, 2, 2, "inverse", ws, stream, n_map=N)

    step()
    P = int(sc.sc_counts_read(down.counts, kmap_inv, N, 2, 2, "inverse").n_pairs)
    flops = 2.0 * P * 64 * 32
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    sc.sc_profile_enable(True)
    for _ in range(args.steps):
        step()
    prof = sc.sc_profile_read()
    sc.sc_profile_enable(False)
    # the same layer straight from the strided map (sc_conv_up_fwd): no transposed map at all
    out2 = torch.empty_like(out)

    def step_direct():
        sc.sc_conv_up_fwd(feat_c, N, w, out2, down.kmap, down.counts, 2, stream)

    for _ in range(args.warmup):
        step_direct()
    torch.cuda.synchronize()
    if not torch.equal(out, out2):
        raise RuntimeError("sc_conv_up_fwd and the transposed map give different layers")
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_direct()
    torch.cuda.synchronize()
    ms_direct = (time.perf_counter() - t0) * 1e3 / args.steps
    print(json.dumps({
        "metric": "effective TFLOP/s over active MACs, inverse layer incl. transposing the strided map",
        "direct_from_strided_map": {"ms_per_step": ms_direct, "value": flops / (ms_direct * 1e-3) / 1e12, "unit": "TFLOP/s"},
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "cfg3-inverse: K=2 stride 2 up-sampling 64->32 onto the cfg2 voxel set",
                   "N_coarse": n_c, "N_fine": N, "P": P},
        "kernels": {k: {"launches_per_step": l / args.steps, "avg_us": round(1e3 * t / l, 3), "median_us": round(1e3 * m, 3)}
                    for k, (l, t, m) in prof.items()},
    }))
    return 0


def host_cpu() -> dict:
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"model": model, "logical_cpus": os.cpu_count()}


def measured_peaks(torch, sc, dev) -> dict:
    """What this GPU sustains on a plain 1 GiB device copy (read + write bytes per second) and on a
    register-operand fp16 MFMA loop: the measured counterparts of the published peaks."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(10):
        dst.copy_(src)
    ev[1].record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * n * 10 / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
    del src, dst
    return {"copy_gbs": copy_gbs, "mfma_f16_tflops": sc.sc_profile_mfma_peak()}


def measure_layer(args, torch, sc, synth, workload: str, steps: int, warmup: int, peaks: dict,
                  others: bool, cpu_baseline: bool) -> dict:
    """One workload, whole layers: returns the record (see the module docstring)."""
    dev = "cuda:0"
    cfg = synth.make_config(workload)
    coords, K, stride, mode = cfg["coords"], cfg["K"], cfg["stride"], cfg["mode"]
    C_in, C_out, dtype = cfg["C_in"], cfg["C_out"], cfg["dtype"]
    N = len(coords)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]
    d_coords = torch.from_numpy(coords).to(dev)
    d_feat = torch.from_numpy(cfg["feat"]).to(dev).to(tdt).contiguous()
    d_w = torch.from_numpy(cfg["weight"]).to(dev).to(tdt).contiguous()
    if args.table != "hash" and mode != "subm":
        raise SystemExit("bench.py: --table grid applies to submanifold workloads only")
    buf = sc.LayerBuffers(N, K, stride, mode, C_in, C_out, dtype, device=dev,
                          grid_dims=cfg["box"] if args.table != "hash" else None)
    stream = torch.cuda.current_stream()
    # the weights of a layer do not change from frame to frame: packed once, outside the timed region
    # (sc_conv_weight_pack); the fused dense-table layer takes raw weights and re-lays them out itself
    d_wp = sc.sc_conv_weight_pack(d_w, K, stream=stream)

    def step():
        if args.table == "fused":
            buf.layer_fused(d_coords, d_feat, d_w, stream)
            return
        if mode == "strided":
            # a strided layer looks nothing up in an input table (Section III-D builds the output side
            # only): its step is map build + convolution; sc_hash_build would only add the check for
            # repeated input coordinates
            buf.kmap_build(d_coords, stream, standalone=True)
        else:
            buf.hash_build(d_coords, stream)
            buf.kmap_build(d_coords, stream)
        buf.conv_fwd_packed(d_feat, d_wp, stream)

    step()
    if args.table == "fused":
        buf.kmap_build(d_coords, stream)          # once, outside the timed region: only to count the pairs
    h = buf.read_counts()
    if h.status != 0:
        raise RuntimeError(f"device status {h.status}")
    P, N_out = int(h.n_pairs), int(h.n_out)
    flops = 2.0 * P * C_in * C_out

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # The step is a fixed sequence of kernel launches on one stream, so it can be replayed from a
    # HIP graph: same kernels, same work, without the per-launch host cost.
    graph = None
    if args.graph != "off":
        try:
            gstream = torch.cuda.Stream()
            gstream.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(gstream):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=gstream):
                    if args.table == "fused":
                        buf.layer_fused(d_coords, d_feat, d_w, gstream)
                    else:
                        if mode == "strided":
                            buf.kmap_build(d_coords, gstream, standalone=True)
                        else:
                            # a replay repeats the captured arguments, epoch included: the hash
                            # table is captured with its full build (fill + insert); the dense
                            # table's build is idempotent for one coordinate set and epoch
                            if buf.grid_dims is None:
                                sc.sc_hash_build(d_coords, buf.table, buf.counts, gstream)
                            else:
                                buf.hash_build(d_coords, gstream)
                            buf.kmap_build(d_coords, gstream)
                        buf.conv_fwd_packed(d_feat, d_wp, gstream)
            torch.cuda.synchronize()
            ref = buf.feat_out[:N_out].clone()
            buf.feat_out.zero_()
            g.replay()
            torch.cuda.synchronize()
            if not torch.equal(ref, buf.feat_out[:N_out]):
                raise RuntimeError("graph replay differs from the eager step")
            graph = g
        except Exception as exc:                                    # noqa: BLE001
            if args.graph == "on":
                raise
            print(f"bench.py: graph capture unavailable ({exc}); timing eager launches", file=sys.stderr)
            torch.cuda.synchronize()

    def timed_step():
        if graph is not None:
            graph.replay()
        else:
            step()

    for _ in range(warmup):
        timed_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        timed_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    value = flops / (ms_per_step * 1e-3) / 1e12

    # the cold layer: the step a caller pays on a table that has not been built before (sc_hash_build:
    # every slot filled, then the inserts); the timed steps above reuse the table (sc_hash_rebuild)
    cold = []
    for _ in range(5):
        buf.forget_table()                      # the next build fills the table
        ev_cold = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev_cold[0].record(stream)
        step()
        ev_cold[1].record(stream)
        torch.cuda.synchronize()
        cold.append(ev_cold[0].elapsed_time(ev_cold[1]))
    cold_ms = float(np.median(cold))

    # per-phase split with torch events (the library launches on torch's current stream)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for i in range(steps):
        ev[i][0].record(stream)
        if mode != "strided":
            buf.hash_build(d_coords, stream)
        ev[i][1].record(stream)
        if args.table != "fused":
            buf.kmap_build(d_coords, stream, standalone=(mode == "strided"))
        ev[i][2].record(stream)
        if args.table == "fused":
            sc.sc_conv_fwd_grid(d_feat, d_coords, buf.table, buf.grid_dims, buf.epoch, d_w, buf.feat_out, K,
                                buf.workspace, stream)
        else:
            buf.conv_fwd_packed(d_feat, d_wp, stream)
        ev[i][3].record(stream)
    torch.cuda.synchronize()
    phases = {name: float(np.median([e[j].elapsed_time(e[j + 1]) for e in ev]))
              for j, name in enumerate(["hash_ms", "kmap_ms", "conv_ms"])}

    # per-kernel durations: every launch carries a pair of HIP events stamped with the dispatch's
    # begin and end (hipExtLaunchKernelGGL inside the library), over the same number of steps; the
    # median of a kernel's launches is what the fractions below are computed from
    sc.sc_profile_enable(True)
    for _ in range(steps):
        step()
    prof = sc.sc_profile_read()
    sc.sc_profile_enable(False)
    st = dict(N=N, N_out=N_out, P=P, K3=K ** 3, cap=(sc.sc_hash_bytes(N) - 256) // 16, C_in=C_in, C_out=C_out,
              elem_bytes=d_feat.element_size())
    traffic_table = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
    if os.path.exists(tpath):
        key = workload if args.table == "hash" else f"{workload}-{args.table}"
        traffic_table = json.load(open(tpath)).get(key, {})
    conv_peak = PEAK_MFMA_TFLOPS if dtype != "f32" else PEAK_FP32_TFLOPS
    per_kernel = {}
    for name, (launches, total_ms, median_ms) in prof.items():
        med_s = median_ms * 1e-3
        rec = {"launches_per_step": launches / steps, "median_us": round(median_ms * 1e3, 3),
               "avg_us": round(total_ms * 1e3 / launches, 3)}
        ab = algorithmic_bytes(name, st)
        if ab:
            rec["algorithmic_bytes"] = int(ab)
            rec["hbm_gbs_algorithmic"] = round(ab / med_s / 1e9, 1)
            rec["frac_of_hbm_peak"] = round(ab / med_s / 1e9 / PEAK_HBM_GBS, 4)
            rec["frac_of_measured_copy"] = round(ab / med_s / 1e9 / peaks["copy_gbs"], 4)
        if name in traffic_table:
            rec["hbm_bytes_counters"] = traffic_table[name]
        if name in ("k_conv_mfma", "k_conv_f32"):
            rec["tflops_active"] = round(flops / med_s / 1e12, 2)
            rec["frac_of_mfma_peak" if name == "k_conv_mfma" else "frac_of_fp32_peak"] = round(flops / med_s / 1e12 / conv_peak, 4)
            if name == "k_conv_mfma":
                rec["frac_of_measured_mfma"] = round(flops / med_s / 1e12 / peaks["mfma_f16_tflops"], 4)
        per_kernel[name] = rec
    sum_kernels_us = sum(r["median_us"] * r["launches_per_step"] for r in per_kernel.values())

    # roofline of the convolution kernel (the largest share of every step).  Which roof it is under:
    # its flops per algorithmic byte against the machine balance (peak flops / peak bytes); layers
    # of 32 and 64 channels sit under the HBM roof, 128 channels under the matrix-core roof.
    conv_name = "k_conv_mfma" if "k_conv_mfma" in per_kernel else "k_conv_f32"
    conv_s = per_kernel[conv_name]["median_us"] * 1e-6
    conv_bytes = algorithmic_bytes(conv_name, st)
    conv_under_hbm = flops / conv_bytes * PEAK_HBM_GBS * 1e9 < conv_peak * 1e12
    if conv_under_hbm:
        achieved = conv_bytes / conv_s / 1e9
        roofline = {"kernel": conv_name, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": traffic_table.get(conv_name),
                    "median_us": conv_s * 1e6, "flops_per_algorithmic_byte": flops / conv_bytes,
                    "tflops_active": flops / conv_s / 1e12, "frac_of_mfma_peak": flops / conv_s / 1e12 / conv_peak}
    else:
        achieved = flops / conv_s / 1e12
        roofline = {"kernel": conv_name, "bound": "mfma" if conv_name == "k_conv_mfma" else "alu", "achieved": achieved,
                    "peak": conv_peak, "unit": "TFLOP/s", "frac": achieved / conv_peak,
                    "traffic": traffic_table.get(conv_name), "median_us": conv_s * 1e6,
                    "hbm_gbs_algorithmic": conv_bytes / conv_s / 1e9}

    out = {
        "value": value, "unit": "TFLOP/s", "ms_per_step": ms_per_step, "dtype": dtype,
        "config": {"workload": workload, "table": args.table, "mode": mode, "K": K, "stride": stride, "C_in": C_in,
                   "C_out": C_out, "N": N, "N_out": N_out, "P": P, "pairs_per_voxel": P / max(N, 1)},
        "launch": "hip graph replay" if graph is not None else "eager",
        "table_reuse": ("strided step: no input table" if mode == "strided" else
                        "dense table, epoch per build" if args.table != "hash" else
                        "steps after the first call sc_hash_rebuild (no fill) when the table has at most 2^22 slots"),
        "cold_first_layer_ms": cold_ms,
        "phases_ms": phases, "kernels": per_kernel, "sum_of_kernel_medians_us": round(sum_kernels_us, 2),
        "roofline": roofline,
    }

    # Multiplies issued against multiplies that exist.  The matrix kernels keep an output row in its
    # place and skip a group of rows at an offset only if none of its rows has a neighbour there:
    # 16 rows (v_mfma 16x16x32: k_conv_rows16, k_conv_stream) or 32 rows (32x32x16: k_conv_direct64).
    # Counted from the exported pair lists, outside the timed region.
    if conv_name == "k_conv_mfma" and args.table != "fused" and P > 0:
        _, p_out, ost = sc.sc_kmap_export(buf.kmap, N, K, stride, mode, h, stream)
        k_of = torch.bucketize(torch.arange(P, device=dev, dtype=torch.int32), ost[1:].contiguous(), right=True)
        issued = {}
        for rows, shift in ((16, 4), (32, 5)):
            groups = torch.unique((p_out.long() >> shift) * (K ** 3) + k_of.long()).numel()
            issued[f"groups_of_{rows}_rows"] = round(groups * rows / P, 3)
        out["kernels"][conv_name]["multiplies_issued_over_active"] = issued
        del p_out, ost, k_of

    # the same layer with the other location tables (same checks: the outputs must be identical),
    # for comparison: "grid" = dense array + kernel map, "fused" = dense array, look-ups inside the
    # convolution, no kernel map (3x3x3 16-bit layers with a dedicated kernel only)
    if others and mode == "subm":
        rows = []
        fused_ok = K == 3 and dtype != "f32" and (C_in, C_out) in ((32, 32), (64, 64), (128, 128), (32, 64), (64, 128))
        for other in ("hash", "grid", "fused"):
            if other == args.table or (other == "fused" and not fused_ok):
                continue
            buf2 = sc.LayerBuffers(N, K, stride, mode, C_in, C_out, dtype, device=dev,
                                   grid_dims=cfg["box"] if other != "hash" else None)

            def step2():
                if other == "fused":
                    buf2.layer_fused(d_coords, d_feat, d_w, stream)
                else:
                    buf2.hash_build(d_coords, stream)
                    buf2.kmap_build(d_coords, stream)
                    buf2.conv_fwd_packed(d_feat, d_wp, stream)

            for _ in range(warmup + 1):
                step2()
            # the same kernels give the same bits; where the variants run different kernels (the
            # 64-channel layer) they sum in another order and may differ in the last place
            a, b = buf2.feat_out[:N_out].float(), buf.feat_out[:N_out].float()
            if not torch.equal(a, b) and float((a - b).abs().max() / b.abs().max()) > 2e-3:
                raise RuntimeError(f"location table '{other}' gives a different layer")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                step2()
            torch.cuda.synchronize()
            ms2 = (time.perf_counter() - t0) * 1e3 / steps
            rows.append({"table": other, "ms_per_step": ms2, "value": flops / (ms2 * 1e-3) / 1e12, "unit": "TFLOP/s"})
            del buf2
        out["other_tables"] = rows

    if cpu_baseline:
        import oracle
        # the oracle as it stands, single thread, on the whole workload when that takes seconds,
        # else on a prefix of the rows
        n_s = N if N <= 150_000 else 150_000
        feat64 = cfg["feat"][:n_s].astype(np.float64)
        w64 = cfg["weight"].astype(np.float64)
        reps = 0
        t_cpu0 = time.perf_counter()
        while True:
            km = oracle.kmap(coords[:n_s], K, stride, mode)
            oracle.conv(feat64, w64, km, threads=1)
            reps += 1
            if time.perf_counter() - t_cpu0 > 12.0:      # about 12 s of CPU work, however many layers that is
                break
        t_cpu = (time.perf_counter() - t_cpu0) / reps
        P_s = int(km["offset_start"][-1])
        cpu = host_cpu()
        out["cpu_baseline"] = {
            "value": 2.0 * P_s * C_in * C_out / t_cpu / 1e12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "cpu_model": cpu["model"], "host_logical_cpus": cpu["logical_cpus"], "ms_per_layer": t_cpu * 1e3,
            "sample": (f"whole {workload} layer" if n_s == N else f"first {n_s} of {N} rows of {workload}")
                      + f" (N={n_s}, P={P_s}), kernel map + convolution, {reps} repetitions, mean",
        }
        # the same oracle with its loop over output-channel blocks spread over the host's cores
        # (the kernel map stays single-threaded), a few repetitions
        cores = min(os.cpu_count() or 1, 16)
        if cores > 1:
            reps_p, t_p0 = 0, time.perf_counter()
            while True:
                km = oracle.kmap(coords[:n_s], K, stride, mode)
                oracle.conv(feat64, w64, km, threads=cores)
                reps_p += 1
                if time.perf_counter() - t_p0 > 4.0:
                    break
            t_p = (time.perf_counter() - t_p0) / reps_p
            out["cpu_baseline_all_cores"] = {"value": 2.0 * P_s * C_in * C_out / t_p / 1e12, "unit": "TFLOP/s",
                                             "cores": cores, "kind": "oracle", "cpu_model": cpu["model"],
                                             "ms_per_layer": t_p * 1e3,
                                             "sample": out["cpu_baseline"]["sample"].replace(f"{reps} repetitions", f"{reps_p} repetitions")}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg5",
                    help="headline workload (default cfg5, the largest one that fits one GPU)")
    ap.add_argument("--no-target64", action="store_true",
                    help="leave out the sub-record of the ~110k-voxel 64-channel layer")
    ap.add_argument("--table", choices=["hash", "grid", "fused"], default="hash",
                    help="location table: the open-addressing hash table (default, what the metric is quoted on), "
                         "the dense array over the workload's voxel box (submanifold workloads only), or the dense "
                         "array with the look-ups fused into the convolution (no kernel map; 3x3x3 16-bit layers)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-tables", action="store_true")
    ap.add_argument("--graph", choices=["auto", "on", "off"], default="off",
                    help="replay the step from a captured HIP graph instead of launching eagerly "
                         "(measured slower than back-to-back eager launches here, so off by default)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (one process, one MI355X); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2402_07710_amd import binding as sc
    from paper_2402_07710_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)
    sc.load(build_if_missing=True)

    if args.workload == "cfg2-stage":
        return stage_bench(args, torch, sc, synth)
    if args.workload == "cfg3-inverse":
        return inverse_bench(args, torch, sc, synth)

    peaks = measured_peaks(torch, sc, dev)
    rec = measure_layer(args, torch, sc, synth, args.workload, args.steps, args.warmup, peaks,
                        others=not args.no_other_tables, cpu_baseline=not args.no_cpu_baseline)
    out = {
        "metric": "effective TFLOP/s over active MACs, whole layer incl. kernel map (hash + kmap + conv)",
        "value": rec.pop("value"), "unit": rec.pop("unit"), "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": rec.pop("dtype"), "data": "synthetic", "config": rec.pop("config"),
        "peaks": {"hbm_gbs": PEAK_HBM_GBS, "mfma_f16_tflops": PEAK_MFMA_TFLOPS, "measured_copy_gbs": peaks["copy_gbs"],
                  "measured_mfma_f16_tflops": peaks["mfma_f16_tflops"]},
        "host": host_cpu(),
    }
    roofline, cpu = rec.pop("roofline"), rec.pop("cpu_baseline", None)
    out.update(rec)
    out["roofline"] = roofline
    if cpu is not None:
        out["cpu_baseline"] = cpu
    if args.workload == "cfg5" and not args.no_target64:
        # the layer the 64-channel targets are stated on, measured the same way (more steps: it is 15x shorter)
        t64 = measure_layer(args, torch, sc, synth, "target64", max(args.steps, 100), args.warmup, peaks,
                            others=not args.no_other_tables, cpu_baseline=False)
        out["target64"] = t64
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
