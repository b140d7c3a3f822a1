#!/usr/bin/env python3
"""Benchmark of the sparse-convolution hot path on one MI355X.

One step = one whole layer on synthetic input already resident in HBM:
sc_hash_build -> sc_kmap_build -> sc_conv_fwd (kernel map construction included).
Prints ONE JSON line: effective TFLOP/s over active MACs (2*P*C_in*C_out / time per layer),
ms per layer, the per-phase split, the roofline of the kernel that takes the most time
(durations from HIP events recorded around every kernel launch, on the launch's stream), and the
CPU oracle timed on this host's cores for the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg3|cfg3k3|cfg4|cfg5|cfg1|target64|cfg2-stage] [--table hash|grid]
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
    times the units one launch processes (both are stated in the design doc)."""
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
        down.kmap_build(d_coords, stream)                                   # K == stride: no table needed
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
        "kernels": {k: {"launches_per_step": l / args.steps, "avg_us": round(1e3 * t / l, 3)} for k, (l, t) in prof.items()},
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
        "kernels": {k: {"launches_per_step": l / args.steps, "avg_us": round(1e3 * t / l, 3)} for k, (l, t) in prof.items()},
    }))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--table", choices=["hash", "grid", "fused"], default="hash",
                    help="location table: the open-addressing hash table (default, what the metric is quoted on), "
                         "the dense array over the workload's voxel box (submanifold workloads only), or the dense "
                         "array with the look-ups fused into the convolution (no kernel map; 3x3x3 16-bit layers)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", choices=["auto", "on", "off"], default="off",
                    help="replay the step from a captured HIP graph instead of launching eagerly "
                         "(measured slower than back-to-back eager launches here, so off by default)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run a plain device copy of this many MiB (reference for HBM byte counters)")
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
    cfg = synth.make_config(args.workload)
    coords, K, stride, mode = cfg["coords"], cfg["K"], cfg["stride"], cfg["mode"]
    C_in, C_out, dtype = cfg["C_in"], cfg["C_out"], cfg["dtype"]
    N = len(coords)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]
    d_coords = torch.from_numpy(coords).to(dev)
    d_feat = torch.from_numpy(cfg["feat"]).to(dev).to(tdt).contiguous()
    d_w = torch.from_numpy(cfg["weight"]).to(dev).to(tdt).contiguous()
    if args.table != "hash" and mode != "subm":
        print("bench.py: --table grid applies to submanifold workloads only", file=sys.stderr)
        return 2
    buf = sc.LayerBuffers(N, K, stride, mode, C_in, C_out, dtype, device=dev,
                          grid_dims=cfg["box"] if args.table != "hash" else None)
    stream = torch.cuda.current_stream()

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
        buf.conv_fwd(d_feat, d_w, stream)

    if args.copy_calibration:
        src = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    step()
    if args.table == "fused":
        buf.kmap_build(d_coords, stream)          # once, outside the timed region: only to count the pairs
    h = buf.read_counts()
    if h.status != 0:
        raise RuntimeError(f"device status {h.status}")
    P, N_out = int(h.n_pairs), int(h.n_out)
    flops = 2.0 * P * C_in * C_out

    for _ in range(args.warmup):
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
                        buf.conv_fwd(d_feat, d_w, gstream)
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

    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_eager = (time.perf_counter() - t0) * 1e3 / args.steps
    value = flops / (ms_per_step * 1e-3) / 1e12

    # per-phase split with torch events (the library launches on torch's current stream)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for i in range(args.steps):
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
            buf.conv_fwd(d_feat, d_w, stream)
        ev[i][3].record(stream)
    torch.cuda.synchronize()
    phases = {name: float(np.median([e[j].elapsed_time(e[j + 1]) for e in ev]))
              for j, name in enumerate(["hash_ms", "kmap_ms", "conv_ms"])}

    # per-kernel durations: every launch carries a pair of HIP events stamped with the dispatch's
    # begin and end (hipExtLaunchKernelGGL inside the library), over the same number of steps
    sc.sc_profile_enable(True)
    for _ in range(args.steps):
        step()
    prof = sc.sc_profile_read()
    sc.sc_profile_enable(False)
    kernels = {name: {"launches": l, "avg_us": 1e3 * ms / l} for name, (l, ms) in prof.items()}
    per_step_us = {name: kernels[name]["avg_us"] * l / args.steps for name, (l, ms) in prof.items()}
    dominant = max(per_step_us, key=per_step_us.get)
    launches_per_step = prof[dominant][0] / args.steps
    avg_s = kernels[dominant]["avg_us"] * 1e-6
    st = dict(N=N, N_out=N_out, P=P, K3=K ** 3, cap=(sc.sc_hash_bytes(N) - 256) // 16, C_in=C_in, C_out=C_out,
              elem_bytes=d_feat.element_size())
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
    if os.path.exists(tpath):
        key = args.workload if args.table == "hash" else f"{args.workload}-{args.table}"
        traffic = json.load(open(tpath)).get(key, {}).get(dominant)
    conv_bytes = algorithmic_bytes("k_conv_mfma", st)
    conv_peak = PEAK_MFMA_TFLOPS if dtype != "f32" else PEAK_FP32_TFLOPS
    # which roof a contraction of this shape is under: flops per algorithmic byte against the
    # machine balance (peak flops / peak bytes).  32- and 64-channel layers sit under the HBM roof.
    conv_under_hbm = flops / conv_bytes * PEAK_HBM_GBS * 1e9 < conv_peak * 1e12
    if dominant in ("k_conv_mfma", "k_conv_f32") and not conv_under_hbm:
        # the contraction: flops of the pairs that exist against the matrix-core (or fp32 ALU) peak
        peak = PEAK_MFMA_TFLOPS if dominant == "k_conv_mfma" else PEAK_FP32_TFLOPS
        achieved = flops / avg_s / 1e12
        roofline = {"kernel": dominant, "bound": "mfma" if dominant == "k_conv_mfma" else "alu",
                    "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                    "traffic": traffic, "avg_us": avg_s * 1e6,
                    "hbm_gbs_algorithmic": algorithmic_bytes(dominant, st) / avg_s / 1e9}
    else:
        ab = algorithmic_bytes(dominant, st)
        achieved = ab / avg_s / 1e9 if ab else None
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": (achieved / PEAK_HBM_GBS) if achieved else None,
                    "traffic": traffic, "avg_us": avg_s * 1e6, "launches_per_step": launches_per_step}
        if dominant in ("k_conv_mfma", "k_conv_f32"):
            roofline["flops_per_algorithmic_byte"] = flops / conv_bytes
            roofline["tflops_active"] = flops / avg_s / 1e12
    per_kernel = {}
    for name in kernels:
        ab = algorithmic_bytes(name, st)
        per_kernel[name] = {"avg_us": round(kernels[name]["avg_us"], 3),
                            "per_step_us": round(per_step_us[name], 3)}
        if ab:
            per_kernel[name]["hbm_gbs_algorithmic"] = round(ab / (kernels[name]["avg_us"] * 1e-6) / 1e9, 1)
            per_kernel[name]["frac_of_hbm_peak"] = round(ab / (kernels[name]["avg_us"] * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)
        if name in ("k_conv_mfma", "k_conv_f32"):
            per_kernel[name]["tflops_active"] = round(flops / (kernels[name]["avg_us"] * 1e-6) / 1e12, 2)
            if name == "k_conv_mfma":
                per_kernel[name]["frac_of_mfma_peak"] = round(flops / (kernels[name]["avg_us"] * 1e-6) / 1e12 / PEAK_MFMA_TFLOPS, 4)

    out = {
        "metric": "effective TFLOP/s over active MACs, whole layer incl. kernel map (hash + kmap + conv)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": args.workload, "table": args.table, "mode": mode, "K": K, "stride": stride, "C_in": C_in,
                   "C_out": C_out, "N": N, "N_out": N_out, "P": P, "pairs_per_voxel": P / max(N, 1)},
        "launch": "hip graph replay" if graph is not None else "eager", "ms_per_step_eager": ms_per_step_eager,
        "phases_ms": phases, "kernels": per_kernel, "roofline": roofline,
    }

    # the same layer with the other location tables (same checks: the outputs must be identical),
    # for comparison: "grid" = dense array + kernel map, "fused" = dense array, look-ups inside the
    # convolution, no kernel map (3x3x3 16-bit layers with a dedicated kernel only)
    if mode == "subm":
        others = []
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
                    buf2.layer(d_coords, d_feat, d_w, stream)

            for _ in range(args.warmup + 1):
                step2()
            if not torch.equal(buf2.feat_out[:N_out], buf.feat_out[:N_out]):
                raise RuntimeError(f"location table '{other}' gives a different layer")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                step2()
            torch.cuda.synchronize()
            ms2 = (time.perf_counter() - t0) * 1e3 / args.steps
            others.append({"table": other, "ms_per_step": ms2, "value": flops / (ms2 * 1e-3) / 1e12, "unit": "TFLOP/s"})
            del buf2
        out["other_tables"] = others

    if not args.no_cpu_baseline:
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
        out["cpu_baseline"] = {
            "value": 2.0 * P_s * C_in * C_out / t_cpu / 1e12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "ms_per_layer": t_cpu * 1e3,
            "sample": (f"whole {args.workload} layer" if n_s == N else f"first {n_s} of {N} rows of {args.workload}")
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
                                             "cores": cores, "kind": "oracle", "ms_per_layer": t_p * 1e3,
                                             "sample": out["cpu_baseline"]["sample"].replace(f"{reps} repetitions", f"{reps_p} repetitions")}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
