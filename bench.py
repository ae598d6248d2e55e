#!/usr/bin/env python3
"""Benchmark of the local-block training step on one MI355X.

A step is one pass of the whole hot path (module forward, auxiliary forward,
local cross-entropy, backward stopping at the block input, optimizer update)
over one batch of seeded synthetic images already resident in HBM.  Prints one
JSON line: images/s, the dominant kernel's roofline fraction (HIP events around
every GEMM launch, in a second pass over the same workload) and the CPU oracle
timed on the host cores of the same box.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def step_flops(wl: dict, dense: bool = False) -> float:
    """Flop count of one step (multiply-add = 2): forward + 2x backward for every contraction, minus the input
    gradient that gradient isolation never needs.  dense=True: every encoder layer computed for all tokens (the
    plain definition).  dense=False: what the library executes: of the last auxiliary layer only the class-token
    row is computed behind the key / value projection (the head reads nothing else of it; the result is the same),
    so that layer counts K, V for all tokens and query, attention, projection and MLP for one row per image."""
    B = wl["batch"]
    if wl["arch"] == 0:
        T, D, F, H = wl["tokens"], wl["dim"], wl["mlp_dim"], wl["heads"]
        M = B * T
        layer_fwd = 2.0 * M * (D * 3 * D + D * D + 2 * D * F) + 4.0 * B * H * T * T * (D // H)
        total = 3.0 * layer_fwd * (wl["depth"] + wl["aux_depth"])
        if not dense and wl["aux_depth"] >= 1:
            cls_fwd = 2.0 * M * D * 2 * D + 2.0 * B * (D * D + D * D + 2 * D * F) + 4.0 * B * H * T * (D // H)
            total += 3.0 * (cls_fwd - layer_fwd)
        total += 3.0 * 2.0 * B * D * wl["num_classes"]
        if wl["input_kind"] == 0:
            total += 2.0 * 2.0 * B * (T - 1) * wl["patch"] ** 2 * wl["img_c"] * D
        return total
    C, A, H, W = wl["channels"], wl["aux_channels"], wl["height"], wl["width"]
    t = wl.get("transition_block", 0) - 1
    stem = wl["input_kind"] == 0
    total, first = 0.0, True
    if stem:   # forward + weight gradient; the image needs no gradient
        m = 2 if t >= 0 else 1
        total += 2.0 * 2.0 * B * (m * H) * (m * W) * 9 * wl["img_c"] * (C // m)
        first = False
    for i in range(wl["n_basic_blocks"]):
        if t >= 0 and i < t:
            ci, co, hw = C // 2, C // 2, 4 * H * W
        elif i == t:
            ci, co, hw = C // 2, C, H * W
        else:
            ci, co, hw = C, C, H * W
        conv1, conv2 = 2.0 * B * hw * 9 * ci * co, 2.0 * B * hw * 9 * co * co
        total += (2.0 if first else 3.0) * conv1 + 3.0 * conv2   # the detached block input needs no gradient
        first = False
    aux = 2.0 * B * (((H - 1) // 2 + 1) * ((W - 1) // 2 + 1)) * 9 * C * A
    return total + 3.0 * aux + 3.0 * 2.0 * B * A * wl["num_classes"]


def kernel_source_sha() -> str:
    """Hash of the kernel sources the library is built from: a counter summary is only valid for the sources it
    was taken with."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2411_12780_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, kind: str, launches_per_step: float):
    """HBM bytes per launch of the dominant kernel class (kind "gemm" or "conv") from the committed counter
    summary of this workload (two rocprofv3 --pmc runs, FETCH_SIZE then WRITE_SIZE, each scaled by what the same
    counter reads for the copy probe).  Counters cannot be read inside a timing run, so the figure comes from
    profiles/; it is reported only if that summary was taken with the kernel sources this library is built from
    (their hash is stamped into it) and counts as many launches of the class per step as this run has just
    bracketed, else None with the reason."""
    path = os.path.join(ROOT, "profiles", f"{workload}_{kind}_hbm_traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f)
        if rec.get("kernel_source_sha") != kernel_source_sha():
            return None, f"{os.path.basename(path)} was taken with other kernel sources ({rec.get('kernel_source_sha')})"
        if abs(float(rec["launches_per_step"]) - launches_per_step) > 1e-9:
            return None, (f"{os.path.basename(path)} counts {rec['launches_per_step']} launches of the class per step, "
                          f"this run {launches_per_step}")
        return float(rec["bytes_per_launch"]), None
    except (OSError, KeyError, ValueError):
        return None, "no counter summary committed for this workload"


def device_clock_mhz():
    """Peak engine clock the HIP runtime reports for device 0 (hipDeviceAttributeClockRate, kHz), or None."""
    import ctypes
    try:
        hip = ctypes.CDLL("libamdhip64.so")       # already loaded by PyTorch: the same runtime
        v = ctypes.c_int(0)
        if hip.hipDeviceGetAttribute(ctypes.byref(v), 5, 0) == 0 and 2e5 < v.value < 1e7:
            return v.value / 1e3
    except OSError:
        pass
    return None


def event_step_times(torch, run_one, steps: int):
    """Per-step durations in milliseconds from HIP events recorded on the stream the steps are enqueued on (the
    caller's current stream) between consecutive steps."""
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    evs[0].record()
    for i in range(steps):
        run_one(i)
        evs[i + 1].record()
    torch.cuda.synchronize()
    return [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]


def bench_pipeline(args, torch, P, synth, dev) -> int:
    """The pipeline workload: the 12-layer ViT as 4 blocks of 3 layers on 4 HIP streams, depth-2 device queues
    (vit_lpp12: as 12 blocks of one layer on 12 streams).  A step is one batch entering the pipeline;
    timing is steady state (queues full)."""
    if args.workload == "vit_lpp12":
        # Section 4.2's finest partition: 12 one-layer blocks, auxiliary depths from the d' = 4 schedule
        wls = synth.lpp_workloads(4)
        first = wls[0]
    elif args.workload == "vit_base224_pipeline4":
        # Section 4.3's ViT-Base at 224 x 224 (197 tokens of width 768), its 12 layers as 4 blocks of 3 with one
        # auxiliary layer each, SGD Nesterov
        first = synth.workload("vit_base_224_bf16")
        wls = [first] + [dict(first, input_kind=synth.ACTIVATION) for _ in range(3)]
    elif args.workload == "vit_base224_lpp12":
        # the layer-wise partition of Section 4.2 at ViT-Base / 224 x 224: 12 one-layer blocks, auxiliary depths for d' = 4
        base = synth.workload("vit_base_224_bf16")
        shape = {k: base[k] for k in ("img_h", "img_w", "img_c", "patch", "tokens", "dim", "heads", "mlp_dim", "optimizer",
                                      "momentum", "nesterov", "weight_decay", "lr", "batch")}
        wls = synth.lpp_workloads(4, **shape)
        first = wls[0]
    elif args.workload == "vit_base224_pipeline4_d4":
        # the same 4 blocks with the auxiliary depths of Section 4.2 for d' = 4 (N_l = d' - floor(l / 3) at the last layer
        # l = 2, 5, 8, 11 of each block): 4, 3, 2, 1 auxiliary layers
        first = synth.workload("vit_base_224_bf16", aux_depth=4)
        wls = [first] + [dict(first, input_kind=synth.ACTIVATION, aux_depth=a) for a in (3, 2, 1)]
    elif args.workload == "resnet32_k8":
        # Section 4.1's ResNet-32 at its CIFAR batch of 1024, cut into 8 local modules
        wls = synth.resnet32_modules(8)
        first = wls[0]
    else:
        first, rest = synth.workload("vit_stage_bf16"), synth.workload("vit_stage_act_bf16")
        wls = [first, dict(rest), dict(rest), dict(rest)]
    for j, w in enumerate(wls):
        w["seed"] = j
    vit = first["arch"] == 0
    cfgs = [P.make_config(w) for w in wls]
    depth = 2
    nbytes = P.ppll_pipeline_workspace_bytes(cfgs, depth)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    streams = [torch.cuda.Stream(device=dev) for _ in cfgs]
    pipe = P.ppll_pipeline_init(cfgs, depth, ws, nbytes, [s.cuda_stream for s in streams], None)
    ring = 8
    xs, ys = [], []
    for i in range(ring):
        x, y = synth.make_batch(first, seed=0, index=i)
        xs.append(torch.from_numpy(x).to(torch.bfloat16).to(dev))
        ys.append(torch.from_numpy(y).to(dev))
    lr = float(first["lr"])

    def run(n):
        for i in range(n):
            P.ppll_pipeline_step(pipe, xs[i % ring], ys[i % ring], lr)

    run(max(args.warmup, 8))
    P.ppll_pipeline_sync(pipe, len(cfgs))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    losses = P.ppll_pipeline_sync(pipe, len(cfgs))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    flops = sum(step_flops(w) for w in wls)
    out = {
        "metric": "local-block train step images/sec on 1 MI355X; % bf16 MFMA peak",
        "value": first["batch"] / (elapsed / args.steps), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": max(args.warmup, 8), "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": dict({"workload": args.workload, "batch": first["batch"], "blocks": len(cfgs), "queue_depth": depth,
                        "streams": len(cfgs), "optimizer": "adamw" if first["optimizer"] == 1 else "sgd"},
                       **({"layers_per_block": [w["depth"] for w in wls], "aux_depths": [w["aux_depth"] for w in wls]}
                          if vit else {"basic_blocks_per_module": [w["n_basic_blocks"] for w in wls],
                                       "channels": [w["channels"] for w in wls]})),
        "step_gflop": flops / 1e9, "step_tflops": flops / (elapsed / args.steps) / 1e12,
        "mfma_peak_frac_step": flops / (elapsed / args.steps) / 1e12 / PEAK_BF16_TFLOPS,
        "losses_last_batch": [float(v) for v in losses],
    }
    P.ppll_pipeline_destroy(pipe)
    del ws

    # Conventional local learning on the same GPU: the same blocks, one after the other on one stream
    # (the sequential chain the pipeline is bit-identical to), and the stage-1 phase times in the
    # symbols of the paper's time model (Section 3.3).
    tdt = torch.bfloat16
    blocks, keep = [], []
    for w, c in zip(wls, cfgs):
        n = P.ppll_block_workspace_bytes(c)
        buf = torch.empty(n, dtype=torch.uint8, device=dev)
        blocks.append(P.ppll_block_init(c, buf, n, None, None))
        keep.append((buf, torch.empty(synth.output_shape(w), dtype=tdt, device=dev),
                     torch.zeros(1, dtype=torch.float32, device=dev)))
    stream = torch.cuda.current_stream().cuda_stream

    def run_seq(n):
        for i in range(n):
            cur = xs[i % ring]
            for b, (_, xo, ls) in zip(blocks, keep):
                P.ppll_block_step(b, cur, ys[i % ring], lr, xo, ls, stream)
                cur = xo

    run_seq(max(args.warmup, 3))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_seq(args.steps)
    torch.cuda.synchronize()
    seq_ms = 1e3 * (time.perf_counter() - t0) / args.steps
    P.ppll_block_phase_timers(blocks[0], True)
    run_seq(3)
    f1, fa, Bp, Up = P.ppll_block_phase_times(blocks[0])
    P.ppll_block_phase_timers(blocks[0], False)
    s_stages = len(wls)
    k_layers = wls[0]["aux_depth"] / wls[0]["depth"] if vit else None
    out["sequential_chain_ms_per_step"] = seq_ms
    out["pipelined_over_sequential"] = out["ms_per_step"] / seq_ms
    out["time_model"] = {
        "stage1_phases_ms": {"f_1": f1, "f_a1": fa, "B_a1": Bp, "U_a1": Up},
        "S_PPLL_stage1_ms": f1 + fa + Bp + Up,
        "s": s_stages, "k_aux_over_module_layers": k_layers, "k_measured_f_a1_over_f_1": fa / f1 if f1 > 0 else None,
        "predicted_T_PPLL_over_T_PP": (k_layers + 1) / s_stages if vit else None,
        "note": "Section 3.3.1 predicts T_PPLL / T_PP = (k + 1) / s for s devices; on one GPU the blocks share the "
                "device, so the measured pipelined / sequential ratio above is bounded below by the chip's idle "
                "fraction, not by 1 / s",
    }
    for b in blocks:
        P.ppll_block_destroy(b)
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vit_stage_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also run the 256 MiB copy probe 5 times (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the pipeline: a block's local step runs on a single "
              "MI355X and this build uses no second GPU; run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2411_12780_amd import binding as P
    from paper_2411_12780_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU fallback)"
    dev = "cuda:0"
    if args.workload in ("vit_pipeline4", "vit_lpp12", "resnet32_k8", "vit_base224_pipeline4", "vit_base224_pipeline4_d4", "vit_base224_lpp12"):
        return bench_pipeline(args, torch, P, synth, dev)
    wl = synth.workload(args.workload)
    wl["seed"] = 0
    cfg = P.make_config(wl)
    ws_bytes = P.ppll_block_workspace_bytes(cfg)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    bf16 = wl["precision"] == synth.BF16
    tdt = torch.bfloat16 if bf16 else torch.float32
    blk = P.ppll_block_init(cfg, ws, ws_bytes, None, None)       # seeded draw inside the library
    ring = 8
    xs, ys = [], []
    for i in range(ring):
        x, y = synth.make_batch(wl, seed=0, index=i)
        xs.append(torch.from_numpy(x).to(tdt).to(dev))
        ys.append(torch.from_numpy(y).to(dev))
    x_out = torch.empty(synth.output_shape(wl), dtype=tdt, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    lr = float(wl["lr"])

    def run(n):
        for i in range(n):
            P.ppll_block_step(blk, xs[i % ring], ys[i % ring], lr, x_out, loss, stream)

    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    last_loss = P.ppll_block_sync(blk)
    ms_per_step = 1e3 * elapsed / args.steps
    flops = step_flops(wl)
    # the same steps once more, each between two events on the stream: median and minimum step time
    per_step = sorted(event_step_times(torch, lambda i: P.ppll_block_step(blk, xs[i % ring], ys[i % ring], lr, x_out, loss, stream),
                                       args.steps))
    props = torch.cuda.get_device_properties(0)
    clock_mhz = device_clock_mhz()
    # CUs x 4096 flop/clk/CU (dense bf16 MFMA) x the clock the device reports
    device_peak_tflops = props.multi_processor_count * 4096 * clock_mhz * 1e6 / 1e12 if clock_mhz else None
    out = {
        "metric": "local-block train step images/sec on 1 MI355X; % bf16 MFMA peak",
        "value": wl["batch"] / (elapsed / args.steps),
        "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "batch": wl["batch"],
                   "shape": {k: wl[k] for k in ("tokens", "dim", "heads", "mlp_dim", "depth", "aux_depth",
                                                "channels", "height", "width", "n_basic_blocks") if k in wl},
                   "optimizer": "adamw" if wl["optimizer"] == synth.ADAMW else "sgd"},
        "step_gflop": flops / 1e9,
        **({"step_gflop_note": "executed work: of the last auxiliary layer only the class-token row is computed behind K, V",
            "step_gflop_dense_definition": step_flops(wl, dense=True) / 1e9} if wl["arch"] == synth.VIT else {}),
        "step_tflops": flops / (elapsed / args.steps) / 1e12,
        "mfma_peak_frac_step": flops / (elapsed / args.steps) / 1e12 / PEAK_BF16_TFLOPS,
        "ms_per_step_events": {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1]},
        "images_per_s_at_median": wl["batch"] / (per_step[len(per_step) // 2] * 1e-3),
        "device_reported": {"compute_units": props.multi_processor_count, "clock_mhz": clock_mhz,
                            "bf16_peak_tflops_at_that_clock": device_peak_tflops,
                            "mfma_peak_frac_step_at_that_clock":
                                flops / (elapsed / args.steps) / 1e12 / device_peak_tflops if device_peak_tflops else None},
        "loss_last_step": last_loss,
    }

    if not args.no_roofline:
        # second pass over the same workload with every GEMM launch bracketed by HIP events
        P.ppll_block_profile_enable(blk, True)
        P.ppll_block_profile_read(blk)
        P.ppll_block_profile_read_conv(blk)
        P.ppll_block_profile_read_small(blk)
        run(args.steps)
        torch.cuda.synchronize()
        gemm_ms, gemm_flops, launches = P.ppll_block_profile_read(blk)
        conv_ms, conv_bytes, conv_launches = P.ppll_block_profile_read_conv(blk)
        small_ms, small_flops, small_launches = P.ppll_block_profile_read_small(blk)
        P.ppll_block_profile_enable(blk, False)
        if launches > 0:
            achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12
            traffic, why_not = measured_traffic(args.workload, "gemm", launches / args.steps)
            out["roofline"] = {"bound": "mfma",
                               "kernel": "gemm_mfma_kernel on the token matrices (Linear forward, input gradient) and the grouped weight-gradient launch",
                               "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                               "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                               **({"traffic_missing_because": why_not} if why_not else {}),
                               "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a copy probe)",
                               "launches_per_step": launches / args.steps,
                               "avg_launch_us": 1e3 * gemm_ms / launches,
                               "gemm_ms_per_step": gemm_ms / args.steps,
                               "gemm_flop_share_of_step": gemm_flops / args.steps / flops}
            if small_launches > 0:
                # the class-token products of the pruned last auxiliary layer: a few rows each, bound by launch latency
                out["small_products"] = {"kernel": "gemm_rows_kernel (products with fewer than 256 output rows)",
                                         "launches_per_step": small_launches / args.steps,
                                         "avg_launch_us": 1e3 * small_ms / small_launches,
                                         "ms_per_step": small_ms / args.steps,
                                         "achieved_tflops": small_flops / (small_ms * 1e-3) / 1e12}

        elif conv_launches > 0:
            # ResNet blocks: the dominant kernel is the 3x3 convolution (forward + input gradient), bound by HBM
            gbs = conv_bytes / (conv_ms * 1e-3) / 1e9
            traffic, why_not = measured_traffic(args.workload, "conv", conv_launches / args.steps)
            out["roofline"] = {"bound": "hbm", "kernel": "conv3x3_mfma_kernel (forward and input gradient)",
                               "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                               "traffic": traffic, **({"traffic_missing_because": why_not} if why_not else {}),
                               "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a copy probe)",
                               "launches_per_step": conv_launches / args.steps,
                               "avg_launch_us": 1e3 * conv_ms / conv_launches,
                               "conv_ms_per_step": conv_ms / args.steps,
                               "algorithmic_bytes_per_launch": conv_bytes / conv_launches}

    if not args.no_roofline:
        # third pass: phase times of the step in the paper's symbols (Section 3.3)
        P.ppll_block_phase_timers(blk, True)
        run(3)
        f1, fa, Bp, Up = P.ppll_block_phase_times(blk)
        P.ppll_block_phase_timers(blk, False)
        out["phases_ms"] = {"f_1": f1, "f_a1": fa, "B_a1": Bp, "U_a1": Up}

    if args.probe_copy:
        nbytes = 256 << 20
        src = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        for _ in range(5):
            P.ppll_probe_copy(src, dst, nbytes, stream)
        torch.cuda.synchronize()
        out["probe_copy_bytes"] = nbytes

    if not args.no_cpu_baseline:
        from oracle import ppll_oracle as O
        from helpers import oracle_cfg
        from threadpoolctl import threadpool_info
        ocfg = oracle_cfg(wl)
        st = O.block_init(ocfg, synth.make_params(O.param_spec(ocfg), seed=0), np.float64)
        x, y = synth.make_batch(wl, seed=0, index=0)
        # a bounded sample: whole steps until about 10 s of CPU work are spent (at least 1, at most 10 steps)
        small = wl["batch"] * wl.get("tokens", 1) < 2048
        n_steps, t0 = 0, time.perf_counter()
        while n_steps < 10 and (n_steps == 0 or time.perf_counter() - t0 < 10.0):
            O.block_step(st, x.astype(np.float64), y, lr)
            n_steps += 1
        cpu_s = (time.perf_counter() - t0) / n_steps
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
        out["cpu_baseline"] = {"value": wl["batch"] / cpu_s, "unit": "images/s", "cores": threads,
                               "kind": "oracle", "sample": f"{n_steps} full step(s) of the same workload "
                               f"(batch {wl['batch']}), float64 numpy oracle, {cpu_s:.2f} s per step"}
        if small:   # a small workload: the same on one core as well
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):
                t0 = time.perf_counter()
                for _ in range(n_steps):
                    O.block_step(st, x.astype(np.float64), y, lr)
                one_s = (time.perf_counter() - t0) / n_steps
            out["cpu_baseline"]["one_core"] = {"value": wl["batch"] / one_s, "unit": "images/s", "cores": 1,
                                               "sample": f"{n_steps} step(s), {one_s:.3f} s per step"}
    P.ppll_block_destroy(blk)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
