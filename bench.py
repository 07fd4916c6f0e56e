#!/usr/bin/env python3
"""Throughput of the WCC forward path on one MI355X.

A step is one ``wcc_forward`` (Haar transform -> joint top-k -> gather/quantise -> 1x1
contraction -> scatter + inverse Haar) over one batch of seeded synthetic feature maps that
are already resident in HBM.  The default workload is the largest single-layer configuration
(the expansion layer: B 4, 64 -> 256 channels, 512 x 1024, 3 levels, keep 1/8).  Prints ONE
JSON line: whole-layer Gpixel*ch/s, the roofline fraction of the dominant kernel (measured
with HIP events inside the library around that kernel), every stage against the HBM peak, the
contraction against the matrix-core peak, and the CPU oracle timed on this host as a reported
baseline.
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

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
# dense matrix-core peaks (published) by the contraction's operand type, TFLOP/s (TOP/s for int8);
# fp32 weights or unquantised activations run on the vector ALUs (fp32 vector peak)
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "int8": 5000.0, "f32": 157.3}
CACHE_BYTES = 256 << 20  # memory-side cache


# stage of wcc_forward -> the one kernel it launches (norm_select is four small kernels)
STAGE_KERNEL = {"haar_fwd": "haar_fwd_kernel", "gather": "haar_keep_kernel",
                "pointwise": "pointwise", "scatter_ihaar": "scatter_ihaar_kernel"}


def algorithmic_bytes(cfg, act_bytes: int = 4, xc_bytes: int | None = None) -> dict:
    """Bytes each stage of the fused layer must move per call: what the method itself reads
    and writes (feature maps of act_bytes per element, kept coefficients of xc_bytes -- one for
    8-bit codes, four for fp32 --, int32 positions), not what an implementation adds."""
    B, Ci, Co, N, k = cfg.B, cfg.C_in, cfg.C_out, cfg.N, cfg.k
    bw = {0: 4, 1: 2, 2: 1, 3: 0.5}[cfg.w_dtype]
    a = act_bytes
    if xc_bytes is None:
        xc_bytes = 1 if (cfg.act_bits == 8 and k % 4 == 0) else 4
    return {
        "haar_fwd": a * B * Ci * N + 4 * B * N,                    # read x, write norms
        "norm_select": 4 * B * N + 4 * B * k,                      # read norms, write I
        "gather": a * B * Ci * N + 4 * B * k + xc_bytes * B * Ci * k,  # read x and I, write X_wt[I]
        "pointwise": xc_bytes * B * Ci * k + bw * Ci * Co + 4 * B * Co * k,
        "scatter_ihaar": 4 * B * Co * k + 4 * B * k + a * B * Co * N,
    }


def read_profile_column(profile_dir: str, prefix: str, workload: str, kernel: str, column: int):
    """One number of the committed rocprofv3 summary `<prefix>_<workload>.txt` for the first
    kernel whose name starts with `kernel` (column counted over whitespace-separated fields),
    or None if there is no such file or line."""
    path = os.path.join(profile_dir, f"{prefix}_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        t = line.split()
        if len(t) > column and t[0].startswith(kernel) and not line.startswith("#"):
            try:
                return float(t[column])
            except ValueError:
                return None
    return None


def profiled_kernel_name(profile_dir: str, workload: str, prefix: str, default: str) -> str:
    """Name (without template arguments) of the first kernel starting with `prefix` in the
    committed `kernel_stats_<workload>.txt`: the library picks between two contraction
    kernels by shape, and the profile says which one ran."""
    path = os.path.join(profile_dir, f"kernel_stats_{workload}.txt")
    if os.path.exists(path):
        for line in open(path):
            if line.startswith(prefix):
                return line.split()[0].split("<")[0]
    return default


def read_traffic(profile_dir: str, workload: str, kernel: str):
    """HBM bytes per launch of `kernel` (fetch + write, each scaled by the copy-kernel
    calibration) from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(profile_dir, f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        t = line.split()
        if len(t) >= 4 and t[0].startswith(kernel):
            return float(t[3])
    return None


def stream_ceilings(probe, torch, nbytes: int = 512 << 20, reps: int = 4) -> dict:
    """GB/s of the plain streaming kernels of libwcc_probe.so (read, write, copy; ordinary and
    non-temporal accesses) over buffers of `nbytes`, twice the memory-side cache, each at four
    grid sizes with the best one reported: what this machine's memory system gives to the simplest
    code, for placing the stage rates above."""
    a = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").fill_(1.0)
    b = torch.empty_like(a)
    out = {"bytes": nbytes}
    for name, kind, moved in (("read", probe.READ, 1), ("write", probe.WRITE, 1),
                              ("copy", probe.COPY, 2)):
        for nt in (False, True):
            best = 0.0
            for blocks in (2048, 8192, 32768, 131072):
                probe.wcc_probe_stream(kind, a, b, nbytes, nt, blocks)
                t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                t0.record()
                for _ in range(reps):
                    probe.wcc_probe_stream(kind, a, b, nbytes, nt, blocks)
                t1.record()
                t1.synchronize()
                best = max(best, moved * nbytes * reps / (t0.elapsed_time(t1) * 1e-3) / 1e9)
            out[name + ("_nt" if nt else "")] = round(best, 1)
    for nt in (False, True):  # the same fill with eight stores a thread (what a strip kernel's waves do)
        probe.wcc_probe_stream(probe.WRITE8, None, b, nbytes, nt)
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record()
        for _ in range(reps):
            probe.wcc_probe_stream(probe.WRITE8, None, b, nbytes, nt)
        t1.record()
        t1.synchronize()
        out["write8" + ("_nt" if nt else "")] = round(nbytes * reps / (t0.elapsed_time(t1) * 1e-3) / 1e9, 1)
    return out


def bench_stack(args, synth, run_layer, ctx) -> int:
    """The 16 point-wise layers of the backbone stack, one after the other (each on its own
    synthetic input; the depthwise convolutions between them are not on the path)."""
    num, den = (int(t) for t in args.keep.split("/"))
    layers = synth.stack_layers(num, den, B=4)
    per_layer, total_s, total_pix, total_alg = [], 0.0, 0, 0
    worst = None
    for cfg in layers:
        dt, stage_us, _, _, _ = run_layer(cfg, ctx)
        alg = algorithmic_bytes(cfg, 2 if args.act == "bf16" else 4)
        total_s += dt
        total_pix += cfg.B * cfg.H * cfg.W * cfg.C_in
        total_alg += sum(alg.values())
        per_layer.append({"layer": cfg.name, "us": round(dt * 1e6, 2), "levels": cfg.levels,
                          "stages_us": {n: round(v, 2) for n, v in stage_us.items()}})
        dom = max(STAGE_KERNEL, key=lambda n: stage_us[n])
        if worst is None or stage_us[dom] > worst[0]:
            worst = (stage_us[dom], dom, alg[dom], cfg.name)
    achieved = worst[2] / (worst[0] * 1e-6) / 1e9
    out = {
        "metric": "WCC layer forward throughput", "value": round(total_pix / total_s / 1e9, 3),
        "unit": "Gpixel*ch/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(total_s * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "launch": args.launch,
        "config": {"workload": f"stack16_B4_keep{num}/{den}", "layers": len(layers), "act_bits": 8},
        "roofline": {"bound": "hbm", "kernel": STAGE_KERNEL[worst[1]], "layer": worst[3],
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes": worst[2], "kernel_us": round(worst[0], 2)},
        "layer_alg_GBs": round(total_alg / total_s / 1e9, 1),
        "per_layer": per_layer,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


ALU_PEAK_TFLOPS = 157.3  # fp32 vector, published (counts packed operations; this build issues none)
# fp32 operations per pixel and middle channel of one chained transform pass (3 levels): the 3x3
# convolution 18, the strip's synthesis 7.9, the two halo rows 2.0, the analysis 7.9, norms 2.1
CHAIN_FLOP_PER_PIXEL_CHANNEL = 37.9

# Table "Inference timing results" of the appendix "Inference times": image side, c_in, expansion,
# batch, kept fraction, and the speed-up the paper measured on a GTX 1080 Ti (context only)
PAPER_TABLE = [
    (96, 512, 2, 48, (1, 4), 1.52), (96, 512, 2, 48, (1, 2), 1.20), (96, 512, 4, 24, (1, 4), 1.71),
    (96, 512, 4, 24, (1, 2), 1.29), (96, 1024, 2, 12, (1, 4), 1.94), (96, 1024, 2, 12, (1, 2), 1.38),
    (96, 1024, 4, 6, (1, 4), 2.13), (96, 1024, 4, 6, (1, 2), 1.47), (128, 128, 4, 80, (1, 4), 1.20),
    (128, 128, 6, 64, (1, 4), 1.28), (128, 256, 4, 32, (1, 8), 1.81), (128, 256, 4, 32, (1, 4), 1.53),
    (128, 256, 4, 32, (1, 2), 1.27), (256, 256, 4, 8, (1, 8), 1.85), (256, 256, 4, 8, (1, 4), 1.57),
    (256, 256, 4, 8, (1, 2), 1.29), (256, 256, 8, 4, (1, 8), 1.99), (256, 256, 8, 4, (1, 4), 1.68),
    (256, 256, 8, 4, (1, 2), 1.39), (512, 128, 6, 4, (1, 4), 1.41), (512, 128, 6, 2, (1, 2), 1.12),
    (512, 256, 4, 2, (1, 8), 1.77), (512, 256, 4, 2, (1, 4), 1.52), (512, 256, 4, 2, (1, 2), 1.20),
]


def block_algorithmic_bytes(cfg, act_bytes: int, chained: bool) -> dict:
    """Bytes every kernel of the block must move per call (see algorithmic_bytes).  Chained, the
    expand layer has no inverse and the project layer's two passes read the expand layer's
    compressed output (and its rank map) instead of the expanded feature map."""
    alg = {}
    for layer in (0, 1):
        for name, v in algorithmic_bytes(cfg.layer(layer), act_bytes).items():
            alg[f"l{layer}_{name}"] = v
    alg["l1_scatter_ihaar"] += act_bytes * cfg.B * cfg.C * cfg.N      # the skip connection is read
    # K_dw is folded into the project layer's passes when W % 4 == 0 (its output is never written)
    alg["depthwise"] = 0 if cfg.W % 4 == 0 else 8 * cfg.B * cfg.C_mid * cfg.N
    if chained:
        l1 = cfg.layer(1)
        xcb = 1 if (cfg.act_bits == 8 and cfg.k % 4 == 0) else 4
        src = 4 * cfg.B * cfg.C_mid * cfg.k + 4 * cfg.B * cfg.N       # Y_wt of the expand layer + its rank map
        alg["l0_scatter_ihaar"] = 0
        alg["l1_haar_fwd"] = src + 4 * cfg.B * cfg.N
        alg["l1_gather"] = src + 4 * cfg.B * cfg.k + xcb * l1.B * l1.C_in * cfg.k
    return alg


def time_block(cfg, args, synth, wcc, torch, np, dense: bool) -> dict:
    """Times args.steps forwards of one inverted residual block (and, if asked, the dense block
    on the same GPU); returns the measurements."""
    x, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    bf16 = args.act == "bf16"
    if bf16:
        x = synth.round_to_bf16(x)
    d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                            cfg.keep_den, cfg.w_dtype, cfg.act_bits, wcc.BF16 if bf16 else wcc.F32,
                            wcc.NORM_L2 if args.norm == "l2" else wcc.NORM_L1)
    chained = wcc.block_is_chained(d)
    ctx = wcc.Context(0)
    ctx.ensure_workspace(d)

    def up(a):
        a = a.view(np.int16) if a.dtype == np.uint16 else a
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    xd, w1d, w3d, wdd = up(x), up(w1.stored), up(w3.stored), up(w_dw)
    if bf16:
        xd = xd.to(torch.bfloat16)
    y = torch.empty_like(xd)

    # (int8 weight codes come with a scale per output channel)
    s1d = None if w1.scale is None else up(w1.scale.astype(np.float32))
    s3d = None if w3.scale is None else up(w3.scale.astype(np.float32))

    def step():
        ctx.wcc_block_forward(d, xd, w1d, s1d, wdd, w3d, s3d, y)

    if args.copy_probe:  # a plain copy of known size, for scaling the traffic counters
        probe = torch.empty_like(xd)
        for _ in range(args.copy_probe):
            probe.copy_(xd)
        torch.cuda.synchronize()
        del probe
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps

    # per-kernel device times: the stage events bracket one of the two layers at a time
    stage_us = {}
    for layer in (0, 1):
        ctx.set_block_profile_layer(layer)
        ctx.set_profiling(True)
        acc = {}
        for _ in range(args.steps):
            step()
            for name, ms in ctx.stage_times().items():
                acc[name] = acc.get(name, 0.0) + ms
        ctx.set_profiling(False)
        acc.pop("event_pair")
        for name, v in acc.items():
            key = name if name == "depthwise" else f"l{layer}_{name}"
            stage_us[key] = 1e3 * v / args.steps

    # The dense block on the same GPU (the "standard" column of the paper's table), twice:
    # (a) the framework's library convolutions in bf16 as they come -- on this stack the
    #     depthwise one falls back to a naive kernel that takes most of the time;
    # (b) the framework's two bf16 1x1 convolutions and the skip addition, plus this library's
    #     own depthwise kernel (fp32) on a tensor of the same shape: the fair comparison.
    dense_ms = dense_fair_ms = None
    if dense:
        try:
            F = torch.nn.functional
            xb = xd.to(torch.bfloat16)
            k1 = torch.from_numpy(w1.values.astype(np.float32)).cuda().to(torch.bfloat16)[:, :, None, None]
            k3 = torch.from_numpy(w3.values.astype(np.float32)).cuda().to(torch.bfloat16)[:, :, None, None]
            kd = wdd.to(torch.bfloat16)[:, None]

            def timed(fn, reps):
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(reps):
                    fn()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) / reps * 1e3

            if not args.table:
                dense_ms = timed(lambda: xb + F.conv2d(F.conv2d(F.conv2d(xb, k1), kd, padding=1,
                                                                groups=cfg.C_mid), k3), args.steps)
            mid_b = F.conv2d(xb, k1)
            mid_f = mid_b.float()
            mid_g = torch.empty_like(mid_f)
            dense_fair_ms = (timed(lambda: F.conv2d(xb, k1), args.steps)
                             + timed(lambda: ctx.wcc_depthwise3x3(mid_f, wdd, mid_g), args.steps)
                             + timed(lambda: xb + F.conv2d(mid_b, k3), args.steps))
            del mid_b, mid_f, mid_g
        except Exception as exc:  # the library convolutions are context only
            print(f"bench.py: dense block baseline skipped ({exc})", file=sys.stderr)
    ctx.close()
    return {"cfg": cfg, "x": x, "w1": w1, "w_dw": w_dw, "w3": w3, "dt": dt, "stage_us": stage_us,
            "chained": chained, "dense_ms": dense_ms, "dense_fair_ms": dense_fair_ms, "bf16": bf16}


def block_from_shape(synth, shape: str, num: int, den: int, weights: str = "bf16"):
    """--shape SIDE,c,e,B or HxW,c,e,B -> a block of the paper's kind (3 levels, 8-bit codes)."""
    side, c, e, B = shape.split(",")
    H, W = (int(t) for t in side.split("x")) if "x" in side else (int(side), int(side))
    return synth.block_shape(H, W, int(c), int(e), int(B), num, den,
                             synth.W_I8 if weights == "i8" else synth.W_BF16)


def bench_block(args, synth, wcc, torch, np) -> int:
    """The inverted residual block the paper timed (appendix "Inference times"): by default
    256x256 image, c_in 256, expansion 4, batch 8, one row of its table per keep ratio."""
    num, den = (int(t) for t in args.keep.split("/"))
    cfg = block_from_shape(synth, args.shape or "256,256,4,8", num, den, args.weights)
    r = time_block(cfg, args, synth, wcc, torch, np, dense=not args.no_dense_baseline)
    dt, stage_us, chained, bf16 = r["dt"], r["stage_us"], r["chained"], r["bf16"]
    dense_ms, dense_fair_ms = r["dense_ms"], r["dense_fair_ms"]
    alg = block_algorithmic_bytes(cfg, 2 if bf16 else 4, chained)
    kernel_of = {"depthwise": "depthwise3x3_kernel"}
    for layer in (0, 1):
        for name, kname in STAGE_KERNEL.items():
            kernel_of[f"l{layer}_{name}"] = kname
    if chained:
        kernel_of["l1_haar_fwd"], kernel_of["l1_gather"] = "chain_norm_kernel", "chain_keep_kernel"
    dom = max(kernel_of, key=lambda n: stage_us[n])
    prof = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles")
    traffic = read_traffic(prof, cfg.name, kernel_of[dom])
    prof_us = read_profile_column(prof, "kernel_stats", cfg.name, kernel_of[dom], 2)
    if chained and dom in ("l1_haar_fwd", "l1_gather"):
        # the chained passes are bound by fp32 vector arithmetic, not by bytes
        flops = CHAIN_FLOP_PER_PIXEL_CHANNEL * cfg.B * cfg.C_mid * cfg.N
        ach = flops / (stage_us[dom] * 1e-6) / 1e12
        roof = {"bound": "alu", "kernel": kernel_of[dom], "stage": dom, "achieved": round(ach, 2),
                "peak": ALU_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / ALU_PEAK_TFLOPS, 4),
                "frac_of_unpacked_peak": round(ach / (ALU_PEAK_TFLOPS / 2), 4), "traffic": traffic,
                "algorithmic_flops": flops, "algorithmic_bytes": alg[dom],
                "kernel_us": round(stage_us[dom], 2), "profile_avg_us": prof_us}
    else:
        achieved = alg[dom] / (stage_us[dom] * 1e-6) / 1e9
        roof = {"bound": "hbm", "kernel": kernel_of[dom], "stage": dom, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "algorithmic_bytes": alg[dom], "kernel_us": round(stage_us[dom], 2),
                "profile_avg_us": prof_us}
    pix_ch = cfg.B * cfg.N * cfg.C
    wname = "int8" if cfg.w_dtype == synth.W_I8 else "bf16"  # operand type of the two contractions
    out = {
        "metric": "WCC layer forward throughput", "value": round(pix_ch / dt / 1e9, 3),
        "unit": "Gpixel*ch/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wname, "data": "synthetic", "launch": "eager",
        "config": {"workload": cfg.name, "B": cfg.B, "C": cfg.C, "expansion": cfg.expansion,
                   "H": cfg.H, "W": cfg.W, "levels": cfg.levels, "keep": f"{num}/{den}",
                   "act_bits": cfg.act_bits, "act": args.act, "norm": args.norm,
                   "route": "chained" if chained else "middle tensors formed"},
        "roofline": roof,
        "stages_us": {n: round(v, 2) for n, v in stage_us.items()},
        "stages_frac_of_hbm_peak": {n: round(alg[n] / (stage_us[n] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
                                    for n in stage_us if stage_us[n] > 0 and alg.get(n)},
        "block_alg_GBs": round(sum(alg.values()) / dt / 1e9, 1),
        # the two contractions against the matrix-core peak of their operand type
        "mfma": {f"l{layer}_pointwise": {
            "flops": 2.0 * cfg.B * cfg.k * cfg.layer(layer).C_in * cfg.layer(layer).C_out,
            "achieved_tflops": round(2.0 * cfg.B * cfg.k * cfg.layer(layer).C_in * cfg.layer(layer).C_out
                                     / (stage_us[f"l{layer}_pointwise"] * 1e-6) / 1e12, 1),
            "peak_tflops": MFMA_PEAK_TFLOPS[wname],
            "frac": round(2.0 * cfg.B * cfg.k * cfg.layer(layer).C_in * cfg.layer(layer).C_out
                          / (stage_us[f"l{layer}_pointwise"] * 1e-6) / 1e12 / MFMA_PEAK_TFLOPS[wname], 4)}
            for layer in (0, 1) if stage_us.get(f"l{layer}_pointwise", 0) > 0},
        "dense_block_ms": {"framework_bf16": None if dense_ms is None else round(dense_ms, 4),
                           "framework_1x1_bf16_plus_own_depthwise_f32":
                               None if dense_fair_ms is None else round(dense_fair_ms, 4)},
        "speedup_vs_dense": {"framework_bf16": None if dense_ms is None else round(dense_ms / (dt * 1e3), 3),
                             "framework_1x1_bf16_plus_own_depthwise_f32":
                                 None if dense_fair_ms is None else round(dense_fair_ms / (dt * 1e3), 3)},
    }
    if not args.no_cpu_baseline:
        from oracle import wcc_ref
        cores = min(len(os.sched_getaffinity(0)), 16)
        wcc_ref.set_threads(cores)
        t1 = time.perf_counter()
        wcc_ref.block_forward(r["x"][:1], r["w1"].values, r["w1"].scale, r["w_dw"], r["w3"].values,
                              r["w3"].scale, cfg.levels,
                              cfg.keep_num, cfg.keep_den, cfg.act_bits)
        cpu_dt = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": round(cfg.N * cfg.C / cpu_dt / 1e9, 5), "unit": "Gpixel*ch/s",
                               "cores": cores, "kind": "oracle",
                               "sample": f"block forward of 1 of the {cfg.B} samples, {cpu_dt:.2f} s"}
    print(json.dumps(out))
    return 0


def bench_table(args, synth, wcc, torch, np) -> int:
    """Every row of the paper's timing table (batch as printed): this library's block, the fair
    dense block on the same GPU, their ratio, and the paper's ratio as context.  One JSON line."""
    rows = []
    for side, c, e, B, (num, den), paper in PAPER_TABLE:
        cfg = block_from_shape(synth, f"{side},{c},{e},{B}", num, den, args.weights)
        print(f"bench.py: {cfg.name}", file=sys.stderr, flush=True)
        r = time_block(cfg, args, synth, wcc, torch, np, dense=True)
        wcc_ms = r["dt"] * 1e3
        fair = r["dense_fair_ms"]
        rows.append({"image": side, "c_in": c, "expansion": e, "batch": B, "keep": f"{num}/{den}",
                     "route": "chained" if r["chained"] else "middle tensors formed",
                     "wcc_ms": round(wcc_ms, 4), "dense_ms": None if fair is None else round(fair, 4),
                     "speedup": None if fair is None else round(fair / wcc_ms, 3),
                     "paper_speedup_gtx1080ti": paper})
        torch.cuda.empty_cache()
    won = [r for r in rows if r["speedup"] and r["speedup"] > 1.0]
    out = {"metric": "inverted residual block, WCC vs dense on the same GPU", "unit": "ms",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
           "dtype": "int8" if args.weights == "i8" else "bf16", "act": args.act, "weights": args.weights,
           "dense": "framework bf16 1x1 convolutions + this library's fp32 depthwise kernel",
           "rows_faster_than_dense": len(won), "rows": rows}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3,
                    help="single-layer workload 1..4 (default 3, the largest), 5 = the 16-layer backbone stack, "
                         "6 = the inverted residual block of the paper's timing table")
    ap.add_argument("--keep", default="1/4", help="kept fraction for --config 5 and 6 (num/den)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--alpha", choices=["dynamic", "static"], default="dynamic",
                    help="static: the clipping parameter is passed in (the value a dynamic call "
                         "finds), as a learned alpha would be (single-layer workloads)")
    ap.add_argument("--act", choices=["f32", "bf16"], default="f32",
                    help="storage type of the feature maps x and y (bf16: a bandwidth variant; the "
                         "metric is quoted on f32)")
    ap.add_argument("--cold-input", action="store_true",
                    help="single-layer workloads: also time steps whose input was evicted from the "
                         "memory-side cache beforehand (reported as cold_input_ms_per_step)")
    ap.add_argument("--norm", choices=["l1", "l2"], default="l1",
                    help="l2: positions ranked by the sum of squares over channels (a variant; the "
                         "metric is quoted on l1)")
    ap.add_argument("--index-list", choices=["select", "prefix"], default="select",
                    help="prefix: wcc_forward_fixed with the first k positions instead of the joint "
                         "shrinkage's top-k (single-layer workloads)")
    ap.add_argument("--weights", choices=["bf16", "i8"], default="bf16",
                    help="block (--config 6, --table): storage type of the two 1x1 kernels; i8 = "
                         "8-bit codes with a scale per output channel (the paper's 8-bit weights)")
    ap.add_argument("--shape", default="", metavar="SIDE,c,e,B",
                    help="--config 6: another block shape (image side or HxW, c_in, expansion, batch)")
    ap.add_argument("--table", action="store_true",
                    help="the 24 rows of the paper's timing table, WCC and fair dense block each "
                         "(use a small --steps)")
    ap.add_argument("--no-dense-baseline", action="store_true",
                    help="--config 6: skip timing the dense block built from library convolutions")
    ap.add_argument("--launch", choices=["eager", "graph"], default="eager",
                    help="graph: the step is recorded once into a HIP graph and replayed")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="single-layer workloads: skip timing the plain read / write / copy kernels "
                         "(reported as stream_ceilings_GBs)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="R",
                    help="also run R plain device-to-device copies of the input tensor (a copy "
                         "kernel of known size, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (the path is per image, so "
              "more GPUs would each take a share of the batch)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2205_12268_amd import synth, wcc

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    wcc.lib()  # fails loudly if the HIP library is missing

    def run_layer(cfg, ctx):
        """Times args.steps forwards of one layer; returns (seconds per step, stage us, event pair us, x, w)."""
        x, w = synth.make_inputs(cfg)
        bf16 = args.act == "bf16"
        if bf16:
            x = synth.round_to_bf16(x)
        d = wcc.make_desc(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                          cfg.keep_den, cfg.w_dtype, cfg.act_bits, wcc.BF16 if bf16 else wcc.F32,
                          wcc.NORM_L2 if args.norm == "l2" else wcc.NORM_L1)
        ctx.ensure_workspace(d)
        xd = torch.from_numpy(x).cuda()
        if bf16:
            xd = xd.to(torch.bfloat16)
        stored = w.stored.view(np.int16) if w.stored.dtype == np.uint16 else w.stored
        wd = torch.from_numpy(np.ascontiguousarray(stored)).cuda()
        wsd = None if w.scale is None else torch.from_numpy(w.scale).cuda()
        y = torch.empty((cfg.B, cfg.C_out, cfg.H, cfg.W), device="cuda",
                        dtype=torch.bfloat16 if bf16 else torch.float32)

        alpha_in = 0.0
        if args.alpha == "static" and cfg.act_bits:
            a_dev = torch.zeros(1, dtype=torch.float32, device="cuda")
            if args.index_list == "prefix":
                ctx.wcc_forward_fixed(d, xd, wd, wsd, 0.0, None, y, a_dev)
            else:
                ctx.wcc_forward(d, xd, wd, wsd, 0.0, y, None, a_dev)
            alpha_in = float(a_dev.item())

        def step():
            if args.index_list == "prefix":
                ctx.wcc_forward_fixed(d, xd, wd, wsd, alpha_in, None, y)
            else:
                ctx.wcc_forward(d, xd, wd, wsd, alpha_in, y)

        if args.copy_probe:
            probe = torch.empty_like(xd)
            for _ in range(args.copy_probe):
                probe.copy_(xd)  # reads and writes xd.numel() * 4 bytes
            torch.cuda.synchronize()
            del probe
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        timed = step
        if args.launch == "graph":
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
            timed = graph.replay
            for _ in range(args.warmup):
                timed()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            timed()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        if args.cold_input:
            # the loop above finds a small x still in the 256 MB memory-side cache from the
            # step before; here 512 MB of other data are read in between (untimed), so every
            # step fetches x from HBM, as after a producer that did not leave it in the cache
            other = torch.ones(128 << 20, dtype=torch.float32, device="cuda")
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            cold = []
            for _ in range(min(args.steps, 30)):
                other.sum()
                e0.record()
                step()
                e1.record()
                e1.synchronize()
                cold.append(e0.elapsed_time(e1))
            run_layer.cold_ms = float(np.median(cold))
            del other
        # per-stage device time: the same K steps again with the library's HIP events switched
        # on (they bracket each stage on the stream the kernels run on)
        ctx.set_profiling(True)
        acc = {}
        for _ in range(args.steps):
            step()
            for name, ms in ctx.stage_times().items():
                acc[name] = acc.get(name, 0.0) + ms
        ctx.set_profiling(False)
        # an empty event bracket measures what the two records cost by themselves; take it off
        acc.pop("depthwise", None)  # a stage of the block workload only
        pair_us = 1e3 * acc.pop("event_pair") / args.steps
        stage_us = {n: max(1e3 * v / args.steps - pair_us, 0.0) for n, v in acc.items()}
        return dt, stage_us, pair_us, x, w

    if args.table:
        return bench_table(args, synth, wcc, torch, np)
    if args.config == 6:
        return bench_block(args, synth, wcc, torch, np)
    ctx = wcc.Context(0)
    if args.config == 5:
        return bench_stack(args, synth, run_layer, ctx)
    cfg = synth.config(args.config)
    dt, stage_us, pair_us, x, w = run_layer(cfg, ctx)

    pix_ch = cfg.B * cfg.H * cfg.W * cfg.C_in
    value = pix_ch / dt / 1e9
    act_bytes = 2 if args.act == "bf16" else 4
    # kept coefficients travel as 8-bit codes whenever the clipping parameter is known before the
    # second transform pass: from the caller, or from the selection (not with a fixed list)
    codes = cfg.act_bits == 8 and cfg.k % 4 == 0 and (args.alpha == "static" or args.index_list == "select")
    alg = algorithmic_bytes(cfg, act_bytes, 1 if codes else 4)
    if args.index_list == "prefix":  # no norm pass, no selection: only the rank map is written
        alg["haar_fwd"], alg["norm_select"] = 0, 4 * cfg.B * cfg.N
    # stage_us is the HIP-event bracket around each stage as recorded (it holds the kernel and its
    # launch gap); the roofline figures use it as it is, so they err on the low side, and the
    # bracket less the cost of the two event records is reported beside it
    dom = max(STAGE_KERNEL, key=lambda n: stage_us[n])  # the single kernel that takes longest
    achieved = alg[dom] / (stage_us[dom] * 1e-6) / 1e9
    prof = os.path.join(ROOT, "profiles")
    traffic = read_traffic(prof, cfg.name, STAGE_KERNEL[dom])
    x_bytes = act_bytes * pix_ch
    wname = {0: "f32", 1: "bf16", 2: "int8", 3: "int8"}[cfg.w_dtype] if cfg.act_bits == 8 else "f32"
    flops = 2.0 * cfg.B * cfg.C_in * cfg.C_out * cfg.k
    gemm_tflops = flops / (stage_us["pointwise"] * 1e-6) / 1e12
    out = {
        "metric": "WCC layer forward throughput",
        "value": round(value, 3),
        "unit": "Gpixel*ch/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(dt * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {0: "f32", 1: "bf16", 2: "int8", 3: "int8"}[cfg.w_dtype],
        "data": "synthetic",
        "launch": args.launch,
        "config": {"workload": cfg.name, "B": cfg.B, "C_in": cfg.C_in, "C_out": cfg.C_out,
                   "H": cfg.H, "W": cfg.W, "levels": cfg.levels,
                   "keep": f"{cfg.keep_num}/{cfg.keep_den}", "act_bits": cfg.act_bits,
                   "index_list": args.index_list, "alpha": args.alpha, "act": args.act,
                   "norm": args.norm},
        "roofline": {"bound": "hbm", "kernel": STAGE_KERNEL[dom], "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "algorithmic_bytes": alg[dom],
                     "kernel_us": round(stage_us[dom], 2),
                     "kernel_us_less_event_pair": round(max(stage_us[dom] - pair_us, 0.0), 2),
                     "profile_avg_us": read_profile_column(prof, "kernel_stats", cfg.name,
                                                           STAGE_KERNEL[dom], 2)},
        "stages_us": {n: round(v, 2) for n, v in stage_us.items()},
        "event_pair_us": round(pair_us, 2),
        "stages_alg_GBs": {n: round(alg[n] / (stage_us[n] * 1e-6) / 1e9, 1)
                           for n in stage_us if stage_us[n] > 0},
        "stages_frac_of_hbm_peak": {n: round(alg[n] / (stage_us[n] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
                                    for n in stage_us if stage_us[n] > 0},
        # an input that fits the memory-side cache is still there from the step before: the
        # transform passes' rates are then cache-served, not HBM rates (see --cold-input)
        "input_cache_resident": bool(x_bytes <= CACHE_BYTES),
        "layer_alg_GBs": round(sum(alg.values()) / dt / 1e9, 1),
        "layer_frac_of_hbm_peak": round(sum(alg.values()) / dt / 1e9 / HBM_PEAK_GBS, 4),
        "gemm_tflops": round(gemm_tflops, 2),
        # the contraction against the matrix-core peak of its operand type, and the counter's
        # own reading of how busy the matrix cores were (profiles/sq_counters_*.txt); the stage
        # is bound by HBM at these shapes, so its HBM fraction stands beside it
        "mfma": {"kernel": profiled_kernel_name(prof, cfg.name, "pointwise_",
                                                "pointwise_mfma_kernel"), "flops": flops,
                 "achieved_tflops": round(gemm_tflops, 2), "peak_tflops": MFMA_PEAK_TFLOPS[wname],
                 "frac": round(gemm_tflops / MFMA_PEAK_TFLOPS[wname], 4),
                 "busy_frac_counter": read_profile_column(prof, "sq_counters", cfg.name,
                                                          "pointwise_", -1),
                 "arithmetic_intensity_flop_per_byte": round(flops / alg["pointwise"], 1),
                 "frac_of_hbm_peak": round(alg["pointwise"] / (stage_us["pointwise"] * 1e-6) / 1e9
                                           / HBM_PEAK_GBS, 4)},
    }

    if not args.no_ceilings:
        from paper_2205_12268_amd import probe
        out["stream_ceilings_GBs"] = stream_ceilings(probe, torch)
    if args.cold_input:
        out["cold_input_ms_per_step"] = round(run_layer.cold_ms, 5)
    if not args.no_cpu_baseline:
        from oracle import wcc_ref
        cores = min(len(os.sched_getaffinity(0)), 16)
        wcc_ref.set_threads(cores)
        # a bounded sample of the same workload: its first image (every step of the path is per
        # image), repeated for about 10 s
        xs = x[:1]
        reps, spent = 0, 0.0
        while reps < 1 or (spent < 10.0 and reps < 50):
            t1 = time.perf_counter()
            wcc_ref.forward(xs, w.values, None if w.scale is None else w.scale, cfg.levels,
                            cfg.keep_num, cfg.keep_den, act_bits=cfg.act_bits)
            spent += time.perf_counter() - t1
            reps += 1
        cpu_dt = spent / reps
        out["cpu_baseline"] = {"value": round(pix_ch / cfg.B / cpu_dt / 1e9, 5), "unit": "Gpixel*ch/s",
                               "cores": cores, "kind": "oracle",
                               "sample": f"forward of 1 of the {cfg.B} images of {cfg.name}, "
                                         f"{reps} repetitions, {cpu_dt:.3f} s each"}
    print(json.dumps(out))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
