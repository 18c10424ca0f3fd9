"""Benchmark of the CP-head hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input:
cp_head_loss_fwd followed by cp_head_loss_bwd (all gradients, unembedding not
frozen).  Inputs are resident in HBM before the timed region.  One JSON line
is printed: whole-job positions/s ("token" = one position, each predicting n
future tokens), the roofline of the dominant kernel timed with events on the
launch stream, and the fp64 CPU oracle timed on a bounded sample of the same
workload as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0
PEAK_FP32_VECTOR_TFLOPS = 157.3   # 256 compute units x 128 fp32 FMA lanes x 2 x 2.4 GHz

# HBM-side bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy) from the rocprofv3 --pmc
# runs summarised in profiles/loss_head_7b_kernel_stats.md (and ..._kept_logits_...); kernels whose counters were not separated
# there report null.
GIB = float(1 << 30)
TRAFFIC_BYTES = {
    # (workload, launch name, launches per step): L2 fills + writes per launch
    ("head_7b", "gemm_z_stats_keep", 1): (203.536 + 32.510) * GIB,       # loss_head_7b_kept_logits_kernel_stats.md
    ("head_7b", "gemm_z_stats_keep", 8): (26.849 + 4.066) * GIB,         # loss_head_7b_single_call_kernel_stats.md
    ("head_7b", "gemm_z_stats", 1): (210.580 + 1.294) * GIB,             # loss_head_7b_kernel_stats.md
    ("head_7b", "gemm_z_dz", 8): (25.455 + 7.813) * GIB,                 # loss_head_7b_kernel_stats.md
    # draft step: L2 fills of its kernels per step at B = 1, 8, 64 (profiles/draft_b8_kernel_stats.md)
    ("draft", 1): 1.985 * GIB,
    ("draft", 8): (1.0018 + 1.0106 + 0.0020 + 0.0316 + 0.0022) * GIB,
    ("draft", 64): 5.014 * GIB,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="head_7b", help="a name from synth.CONFIGS (loss workloads), or 'draft', 'draft_sequential', 'first_token', 'full_heads', 'full_heads_7b', 'distill_7b'")
    ap.add_argument("--batch", type=int, default=8, help="draft workload: rows per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-positions", type=int, default=0, help="oracle sample size (0 = one position per thread for the loss, per two threads for the full heads)")
    ap.add_argument("--frozen-u", action="store_true", help="skip dU (frozen unembedding)")
    ap.add_argument("--single-call", action="store_true",
                    help="loss workloads: time cp_head_loss_fwd_bwd (forward and backward interleaved per chunk of "
                         "positions, one chunk's logits kept as 16-bit floats in between) as the step; an extra mode "
                         "of the default run")
    ap.add_argument("--keep-logits", action="store_true",
                    help="loss workloads: time the step with CP_HEAD_KEEP_LOGITS (the forward pass keeps the logits in "
                         "HBM as 16-bit floats, the backward pass reads them instead of multiplying U y again).  The "
                         "default is the path with no materialised logits; the default run of a shared-unembedding "
                         "workload reports the other variant as an extra mode")
    ap.add_argument("--no-modes", action="store_true", help="loss workloads: skip the forward-only and frozen-unembedding timings")
    ap.add_argument("--no-draft", action="store_true", help="loss workloads: skip the appended draft-step measurements")
    return ap.parse_args()


def cpu_baseline_loss(cfg, inp, positions):
    """The oracle, as it stands, on a few positions of the same workload (forward + backward)."""
    import numpy as np
    from oracle import cp_oracle
    from paper_2410_17765_amd import synth
    cp_oracle.build()
    cores = cp_oracle.num_threads()
    S = positions or cores      # the oracle threads over positions: one each keeps every thread busy
    sel = synth.position_subset(cfg.T, S)
    H, X = inp["H"][sel], inp["X"][sel]
    t0 = time.time()
    cp_oracle.loss_fwd(H, inp["W"], inp["U"], inp["G"], X)
    cp_oracle.loss_bwd(H, inp["W"], inp["U"], inp["G"], X, np.ones(len(sel)))
    dt = time.time() - t0
    # the oracle threads over positions, so with at most one position per thread the wall time is also
    # the time one thread needs for one position
    out = {"value": len(sel) / dt, "unit": "tokens/s", "cores": min(cores, len(sel)), "kind": "oracle",
           "sample": f"{len(sel)} seeded positions of the workload at full d, V, n, r; fp64 forward + backward "
                     f"with all gradients; {dt:.1f} s wall"}
    if len(sel) <= cores:
        out["seconds_per_position_one_thread"] = dt
    return out


def bench_full(args):
    """fwd+bwd step of the full-head variant (eq. 6: a V x d matrix per future token and expert).
    `full_heads` takes its seeded inputs from synth; `full_heads_7b` is the headline shape, whose 8.4 GB of
    head weights are drawn on the device (seeded torch generator): timing only, parity is shown at `full_heads`."""
    import numpy as np
    import torch
    from paper_2410_17765_amd import binding, head, synth

    binding.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    on_device = args.workload == "full_heads_7b"
    cfg = synth.CONFIGS["head_7b"].with_(name="full_heads_7b") if on_device else synth.CONFIGS["full_heads"]
    if on_device:
        gen = torch.Generator(device=dev)
        gen.manual_seed(synth.SEED_F)
        F = torch.empty((cfg.n, cfg.r, cfg.V, cfg.d), dtype=torch.bfloat16, device=dev)
        for s in range(cfg.n):
            for a in range(cfg.r):
                F[s, a] = (torch.randn((cfg.V, cfg.d), generator=gen, device=dev) * cfg.d ** -0.5).to(torch.bfloat16)
        G = head.to_device(synth.gate(cfg), cfg.dtype)
        H = head.to_device(synth.hidden(cfg), cfg.dtype)
        X = torch.from_numpy(synth.targets(cfg)).to(dev)
        inp = None
    else:
        inp = {"H": synth.hidden(cfg), "F": synth.full_head_weights(cfg), "G": synth.gate(cfg), "X": synth.targets(cfg)}
        F, G = head.to_device(inp["F"], cfg.dtype), head.to_device(inp["G"], cfg.dtype)
        H = head.to_device(inp["H"], cfg.dtype)
        X = torch.from_numpy(inp["X"]).to(dev)
    keep = bool(args.keep_logits)
    ds = binding.make_desc(cfg.T, cfg.d, cfg.V, cfg.n, cfg.r, binding.BF16, binding.KEEP_LOGITS if keep else 0)
    ctx = torch.empty(binding.cp_head_full_ctx_bytes(ds), dtype=torch.uint8, device=dev)
    ws = torch.empty(max(binding.cp_head_workspace_bytes(ds, binding.OP_FULL_LOSS_FWD),
                         binding.cp_head_workspace_bytes(ds, binding.OP_FULL_LOSS_BWD)), dtype=torch.uint8, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    loss = torch.empty(cfg.T, **f32)
    dH = torch.empty((cfg.T, cfg.d), **f32)
    dF = torch.empty((cfg.n, cfg.r, cfg.V, cfg.d), **f32)
    dG = torch.empty((cfg.r, cfg.d), **f32)
    scale = 1.0 / cfg.T
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        binding.cp_head_full_loss_fwd(ds, H, F, G, X, loss, ctx, ws, stream)
        binding.cp_head_full_loss_bwd(ds, H, F, G, X, None, scale, ctx, dH, dF, dG, ws, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.cp_head_profile_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # on the launch stream
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    binding.cp_head_profile_enable(False)
    kernels = binding.cp_head_profile_read()
    ms_per_step = dt * 1e3 / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    gemms = [k for k in kernels if "gemm_" in k[0]]
    dom = max(gemms, key=lambda k: k[2])
    achieved = dom[3] / (dom[2] * 1e-3) / 1e12
    model_flops = 6.0 * cfg.n * cfg.r * cfg.d * cfg.V * cfg.T
    out = {
        "metric": "CP-head (full heads) fwd+bwd tokens/s", "value": cfg.T * args.steps / dt, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic (head weights drawn on the device)" if on_device else "synthetic",
        "config": {"workload": cfg.name, "T": cfg.T, "d": cfg.d, "V": cfg.V, "n": cfg.n, "r": cfg.r,
                   "token": "one position (n future tokens each)",
                   "logits": "kept in HBM between forward and backward" if keep else "never stored (recomputed in the backward pass)",
                   "ctx_gib": ctx.numel() / GIB},
        "model_tflops": model_flops / (ms_per_step * 1e-3) / 1e12,
        "model_flop_frac_of_bf16_peak": model_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "mean_loss": float(loss.mean()),
        "roofline": {"bound": "mfma", "kernel": dom[0], "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None, "launches": dom[1],
                     "avg_ms": dom[2] / dom[1]},
        "kernels": [{"name": k[0], "launches": k[1], "ms_per_step": k[2] / args.steps,
                     "rate": (k[3] / (k[2] * 1e-3) / 1e12) if k[2] > 0 else None,
                     "rate_unit": "TFLOP/s" if "gemm_" in k[0] else "TB/s"} for k in kernels],
    }
    if inp is not None and not args.no_cpu_baseline:
        from oracle import cp_oracle
        cp_oracle.build()
        cores = cp_oracle.num_threads()
        sel = synth.position_subset(cfg.T, args.cpu_positions or max(1, cores // 2))
        t0 = time.time()
        cp_oracle.full_loss_fwd(inp["H"][sel], inp["F"], inp["G"], inp["X"][sel])
        cp_oracle.full_loss_bwd(inp["H"][sel], inp["F"], inp["G"], inp["X"][sel], np.ones(len(sel)))
        dtc = time.time() - t0
        out["cpu_baseline"] = {"value": len(sel) / dtc, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "sample": f"{len(sel)} seeded positions of the workload at full d, V, n, r; fp64 forward "
                                         f"+ backward with all gradients; {dtc:.1f} s wall"}
    return out


def bench_distill(args):
    """fwd+bwd step of the head-only fine-tuning loss (eq. 14) at the headline shape, unembedding frozen
    (dU = NULL), beta = 0.9, discount = 0.8.  The 4.2 GB of teacher logits are drawn on the device (seeded
    torch generator, N(0, 1.5^2)): timing only, parity is shown by the tests on seeded host inputs."""
    import torch
    from paper_2410_17765_amd import binding, head, synth

    binding.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.CONFIGS["head_7b"]
    inp = synth.make_inputs(cfg)
    keep = bool(args.keep_logits)
    h = head.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype, flags=binding.KEEP_LOGITS if keep else 0)
    H = head.to_device(inp["H"], cfg.dtype)
    X = torch.from_numpy(inp["X"]).to(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED_TEACHER)
    TZ = torch.empty((cfg.T, cfg.n, cfg.V), dtype=torch.bfloat16, device=dev)
    for t0 in range(0, cfg.T, 2048):
        TZ[t0:t0 + 2048] = (torch.randn((min(2048, cfg.T - t0), cfg.n, cfg.V), generator=gen, device=dev) * 1.5).to(torch.bfloat16)
    ds = h.desc(cfg.T)
    ctx = torch.empty(binding.cp_head_distill_ctx_bytes(ds), dtype=torch.uint8, device=dev)
    ws = torch.empty(max(binding.cp_head_workspace_bytes(ds, binding.OP_DISTILL_FWD),
                         binding.cp_head_workspace_bytes(ds, binding.OP_DISTILL_BWD)), dtype=torch.uint8, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    loss = torch.empty(cfg.T, **f32)
    dH = torch.empty((cfg.T, cfg.d), **f32)
    dW = torch.empty((cfg.n, cfg.r, cfg.d, cfg.d), **f32)
    dG = torch.empty((cfg.r, cfg.d), **f32)
    scale = 1.0 / cfg.T
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        binding.cp_head_distill_loss_fwd(ds, H, h.W, h.U, h.G, X, TZ, 0.9, 0.8, loss, ctx, ws, stream)
        binding.cp_head_distill_loss_bwd(ds, H, h.W, h.U, h.G, X, TZ, None, scale, ctx, dH, dW, None, dG, ws, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.cp_head_profile_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # on the launch stream
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    binding.cp_head_profile_enable(False)
    kernels = binding.cp_head_profile_read()
    ms_per_step = dt * 1e3 / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    gemms = [k for k in kernels if "gemm_" in k[0]]
    dom = max(gemms, key=lambda k: k[2])
    achieved = dom[3] / (dom[2] * 1e-3) / 1e12
    # algorithmic products: y, z, dY, dH, dW (without kept logits the hardware multiplies U y twice more)
    model_flops = (2.0 * cfg.n * cfg.r * cfg.d * (3 * cfg.d + 2 * cfg.V)) * cfg.T
    return {
        "metric": "CP-head fine-tuning loss fwd+bwd tokens/s", "value": cfg.T * args.steps / dt, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic (teacher logits drawn on the device)",
        "config": {"workload": "distill_7b", "T": cfg.T, "d": cfg.d, "V": cfg.V, "n": cfg.n, "r": cfg.r,
                   "beta": 0.9, "discount": 0.8, "frozen_u": True, "token": "one position (n future tokens each)",
                   "logits": "kept in HBM between forward and backward" if keep else "never stored (recomputed twice)",
                   "ctx_gib": ctx.numel() / GIB},
        "model_tflops": model_flops / (ms_per_step * 1e-3) / 1e12,
        "model_flop_frac_of_bf16_peak": model_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "mean_loss": float(loss.mean()),
        "roofline": {"bound": "mfma", "kernel": dom[0], "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None, "launches": dom[1],
                     "avg_ms": dom[2] / dom[1]},
        "kernels": [{"name": k[0], "launches": k[1], "ms_per_step": k[2] / args.steps,
                     "rate": (k[3] / (k[2] * 1e-3) / 1e12) if k[2] > 0 else None,
                     "rate_unit": "TFLOP/s" if "gemm_" in k[0] else "TB/s"} for k in kernels],
    }


def bench_loss(args):
    import numpy as np
    import torch
    from paper_2410_17765_amd import binding, head, synth

    cfg = synth.CONFIGS[args.workload]
    binding.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    t0 = time.time()
    inp = synth.make_inputs(cfg)
    print(f"[bench] inputs for {cfg.name} generated in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    keep = cfg.dtype == "bf16" and bool(args.keep_logits)
    h = head.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype, flags=binding.KEEP_LOGITS if keep else 0)
    H = head.to_device(inp["H"], cfg.dtype)
    X = torch.from_numpy(inp["X"]).to(dev)
    ds = h.desc(cfg.T)                                                                  # the timed step's variant
    ds_plain = binding.make_desc(cfg.T, cfg.d, cfg.V, cfg.n, cfg.r, ds.dtype, 0)         # no materialised logits
    ds_keep = binding.make_desc(cfg.T, cfg.d, cfg.V, cfg.n, cfg.r, ds.dtype, binding.KEEP_LOGITS)
    both = cfg.dtype == "bf16" and not args.no_modes                                    # the other variant as a mode
    ctx_bytes = binding.cp_head_ctx_bytes(ds)
    ctx = torch.empty(max(ctx_bytes, binding.cp_head_ctx_bytes(ds_keep) if both else 0), dtype=torch.uint8, device=dev)
    ws_bytes = max(binding.cp_head_workspace_bytes(dsc, op) for dsc in (ds_plain, ds_keep)
                   for op in (binding.OP_LOSS_FWD, binding.OP_LOSS_BWD))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    loss = torch.empty(cfg.T, **f32)
    dH = torch.empty((cfg.T, cfg.d), **f32)
    dW = torch.empty((cfg.n, cfg.r, cfg.d, cfg.d), **f32)
    dU = None if args.frozen_u else torch.empty((cfg.V, cfg.d), **f32)
    dG = torch.empty((cfg.r, cfg.d), **f32)
    scale = 1.0 / cfg.T
    stream = torch.cuda.current_stream().cuda_stream

    single = cfg.dtype == "bf16" and bool(args.single_call)
    if single:
        ws_step = binding.cp_head_workspace_bytes(ds_plain, binding.OP_LOSS_FWD_BWD)
        if ws_step > ws.numel():
            del ws
            ws = torch.empty(ws_step, dtype=torch.uint8, device=dev)

    def step():
        if single:
            binding.cp_head_loss_fwd_bwd(ds_plain, H, h.W, h.U, h.G, X, None, scale, loss, dH, dW, dU, dG, ws, stream)
            return
        binding.cp_head_loss_fwd(ds, H, h.W, h.U, h.G, X, loss, ctx, ws, stream)
        binding.cp_head_loss_bwd(ds, H, h.W, h.U, h.G, X, None, scale, ctx, dH, dW, dU, dG, ws, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.cp_head_profile_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # on the launch stream
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    binding.cp_head_profile_enable(False)
    kernels = binding.cp_head_profile_read()
    ms_per_step = dt * 1e3 / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    value = cfg.T * args.steps / dt
    mean_loss = float(loss.mean())

    # roofline of the dominant matrix-product kernel: algorithmic FLOPs of its launches / their summed duration
    model_flops = 6.0 * cfg.n * cfg.r * cfg.d * (cfg.d + cfg.V) * cfg.T
    if args.frozen_u:
        model_flops = 2.0 * cfg.n * cfg.r * cfg.d * (3 * cfg.d + 2 * cfg.V) * cfg.T
    gemms = [k for k in kernels if k[0].startswith("gemm_")]
    if gemms:
        dom = max(gemms, key=lambda k: k[2])
        achieved = dom[3] / (dom[2] * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": dom[0], "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_TFLOPS,
                "traffic": TRAFFIC_BYTES.get((cfg.name, dom[0], dom[1] // max(args.steps, 1))),
                "traffic_unit": "bytes per launch", "launches": dom[1], "avg_ms": dom[2] / dom[1]}
    else:
        # the plain fp32 path (fp32 storage or shapes off the matrix-core path: the small parity workloads): plain
        # vector arithmetic, the whole step against the fp32 vector peak
        achieved = model_flops / (ms_per_step * 1e-3) / 1e12
        roof = {"bound": "alu", "kernel": "plain fp32 path, whole step", "achieved": achieved, "peak": PEAK_FP32_VECTOR_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_VECTOR_TFLOPS, "traffic": None,
                "traffic_unit": "bytes per launch", "launches": args.steps, "avg_ms": ms_per_step}
    out = {
        "metric": "CP-head fwd+bwd tokens/s", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": cfg.name, "T": cfg.T, "d": cfg.d, "V": cfg.V, "n": cfg.n, "r": cfg.r,
                   "frozen_u": bool(args.frozen_u), "token": "one position (n future tokens each)",
                   "logits": ("one chunk of positions at a time kept in HBM between its forward and backward halves" if single
                              else "kept in HBM between forward and backward" if keep
                              else "never stored (recomputed in the backward pass)"),
                   "call": "cp_head_loss_fwd_bwd" if single else "cp_head_loss_fwd + cp_head_loss_bwd",
                   "ctx_gib": ctx_bytes / GIB},
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "predicted_tokens_per_s": value * cfg.n,      # every position predicts n tokens
        "model_tflops": model_flops / (ms_per_step * 1e-3) / 1e12,
        "model_flop_frac_of_bf16_peak": model_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "hardware_flop_frac_of_bf16_peak": sum(k[3] for k in gemms) / args.steps / (ms_per_step * 1e-3) / 1e12
                                           / PEAK_BF16_TFLOPS,
        "mean_loss": mean_loss,
        "roofline": roof,
        "kernels": [{"name": k[0], "launches": k[1], "ms_per_step": k[2] / args.steps,
                     "rate": (k[3] / (k[2] * 1e-3) / 1e12) if k[2] > 0 else None,
                     "rate_unit": "TFLOP/s" if k[0].startswith("gemm_") else "TB/s"} for k in kernels],
    }
    # the same workload in the two other modes the method is used in: forward only (evaluation), and
    # backward with the shared unembedding frozen (head-only fine tuning: no dU product)
    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    fwd_flops = 2.0 * cfg.n * cfg.r * cfg.d * (cfg.d + cfg.V) * cfg.T
    if not args.no_modes:
        # evaluation keeps no logits: the forward call alone runs without CP_HEAD_KEEP_LOGITS
        t_fwd = timed(lambda: binding.cp_head_loss_fwd(ds_plain, H, h.W, h.U, h.G, X, loss, ctx, ws, stream))
        out["forward_only"] = {"ms_per_step": t_fwd * 1e3, "tokens_per_s": cfg.T / t_fwd,
                               "model_tflops": fwd_flops / t_fwd / 1e12}
        # backward alone, on the ctx of a forward call of the timed step's kind
        binding.cp_head_loss_fwd(ds, H, h.W, h.U, h.G, X, loss, ctx, ws, stream)
        t_bwd = timed(lambda: binding.cp_head_loss_bwd(ds, H, h.W, h.U, h.G, X, None, scale, ctx, dH, dW, dU, dG, ws,
                                                       stream))
        out["backward_only"] = {"ms_per_step": t_bwd * 1e3, "model_tflops": (model_flops - fwd_flops) / t_bwd / 1e12}
    if not args.frozen_u and not args.no_modes:
        def frozen_step():
            binding.cp_head_loss_fwd(ds, H, h.W, h.U, h.G, X, loss, ctx, ws, stream)
            binding.cp_head_loss_bwd(ds, H, h.W, h.U, h.G, X, None, scale, ctx, dH, dW, None, dG, ws, stream)
        t_fr = timed(frozen_step)
        fr_flops = 2.0 * cfg.n * cfg.r * cfg.d * (3 * cfg.d + 2 * cfg.V) * cfg.T
        out["frozen_u"] = {"ms_per_step": t_fr * 1e3, "tokens_per_s": cfg.T / t_fr,
                           "model_tflops": fr_flops / t_fr / 1e12,
                           "model_flop_frac_of_bf16_peak": fr_flops / t_fr / 1e12 / PEAK_BF16_TFLOPS}
    if both:
        # the same step in the other variant: logits kept in HBM as 16-bit floats for the backward pass (an opt-in
        # trade of HBM capacity for the recompute product; it materialises the logits, so it is not the headline),
        # or, under --keep-logits, the default with no materialised logits
        ds_other = ds_plain if keep else ds_keep

        def other_step():
            binding.cp_head_loss_fwd(ds_other, H, h.W, h.U, h.G, X, loss, ctx, ws, stream)
            binding.cp_head_loss_bwd(ds_other, H, h.W, h.U, h.G, X, None, scale, ctx, dH, dW, dU, dG, ws, stream)
        t_o = timed(other_step)
        out["recompute_logits" if keep else "kept_logits"] = {
            "ms_per_step": t_o * 1e3, "tokens_per_s": cfg.T / t_o, "ctx_gib": binding.cp_head_ctx_bytes(ds_other) / GIB,
            "model_flop_frac_of_bf16_peak": model_flops / t_o / 1e12 / PEAK_BF16_TFLOPS}
    if both:
        # the single-call training step: forward and backward interleaved per chunk of positions, the logits of one
        # chunk (at most 4 GiB here, whatever T is) kept as 16-bit floats between the two halves.  It multiplies U y
        # once per step like the kept-logits pair, without a buffer that grows with the batch; logits do reach HBM, a
        # bounded chunk at a time, so this is an extra mode too and never the headline value.
        ws_step = binding.cp_head_workspace_bytes(ds_plain, binding.OP_LOSS_FWD_BWD)
        if ws_step > ws.numel():
            del ws
            torch.cuda.empty_cache()
            ws = torch.empty(ws_step, dtype=torch.uint8, device=dev)
        t_s = timed(lambda: binding.cp_head_loss_fwd_bwd(ds_plain, H, h.W, h.U, h.G, X, None, scale, loss, dH, dW, dU, dG,
                                                         ws, stream))
        out["single_call_step"] = {
            "ms_per_step": t_s * 1e3, "tokens_per_s": cfg.T / t_s, "workspace_gib": ws_step / GIB,
            "model_flop_frac_of_bf16_peak": model_flops / t_s / 1e12 / PEAK_BF16_TFLOPS}
    del ws, ctx, dW, dH, dU, H, h
    torch.cuda.empty_cache()
    if not args.no_draft:
        # the forward-only draft step of the same method (its own workload shape), as extra context
        out["draft"] = []
        for B in (1, 8, 64):
            a = argparse.Namespace(**vars(args))
            a.batch, a.steps, a.warmup = B, 20, 3
            dr = bench_draft(a)
            rf = dr["roofline"]
            out["draft"].append({"B": B, "ms_per_step": dr["ms_per_step"], "ms_per_step_graph": dr["ms_per_step_graph"],
                                 "bound": rf["bound"], "achieved": rf["achieved"], "unit": rf["unit"],
                                 "frac_of_bound_peak": rf["frac"], "hbm_gbs": rf["hbm_gbs"],
                                 "mfma_tflops": rf["mfma_tflops"], "config": dr["config"]})
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_loss(cfg, inp, args.cpu_positions)
    return out


_DRAFT_CACHE = {}


def bench_draft(args, mode="draft"):
    """Latency of one forward-only step at the draft workload's shape.  mode: "draft" (expert first),
    "draft_sequential" (the paper-form sampler, eq. 11-13) or "first_token" (eq. 11 over the vocabulary)."""
    import numpy as np
    import torch
    from paper_2410_17765_amd import binding, head, synth

    cfg = synth.CONFIGS["draft"].with_(T=args.batch)
    binding.lib()
    dev = torch.device("cuda:0")
    if "head" not in _DRAFT_CACHE:      # the weights do not depend on the batch size
        full = synth.CONFIGS["draft"].with_(T=64)
        inp = synth.make_inputs(full)
        _DRAFT_CACHE["head"] = head.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype)
        _DRAFT_CACHE["H"] = inp["H"]
    h = _DRAFT_CACHE["head"]
    H = head.to_device(_DRAFT_CACHE["H"][:cfg.T], cfg.dtype)
    un = synth.uniforms(cfg.T, cfg.n)
    ds = h.desc(cfg.T)
    op = {"draft": binding.OP_DRAFT, "draft_sequential": binding.OP_DRAFT_SEQUENTIAL,
          "first_token": binding.OP_FIRST_TOKEN}[mode]
    ws = torch.empty(binding.cp_head_workspace_bytes(ds, op), dtype=torch.uint8, device=dev)
    alpha = torch.zeros(cfg.T, dtype=torch.int32, device=dev)          # not every mode writes all three
    tokens = torch.zeros((cfg.T, cfg.n), dtype=torch.int32, device=dev)
    logq = torch.zeros(cfg.T, dtype=torch.float32, device=dev)
    weight_bytes = 2.0 * cfg.n * cfg.r * cfg.d * cfg.d + 2.0 * cfg.V * cfg.d
    if mode == "draft":
        u = torch.from_numpy(un).to(dev)
        call = lambda st: binding.cp_head_draft_sample(ds, H, h.W, h.U, h.G, u, alpha, tokens, logq, ws, st)
    elif mode == "draft_sequential":
        u = torch.from_numpy(np.ascontiguousarray(un[:, 1:])).to(dev)
        call = lambda st: binding.cp_head_draft_sample_sequential(ds, H, h.W, h.U, h.G, u, tokens, logq, ws, st)
    else:
        # only the first head's matrices are read; the [B,V] output and the stored logits of its r rows are
        # written once and the logits read twice (log-normaliser, mixture)
        logp = torch.empty((cfg.T, cfg.V), dtype=torch.float32, device=dev)
        weight_bytes = 2.0 * cfg.r * cfg.d * cfg.d + 2.0 * cfg.V * cfg.d + 4.0 * cfg.T * cfg.V * (1 + 3 * cfg.r)
        call = lambda st: binding.cp_head_first_token_logprob(ds, H, h.W, h.U, h.G, logp, ws, st)
        logq = logp     # the output whose graph replays are compared below
    stream = torch.cuda.current_stream().cuda_stream
    step = lambda: call(stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt * 1e3 / args.steps
    # the same step replayed from a HIP graph, as a serving loop would issue it (the call only launches
    # kernels on the stream it is given, so it can be captured); every replay is checked against the eager result
    ref = (alpha.clone(), tokens.clone(), logq.clone())
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call(side.cuda_stream)
    graph_ok = True
    for _ in range(3):
        alpha.zero_(); tokens.zero_(); logq.zero_()
        graph.replay()
        torch.cuda.synchronize()
        graph_ok = graph_ok and bool((alpha == ref[0]).all() and (tokens == ref[1]).all() and (logq == ref[2]).all())
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_graph = (time.perf_counter() - t0) * 1e3 / args.steps
    # per-kernel times from a second, event-instrumented pass (kept out of the latency above)
    binding.cp_head_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    binding.cp_head_profile_enable(False)
    kernels = binding.cp_head_profile_read()
    gbs = weight_bytes / (ms * 1e-3) / 1e9
    # which roofline bounds the step: streaming the weights once (HBM), or the matrix work of y and z, which grows
    # with the batch (B = 64 at the draft shape: 2.2 TFLOP, 0.86 ms at the bf16 peak against 0.27 ms of streaming)
    heads = cfg.r if mode == "first_token" else cfg.n * cfg.r
    flops = 2.0 * cfg.T * heads * cfg.d * (cfg.d + cfg.V)
    tflops = flops / (ms * 1e-3) / 1e12
    if flops / (PEAK_BF16_TFLOPS * 1e12) > weight_bytes / (PEAK_HBM_GBS * 1e9):
        roof = {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": tflops / PEAK_BF16_TFLOPS}
    else:
        roof = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
    roof.update({"traffic": TRAFFIC_BYTES.get((mode, cfg.T)), "traffic_unit": "bytes per step",
                 "hbm_gbs": gbs, "mfma_tflops": tflops})
    return {
        "metric": {"draft": "CP-head draft step latency", "draft_sequential": "CP-head sequential draft step latency",
                   "first_token": "CP-head first-token marginal latency"}[mode], "value": ms, "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": mode, "B": cfg.T, "d": cfg.d, "V": cfg.V, "n": cfg.n, "r": cfg.r},
        "ms_per_step_graph": ms_graph, "graph_replays_match_eager": graph_ok,
        "graph_gbs": weight_bytes / (ms_graph * 1e-3) / 1e9,
        "roofline": roof,
        "kernels": [{"name": k[0], "launches": k[1], "ms_per_step": k[2] / args.steps} for k in kernels],
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)
    if args.workload in ("draft", "draft_sequential", "first_token"):
        out = bench_draft(args, args.workload)
    elif args.workload in ("full_heads", "full_heads_7b"):
        out = bench_full(args)
    elif args.workload == "distill_7b":
        out = bench_distill(args)
    else:
        out = bench_loss(args)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
