"""Benchmark of the MixLoRA FFN block (forward + backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--forward-only]
                    [--schedule linear_down|shared|vanilla] [--dora] [--no-cpu-baseline]

One step = one pass of the whole hot path: mixlora_ffn_forward followed by
mixlora_ffn_backward on the LLaMA-2-7B-shaped workload (T=4096 tokens, d=4096, d_ff=11008,
8 experts, top-2, rank 16, bf16), inputs resident in HBM before the timed region.
Prints ONE JSON line: tokens/s, the roofline record of the dominant kernel (the large-tile
bf16 MFMA GEMM, timed live with HIP events on its stream) and the CPU oracle's rate on a
bounded token sample of the same workload.  --workload picks the other shapes (13B-skew,
L3-8B-clusters, two adapters, decode, the attention-projection LoRA linear); --schedule runs the
paper's own shared / unshared schedules and --dora the weight-decomposed expert variant, for
comparison with the default.
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

MFMA_BF16_PEAK = 2.5e15     # dense bf16 MFMA, FLOP/s (MI355X published)
HBM_PEAK = 8.0e12           # HBM3E, B/s (MI355X published)


def flop_model(cfg, units_fwd, units_bwd):
    """Algorithmic FLOPs of one step: frozen GEMM units (one unit = 2*T*d*d_ff) plus the rank-r
    LoRA and router work of the method itself (no padding, no dense-over-all-experts work)."""
    T, d, f, N, k, r = cfg.T, cfg.d, cfg.d_ff, cfg.N, cfg.k, cfg.r
    unit = 2.0 * T * d * f
    fwd = unit * units_fwd + T * (6.0 * k * r * (d + f) + 2.0 * d * N)
    bwd = unit * units_bwd + T * (12.0 * k * r * (d + f) + 4.0 * d * N)
    return unit, fwd, bwd


def read_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (profiles/), or None when no such summary exists."""
    path = os.path.join(ROOT, "profiles", f"gemm_bf16_traffic_{workload}.txt")
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split()[1])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, host, n_tokens):
    """The oracle as it stands on the first n_tokens tokens (forward + backward)."""
    import numpy as np
    from oracle import mixlora_oracle as orc
    from paper_2404_15159_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    W = {n: np.asarray(host[n], dtype=np.float64) for n in synth.WEIGHT_NAMES}
    x = np.asarray(host["x"][:n_tokens], dtype=np.float64)
    dy = np.asarray(host["dy"][:n_tokens], dtype=np.float64)
    def once():
        if cfg.M > 1:
            tm = synth.token_model(cfg)[:n_tokens]
            orc.multi_backward(x, tm, synth.split_adapters(cfg, W), cfg.k, cfg.lora_scale, dy, None,
                               cfg.aux_coeff, "top1")
        else:
            orc.backward(x, W, cfg.k, cfg.lora_scale, dy, 1.0, cfg.aux_coeff, "top1")

    # repeat the same sample until about ten seconds of CPU work are on the clock (at most 8 runs)
    reps, t0 = 0, time.perf_counter()
    while True:
        once()
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or reps >= 8:
            break
    return {"value": reps * n_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n_tokens} of {cfg.T} tokens, forward+backward, float64 NumPy, "
                      f"{reps} runs in {dt:.1f} s"}


LINEAR_WORKLOADS = {
    # a q/k/v/o projection of the LLaMA-2-7B shape with its rank-16 adapter (alpha 32)
    "llama2_7b_attn_proj": dict(T=4096, d_in=4096, d_out=4096, r=16, lora_scale=2.0, seed_index=8),
}


def bench_linear(args):
    """Plain LoRA linear (the attention-projection form): forward + backward per step."""
    import numpy as np
    import torch
    from paper_2404_15159_amd import binding as B
    from paper_2404_15159_amd import synth
    from paper_2404_15159_amd.runner import LoraLinear

    w = LINEAR_WORKLOADS[args.workload]
    T, di, dn, r, s = w["T"], w["d_in"], w["d_out"], w["r"], w["lora_scale"]
    host = synth.make_linear_inputs(T, di, dn, r, "bf16", seed=synth.SEED_BASE + w["seed_index"])
    m = LoraLinear(T, di, dn, r, s, "bf16", host)

    def step():
        m.forward()
        m.backward()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    B.mixlora_profile_begin(args.steps * 4)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    k_ms, k_launches, k_flops_exec = B.mixlora_profile_end()
    unit = 2.0 * T * di * dn
    step_flops = 2 * unit + T * 6.0 * r * (di + dn) * 1.5   # two frozen products + rank-r work
    avg_launch_s = k_ms / 1e3 / max(k_launches, 1)
    achieved = (2 * unit / max(k_launches / args.steps, 1e-9)) / avg_launch_s if k_launches else 0.0
    out = {
        "metric": "LoRA linear fwd+bwd tokens/sec on 1 MI355X + % bf16 MFMA peak",
        "value": T / (ms_per_step / 1e3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: T={T} d_in={di} d_out={dn} r={r} bf16 forward+backward",
                   "algorithmic_tflop_per_step": step_flops / 1e12,
                   "mfma_frac_whole_step": step_flops / (ms_per_step / 1e3) / MFMA_BF16_PEAK},
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_dl_kernel<256,256,64,2 stages,8 waves>",
                     "achieved": achieved / 1e12, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK, "launches_per_step": k_launches / args.steps,
                     "avg_launch_ms": avg_launch_s * 1e3, "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import mixlora_oracle as orc
        h64 = {n: np.asarray(v, dtype=np.float64) for n, v in host.items()}
        reps, t0 = 0, time.perf_counter()
        while True:
            orc.lora_linear_forward(h64["x"], h64["W"], h64["A"], h64["B"], s)
            orc.lora_linear_backward(h64["x"], h64["W"], h64["A"], h64["B"], s, h64["dy"])
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= 10.0 or reps >= 50:
                break
        out["cpu_baseline"] = {"value": reps * T / dt, "unit": "tokens/s", "cores": os.cpu_count() or 1,
                               "kind": "oracle",
                               "sample": f"all {T} tokens, forward+backward, float64 NumPy, {reps} runs in {dt:.1f} s"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama2_7b")
    ap.add_argument("--cpu-tokens", type=int, default=4096)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--schedule", default="linear_down", choices=["linear_down", "shared", "vanilla"],
                    help="linear_down: the library's schedule (3 frozen units per direction); "
                         "shared / vanilla: the paper's Figure 3(b) / 3(a) schedules (2+k / 3k "
                         "units), for comparison")
    ap.add_argument("--dora", action="store_true",
                    help="weight-decomposed experts (magnitude / row norm on every expert "
                         "projection) through mixlora_dora_forward / _backward")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known HBM traffic, used to "
                         "scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the block would shard by tokens, data parallel, with one all-reduce of the "
              "adapter gradients per step)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2404_15159_amd import binding as B
    from paper_2404_15159_amd import synth
    from paper_2404_15159_amd.runner import MixLoraFFN

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load()   # raises if the HIP library is missing: there is no fallback path
    if args.workload in LINEAR_WORKLOADS:
        bench_linear(args)
        return
    cfg = synth.CONFIGS[args.workload]
    if cfg.dtype != "bf16":
        print("bench.py: the timed workloads are the bf16 ones", file=sys.stderr)
        sys.exit(2)
    do_bwd = not args.forward_only
    t0 = time.perf_counter()
    host = synth.make_inputs(cfg)
    t_inputs = time.perf_counter() - t0
    schedule = {"linear_down": B.SCHEDULE_LINEAR_DOWN, "shared": B.SCHEDULE_SHARED,
                "vanilla": B.SCHEDULE_VANILLA}[args.schedule]
    if args.schedule != "linear_down" and cfg.M > 1:
        print("bench.py: --schedule shared/vanilla runs one adapter", file=sys.stderr)
        sys.exit(2)
    if args.dora and (args.schedule != "linear_down" or cfg.M > 1):
        print("bench.py: --dora runs one adapter and chooses its own schedule", file=sys.stderr)
        sys.exit(2)
    m = MixLoraFFN(cfg, host, with_backward=do_bwd,
                   token_model=synth.token_model(cfg) if cfg.M > 1 else None, schedule=schedule,
                   magnitudes=synth.make_magnitudes(cfg) if args.dora else None)
    if args.dora:
        args.schedule = "shared"      # gate/up shared, down projection per routed pair

    def step():
        m.forward()
        if do_bwd:
            m.backward(d_aux=1.0)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # dominant kernel, timed live with HIP events on its launch stream
    B.mixlora_profile_begin(args.steps * 8)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    k_ms, k_launches, k_flops_exec = B.mixlora_profile_end()

    # context for the rooflines, measured live: what the matrix pipe alone sustains on
    # pseudo-random bf16 operands (register-only MFMA loop) and what a plain device copy moves
    sink = torch.empty(1 << 20, dtype=torch.float32, device="cuda:0")
    mfma_ctx = max(B.mixlora_mfma_probe(sink, sink.numel() * 4, 2, 20000) for _ in range(2))
    src = torch.empty(1 << 27, dtype=torch.int32, device="cuda:0")   # 512 MiB
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(4):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_tb_s = 4 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    del src, dst, sink

    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # frozen units per direction of the executed schedule; FLOPs are counted as executed
    U = {"linear_down": 3, "shared": 2 + cfg.k, "vanilla": 3 * cfg.k}[args.schedule]
    unit, fwd_fl, bwd_fl = flop_model(cfg, U, U)
    _, fwd_paper, bwd_paper = flop_model(cfg, 2 + cfg.k, 2 + cfg.k)
    exec_flops = fwd_fl + (bwd_fl if do_bwd else 0.0)
    _, fwd_min, bwd_min = flop_model(cfg, 3, 3)       # what the block needs at least
    step_flops = fwd_min + (bwd_min if do_bwd else 0.0)
    units_per_step = U + (U if do_bwd else 0)
    schedule_text = {
        "linear_down": "shared gate/up (2 units) + linear frozen down (1 unit) per direction; "
                       "LoRA as rank-r terms on routed pairs",
        "shared": "paper Figure 3(b): shared gate/up (2 units) + down projection per routed pair "
                  "(k units) per direction; LoRA as rank-r terms on routed pairs",
        "vanilla": "paper Figure 3(a): gate, up and down per routed pair (3k units) per direction; "
                   "LoRA as rank-r terms on routed pairs"}[args.schedule]
    launches_per_step = k_launches / args.steps
    avg_launch_s = k_ms / 1e3 / max(k_launches, 1)
    traffic = read_traffic(args.workload) if args.schedule == "linear_down" else None
    if cfg.T <= 128:
        # decode-shaped call: the frozen-projection launches stream every weight once and do
        # little arithmetic per byte, so their roofline is HBM bandwidth.  Algorithmic bytes per
        # launch: the frozen matrices (units_per_step * d * d_ff * 2 B) over the launches.
        alg_bytes_per_launch = units_per_step * cfg.d * cfg.d_ff * 2.0 / max(launches_per_step, 1e-9)
        achieved = alg_bytes_per_launch / avg_launch_s if k_launches else 0.0
        roofline = {"bound": "hbm",
                    "kernel": "gemm_bf16_dl_kernel<64 or 128 rows,64,64,4 stages> (weight streaming)",
                    "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK, "launches_per_step": launches_per_step,
                    "avg_launch_ms": avg_launch_s * 1e3, "traffic": traffic}
    else:
        alg_flops_per_launch = units_per_step * unit / max(launches_per_step, 1e-9)
        achieved = alg_flops_per_launch / avg_launch_s if k_launches else 0.0
        roofline = {"bound": "mfma", "kernel": "gemm_bf16_dl_kernel<256,256,64,2 stages,8 waves>",
                    "achieved": achieved / 1e12, "peak": MFMA_BF16_PEAK / 1e12,
                    "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK,
                    "launches_per_step": launches_per_step,
                    "avg_launch_ms": avg_launch_s * 1e3,
                    "executed_tflop_per_launch": k_flops_exec / max(k_launches, 1) / 1e12,
                    "traffic": traffic}

    out = {
        "metric": "MixLoRA FFN fwd+bwd tokens/sec on 1 MI355X + % bf16 MFMA peak",
        "value": cfg.T / (ms_per_step / 1e3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} d_ff={cfg.d_ff} N={cfg.N} "
                               f"top-{cfg.k} r={cfg.r} {'adapters=%d ' % cfg.M if cfg.M > 1 else ''}bf16 "
                               f"{'forward+backward' if do_bwd else 'forward'}",
                   "schedule": schedule_text + (
                       "; weight-decomposed experts: per-expert magnitude / row-norm factors on "
                       "gate, up and down, row norms recomputed every forward" if args.dora else ""),
                   "frozen_gemm_units_per_step": units_per_step,
                   "workspace_gib": round(m.ws_bytes / 2**30, 3),
                   "algorithmic_tflop_per_step": step_flops / 1e12,
                   "executed_schedule_tflop_per_step": exec_flops / 1e12,
                   "paper_schedule_tflop_per_step": (fwd_paper + (bwd_paper if do_bwd else 0)) / 1e12,
                   "mfma_frac_whole_step": step_flops / (ms_per_step / 1e3) / MFMA_BF16_PEAK,
                   "measured_context": {
                       "mfma_register_only_random_operands_tflops": round(mfma_ctx, 1),
                       "device_copy_read_plus_write_tb_s": round(copy_tb_s, 2)},
                   "input_generation_s": round(t_inputs, 1)},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, host, min(args.cpu_tokens, cfg.T))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
