"""Benchmark of the MixLoRA FFN block (forward + backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--forward-only]
                    [--schedule linear_down|shared|vanilla] [--dora] [--no-cpu-baseline]

One step = one pass of the whole hot path: mixlora_ffn_forward followed by
mixlora_ffn_backward on the LLaMA-2-7B-shaped workload (T=4096 tokens, d=4096, d_ff=11008,
8 experts, top-2, rank 16, bf16), inputs resident in HBM before the timed region.
Prints ONE JSON line: tokens/s (wall clock over the K timed steps; median and minimum of the
per-step HIP-event times beside it), the roofline record of the dominant kernel (the large-tile
bf16 MFMA GEMM, timed live with HIP events on its stream), achieved GB/s of the bandwidth-bound
kernel families, the other LLaMA-shaped workloads (7B forward only, 13B with skewed load, LLaMA-3
8B with clustered tokens) at a few steps each, and the CPU oracle's rate on a bounded token
sample of the same workload with the HIP path's errors against it.  --workload picks the other shapes (13B-skew,
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


def kernel_source_id():
    """First 16 hex digits of the SHA-256 of the GEMM kernel's source file."""
    import hashlib
    path = os.path.join(ROOT, "paper_2404_15159_amd", "csrc", "gemm.hip")
    with open(path, "rb") as fh:
        return hashlib.sha256(fh.read()).hexdigest()[:16]


def read_traffic(workload):
    """(HBM bytes per launch of the dominant kernel, note) from the committed rocprofv3 --pmc
    summary under profiles/.  The summary names the kernel source it was measured on; when that
    differs from the source in the tree the figure is stale and None is returned instead."""
    name = f"gemm_bf16_traffic_{workload}.txt"
    path = os.path.join(ROOT, "profiles", name)
    value, src = None, None
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch"):
                    value = float(line.split()[1])
                if line.startswith("kernel_source_sha256_16"):
                    src = line.split()[1]
    except OSError:
        return None, "no counter summary committed for this workload"
    if value is None:
        return None, f"profiles/{name} holds no traffic figure"
    if src != kernel_source_id():
        return None, f"profiles/{name} was measured on another version of csrc/gemm.hip"
    return value, f"profiles/{name} (kernel source {src})"


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
            return orc.multi_backward(x, tm, synth.split_adapters(cfg, W), cfg.k, cfg.lora_scale,
                                      dy, None, cfg.aux_coeff, "top1")
        return orc.backward(x, W, cfg.k, cfg.lora_scale, dy, 1.0, cfg.aux_coeff, "top1")

    # repeat the same sample until about ten seconds of CPU work are on the clock (at most 8 runs)
    reps, t0 = 0, time.perf_counter()
    while True:
        last = once()
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or reps >= 8:
            break
    rec = {"value": reps * n_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": f"first {n_tokens} of {cfg.T} tokens, forward+backward, float64 NumPy, "
                     f"{reps} runs in {dt:.1f} s"}
    return rec, last


def parity_errors(res, bw):
    """max|delta| / max|ref| of the HIP path's outputs against the oracle run of cpu_baseline (all
    tokens, tokens routed alike), plus the number of tokens routed differently."""
    import numpy as np
    fw = bw["forward"]
    same = (res["topk_idx"] == fw["topk_idx"]).all(axis=1)
    out = {"tokens_routed_differently": int((~same).sum())}

    def rel(a, b):
        den = float(np.abs(b).max())
        return float(np.abs(np.asarray(a, dtype=np.float64) - b).max() / den) if den else 0.0

    out["y"] = rel(res["y"][same], fw["y"][same])
    if "dx" in res:
        out["dx"] = rel(res["dx"][same], bw["dx"][same])
        for n in ("dA_gate", "dB_gate", "dA_up", "dB_up", "dA_down", "dB_down", "dW_router"):
            out[n] = rel(res[n], bw[n])
    out["aux_loss"] = abs(res["aux_loss"] - fw["aux_loss"]) / abs(fw["aux_loss"])
    return {k: (v if isinstance(v, int) else float(f"{v:.3e}")) for k, v in out.items()}


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


def timed_steps(step, steps, warmup):
    """Warm-up, then exactly `steps` steps between two synchronisations (wall clock), with one
    HIP event after every step on the stream the kernels are launched on.  Returns
    (wall ms per step, median and minimum of the per-step event times in ms)."""
    import torch
    for _ in range(warmup):
        step()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) / steps * 1e3
    per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    return wall_ms, per[len(per) // 2], per[0]


def profile_kinds(step, steps):
    """One more pass of `steps` steps with every launch bracketed by HIP events inside the
    library; returns {kind: (ms per step, launches per step, declared work per step)}."""
    import torch
    from paper_2404_15159_amd import binding as B
    B.mixlora_profile_begin(steps * 64)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    B.mixlora_profile_end()
    out = {}
    for i, name in enumerate(B.PROFILE_KINDS):
        ms, n, work = B.mixlora_profile_kind(i)
        out[name] = (ms / steps, n / steps, work / steps)
    return out


def matmul_context(cfg):
    """torch.matmul (the vendor GEMM library) in bf16 on the four frozen-projection launch shapes
    of this workload, TFLOP/s: context for what a GEMM reaches on this machine, never on the product
    path."""
    import torch
    T, d, f = cfg.T, cfg.d, cfg.d_ff
    shapes = {"gate_up_T_x_2f_x_d": (T, 2 * f, d), "down_T_x_d_x_f": (T, d, f),
              "dy_Wdown_T_x_f_x_d": (T, f, d), "dx_T_x_d_x_2f": (T, d, 2 * f)}
    out = {}
    for name, (M, N, K) in shapes.items():
        a = torch.randn(M, K, device="cuda:0", dtype=torch.bfloat16)
        b = torch.randn(N, K, device="cuda:0", dtype=torch.bfloat16) * 0.02
        for _ in range(3):
            c = a @ b.t()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
        ev[0].record()
        for i in range(10):
            c = a @ b.t()
            ev[i + 1].record()
        torch.cuda.synchronize()
        per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(10))
        out[name] = round(2.0 * M * N * K / (per[5] * 1e-3) / 1e12, 1)
        del a, b, c
    return out


def other_workload(name, forward_only, steps, warmup, host=None):
    """A short run of another workload: ms per step (wall, median, min), tokens/s, fraction of
    the bf16 MFMA peak over the step and of the GEMM launches."""
    import torch
    from paper_2404_15159_amd import synth
    from paper_2404_15159_amd.runner import MixLoraFFN
    cfg = synth.CONFIGS[name]
    host = host if host is not None else synth.make_inputs(cfg)
    m = MixLoraFFN(cfg, host, with_backward=not forward_only)

    def step():
        m.forward()
        if not forward_only:
            m.backward(d_aux=1.0)

    wall, med, mn = timed_steps(step, steps, warmup)
    kinds = profile_kinds(step, steps)
    unit, fwd_fl, bwd_fl = flop_model(cfg, 3, 3)
    fl = fwd_fl + (0.0 if forward_only else bwd_fl)
    g_ms, g_n, g_fl = kinds["gemm"]
    units = 3 if forward_only else 6
    rec = {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} d_ff={cfg.d_ff} N={cfg.N} top-{cfg.k} "
                       f"r={cfg.r} bf16 {'forward' if forward_only else 'forward+backward'}",
           "steps": steps, "ms_per_step": round(wall, 4), "step_ms_median": round(med, 4),
           "step_ms_min": round(mn, 4), "tokens_per_s": round(cfg.T / (wall / 1e3), 1),
           "mfma_frac_whole_step": round(fl / (wall / 1e3) / MFMA_BF16_PEAK, 4),
           "gemm_frac_of_peak": round(units * unit / (g_ms / 1e3) / MFMA_BF16_PEAK, 4) if g_ms else None,
           "non_gemm_ms_per_step": round(sum(v[0] for k, v in kinds.items() if k != "gemm"), 4)}
    del m
    torch.cuda.empty_cache()
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama2_7b")
    ap.add_argument("--cpu-tokens", type=int, default=4096)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other LLaMA-shaped workloads")
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

    # the timed region: W warm-up steps, then exactly K steps between two synchronisations
    ms_per_step, step_med, step_min = timed_steps(step, args.steps, args.warmup)

    # every kernel family, timed live with HIP events on its launch stream (a separate pass)
    kinds = profile_kinds(step, args.steps)
    k_ms, launches_per_step, k_flops_exec = kinds["gemm"]

    # context for the rooflines, measured live: what the matrix pipe alone sustains on
    # pseudo-random bf16 operands (register-only MFMA loop), what a plain device copy moves and
    # what the vendor GEMM library reaches on the same launch shapes
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
    mm_ctx = matmul_context(cfg) if cfg.T > 128 else None

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
    avg_launch_s = k_ms / 1e3 / max(launches_per_step, 1e-9)
    traffic, traffic_note = (read_traffic(args.workload) if args.schedule == "linear_down"
                             else (None, "counter summaries cover the default schedule only"))
    if cfg.T <= 128:
        # decode-shaped call: the frozen-projection launches stream every weight once and do
        # little arithmetic per byte, so their roofline is HBM bandwidth.  Algorithmic bytes per
        # launch: the frozen matrices (units_per_step * d * d_ff * 2 B) over the launches.
        alg_bytes_per_launch = units_per_step * cfg.d * cfg.d_ff * 2.0 / max(launches_per_step, 1e-9)
        achieved = alg_bytes_per_launch / avg_launch_s if launches_per_step else 0.0
        roofline = {"bound": "hbm",
                    "kernel": "gemm_bf16_dl_kernel<64 or 128 rows,64,64,4 stages> (weight streaming)",
                    "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK, "launches_per_step": launches_per_step,
                    "avg_launch_ms": avg_launch_s * 1e3, "traffic": traffic,
                    "traffic_source": traffic_note}
    else:
        alg_flops_per_launch = units_per_step * unit / max(launches_per_step, 1e-9)
        achieved = alg_flops_per_launch / avg_launch_s if launches_per_step else 0.0
        roofline = {"bound": "mfma", "kernel": "gemm_bf16_dl_kernel<256,256,64,2 stages,8 waves>",
                    "achieved": achieved / 1e12, "peak": MFMA_BF16_PEAK / 1e12,
                    "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK,
                    "launches_per_step": launches_per_step,
                    "avg_launch_ms": avg_launch_s * 1e3,
                    "executed_tflop_per_launch": k_flops_exec / max(launches_per_step, 1e-9) / 1e12,
                    "traffic": traffic, "traffic_source": traffic_note}

    # bandwidth-bound kernel families: algorithmic bytes (as declared at each launch site in
    # csrc/api.hip) over the HIP-event time of their launches, against the HBM peak
    hbm_kernels = {}
    for name in ("fused_forward", "fused_backward", "combine", "gradient_sums"):
        ms, n, work = kinds[name]
        if n:
            hbm_kernels[name] = {"ms_per_step": round(ms, 4), "launches_per_step": n,
                                 "algorithmic_mb_per_step": round(work / 1e6, 1),
                                 "achieved_gb_s": round(work / (ms * 1e-3) / 1e9, 1),
                                 "frac_of_hbm_peak": round(work / (ms * 1e-3) / HBM_PEAK, 3)}
    small_ms = kinds["routing"][0] + kinds["other"][0]

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
                   "step_ms_median": round(step_med, 4), "step_ms_min": round(step_min, 4),
                   "tokens_per_s_at_median": round(cfg.T / (step_med / 1e3), 1),
                   "algorithmic_tflop_per_step": step_flops / 1e12,
                   "executed_schedule_tflop_per_step": exec_flops / 1e12,
                   "paper_schedule_tflop_per_step": (fwd_paper + (bwd_paper if do_bwd else 0)) / 1e12,
                   "mfma_frac_whole_step": step_flops / (ms_per_step / 1e3) / MFMA_BF16_PEAK,
                   "gemm_ms_per_step": round(k_ms, 4),
                   "hbm_kernels": hbm_kernels,
                   "routing_and_small_launches_ms_per_step": round(small_ms, 4),
                   "measured_context": {
                       "mfma_register_only_random_operands_tflops": round(mfma_ctx, 1),
                       "device_copy_read_plus_write_tb_s": round(copy_tb_s, 2),
                       "torch_matmul_bf16_tflops": mm_ctx},
                   "input_generation_s": round(t_inputs, 1)},
        "roofline": roofline,
    }
    gpu_res = m.results() if not args.no_cpu_baseline else None
    is_default = (args.workload == "llama2_7b" and do_bwd and args.schedule == "linear_down"
                  and not args.dora)
    if is_default and not args.no_other_workloads:
        del m
        torch.cuda.empty_cache()
        others = [other_workload("llama2_7b", True, 10, 3, host=host)]
        if not args.no_cpu_baseline:
            pass   # host is still needed below
        for name in ("llama2_13b_skew", "llama3_8b_clusters"):
            others.append(other_workload(name, False, 10, 3))
        out["config"]["other_workloads"] = others
    if not args.no_cpu_baseline:
        n_cpu = min(args.cpu_tokens, cfg.T)
        out["cpu_baseline"], last = cpu_baseline(cfg, host, n_cpu)
        if n_cpu == cfg.T and cfg.M == 1 and not args.dora:
            out["config"]["parity_max_rel_err_vs_oracle"] = parity_errors(gpu_res, last)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
