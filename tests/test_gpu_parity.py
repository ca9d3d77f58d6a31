"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Small and medium cases span several tiles and ragged tails of every kernel (GEMM tiles of
256/128/64, 512-column element-wise tiles, 8/16-row grouped tiles); full-size cases run in
the launch configuration bench.py times.
"""
import time

import numpy as np
import pytest
import torch

from oracle import mixlora_oracle as orc
from paper_2404_15159_amd import binding as B
from paper_2404_15159_amd import synth
from paper_2404_15159_amd.runner import MixLoraFFN

import parity_utils as pu

pytestmark = pytest.mark.gpu

BASE_BF16 = synth.CONFIGS["llama2_7b"]
BASE_F32 = synth.CONFIGS["tiny_f32"]


def run_case(cfg, host, aux_mode="top1", d_aux=1.0, pretransposed=True, backward=True):
    print(f"\ncase {cfg.name}: T={cfg.T} d={cfg.d} f={cfg.d_ff} N={cfg.N} k={cfg.k} r={cfg.r} "
          f"{cfg.dtype} aux={aux_mode}", flush=True)
    mode = B.AUX_TOP1 if aux_mode == "top1" else B.AUX_TOPK
    m = MixLoraFFN(cfg, host, aux_mode=mode, pretransposed=pretransposed, with_backward=backward)
    m.forward()
    if backward:
        m.backward(d_aux=d_aux)
    res = m.results()
    W = {n: host[n] for n in synth.WEIGHT_NAMES}
    if backward:
        bw = orc.backward(host["x"], W, cfg.k, cfg.lora_scale, host["dy"], d_aux, cfg.aux_coeff,
                          aux_mode)
        fw = bw["forward"]
    else:
        bw = None
        fw = orc.forward(host["x"], W, cfg.k, cfg.lora_scale, cfg.aux_coeff, aux_mode)
    return res, fw, bw, m


def test_tiny_f32_config():
    cfg = BASE_F32
    host = synth.make_inputs(cfg)
    for aux_mode in ("top1", "topk"):
        res, fw, bw, _ = run_case(cfg, host, aux_mode)
        rep = pu.compare_all(res, fw, bw, cfg)
        assert rep["routing_mismatch_tokens"] == 0


SMALL_CASES = [
    # name, base, overrides
    ("bf16_ragged", BASE_BF16, dict(T=300, d=256, d_ff=520, N=8, k=2, r=16)),
    ("bf16_ragged_f32x", BASE_BF16, dict(T=300, d=256, d_ff=544, N=8, k=2, r=16)),
    ("bf16_r8_f32x", BASE_BF16, dict(T=777, d=192, d_ff=1056, N=16, k=2, r=8, alpha=16.0)),
    ("bf16_top3_r24_f32x", BASE_BF16, dict(T=257, d=136, d_ff=288, N=5, k=3, r=24, alpha=48.0)),
    ("bf16_r64_f32x", BASE_BF16, dict(T=130, d=128, d_ff=256, N=4, k=2, r=64, alpha=128.0)),
    ("bf16_multi_tile", BASE_BF16, dict(T=1000, d=512, d_ff=1288, N=16, k=2, r=8, alpha=16.0)),
    ("bf16_top3_r32", BASE_BF16, dict(T=257, d=136, d_ff=264, N=5, k=3, r=32, alpha=64.0)),
    ("bf16_k_eq_N", BASE_BF16, dict(T=130, d=128, d_ff=256, N=4, k=4, r=8, alpha=16.0)),
    ("bf16_top1", BASE_BF16, dict(T=200, d=128, d_ff=384, N=8, k=1, r=16)),
    ("bf16_one_expert", BASE_BF16, dict(T=70, d=64, d_ff=136, N=1, k=1, r=8, alpha=16.0)),
    ("bf16_one_token", BASE_BF16, dict(T=1, d=64, d_ff=128, N=8, k=2, r=16)),
    # the largest expert count and rank-column total the library accepts, and a wide top-k
    ("bf16_64_experts", BASE_BF16, dict(T=640, d=128, d_ff=256, N=64, k=4, r=8, alpha=16.0)),
    ("bf16_top8_of_16", BASE_BF16, dict(T=200, d=128, d_ff=384, N=16, k=8, r=16)),
    ("f32_64_experts", BASE_F32, dict(T=320, d=64, d_ff=136, N=64, k=2, r=8)),
    ("bf16_wide_d", BASE_BF16, dict(T=300, d=1024, d_ff=520, N=8, k=2, r=16)),
    # few tokens: narrow weight-streaming GEMM tiles and the K-split down projection
    ("bf16_decode_64", BASE_BF16, dict(T=64, d=256, d_ff=1024, N=8, k=2, r=16)),
    ("bf16_decode_17", BASE_BF16, dict(T=17, d=512, d_ff=704, N=8, k=2, r=16)),
    ("bf16_decode_100", BASE_BF16, dict(T=100, d=256, d_ff=520, N=4, k=2, r=32, alpha=64.0)),
    ("bf16_decode_128", BASE_BF16, dict(T=128, d=192, d_ff=576, N=8, k=2, r=8, alpha=16.0)),
    # few tokens: the rank-r partial sums ride in the combine's launch while k * r <= 256 ...
    ("bf16_decode_top8_r32", BASE_BF16, dict(T=40, d=256, d_ff=640, N=8, k=8, r=32, alpha=64.0)),
    ("bf16_decode_1_token", BASE_BF16, dict(T=1, d=256, d_ff=520, N=8, k=2, r=16)),
    # ... and have a launch of their own beyond that
    ("bf16_decode_top8_r64", BASE_BF16, dict(T=24, d=256, d_ff=576, N=8, k=8, r=64, alpha=128.0)),
    ("bf16_skew", synth.CONFIGS["llama2_13b_skew"], dict(T=600, d=256, d_ff=768)),
    ("bf16_clusters", synth.CONFIGS["llama3_8b_clusters"], dict(T=1024, d=256, d_ff=512, seq_len=64)),
    # more than 8192 pairs: grouping and Eq. 8-9 run as multi-workgroup passes (ragged last chunk)
    ("bf16_long_batch", BASE_BF16, dict(T=5001, d=64, d_ff=128, N=8, k=2, r=8, alpha=16.0)),
    ("bf16_long_top3", BASE_BF16, dict(T=3100, d=64, d_ff=136, N=5, k=3, r=8, alpha=16.0)),
    ("bf16_long_64_experts", BASE_BF16, dict(T=2500, d=64, d_ff=128, N=64, k=4, r=8, alpha=16.0)),
    ("f32_long_batch", BASE_F32, dict(T=4200, d=32, d_ff=72, N=16, k=2, r=8)),
    ("f32_ragged", BASE_F32, dict(T=333, d=72, d_ff=200, N=6, k=2, r=8)),
    ("f32_top3", BASE_F32, dict(T=129, d=64, d_ff=136, N=8, k=3, r=16, alpha=32.0)),
    # very wide model or hidden dimension (long contractions, many column tiles)
    ("bf16_d_16384", BASE_BF16, dict(T=520, d=16384, d_ff=1032, N=4, k=2, r=64, alpha=128.0)),
    ("bf16_dff_53248", BASE_BF16, dict(T=200, d=264, d_ff=53248, N=8, k=2, r=16)),
    # LoRA scales alpha / r that are not powers of two
    ("bf16_scale_1p5", BASE_BF16, dict(T=300, d=256, d_ff=520, N=8, k=2, r=16, alpha=24.0)),
    ("bf16_scale_0p7", BASE_BF16, dict(T=257, d=136, d_ff=264, N=5, k=3, r=40, alpha=28.0)),
    ("f32_scale_1p3", BASE_F32, dict(T=333, d=72, d_ff=200, N=6, k=2, r=8, alpha=10.4)),
    # edges of the stage that runs on token tiles of one expert pair (top-2, bf16, r <= 16,
    # N <= 16, 128 < T <= 65536, d_ff >= 64): fewest tokens, a single pair group with many tiles,
    # sixteen experts (120 groups, most tiles ragged) with a ragged last column block, the
    # narrowest d_ff, the largest token count and the first one past it (expert-grouped path)
    ("bf16_pg_129_tokens", BASE_BF16, dict(T=129, d=128, d_ff=264, N=8, k=2, r=16)),
    ("bf16_pg_two_experts", BASE_BF16, dict(T=300, d=128, d_ff=328, N=2, k=2, r=16)),
    ("bf16_pg_16_experts_r4", BASE_BF16, dict(T=1500, d=128, d_ff=392, N=16, k=2, r=4, alpha=8.0)),
    ("bf16_pg_dff_64", BASE_BF16, dict(T=200, d=64, d_ff=64, N=4, k=2, r=8, alpha=16.0)),
    ("bf16_pg_65536_tokens", BASE_BF16, dict(T=65536, d=64, d_ff=136, N=8, k=2, r=8, alpha=16.0)),
    ("bf16_pg_65537_tokens", BASE_BF16, dict(T=65537, d=64, d_ff=72, N=8, k=2, r=8, alpha=16.0)),
    # ranks off the multiples of 8 (the rank study of Section 4.3 starts at r = 2), at the 7B
    # model's d : d_ff ratio: the library runs them on zero-padded banks and cuts the gradients back
    ("bf16_r2_7b_ratio", BASE_BF16, dict(T=300, d=256, d_ff=688, N=8, k=2, r=2, alpha=4.0)),
    ("bf16_r4_7b_ratio", BASE_BF16, dict(T=300, d=256, d_ff=688, N=8, k=2, r=4, alpha=8.0)),
    ("bf16_r1_decode", BASE_BF16, dict(T=33, d=128, d_ff=344, N=8, k=2, r=1, alpha=2.0)),
    ("bf16_r12_top3", BASE_BF16, dict(T=257, d=136, d_ff=264, N=5, k=3, r=12, alpha=24.0)),
    ("bf16_r20_long", BASE_BF16, dict(T=4200, d=64, d_ff=136, N=8, k=2, r=20, alpha=40.0)),
    ("f32_r7", BASE_F32, dict(T=129, d=64, d_ff=136, N=8, k=2, r=7, alpha=14.0)),
    # top-1 with nearly balanced first-slot counts: the router is trained by the auxiliary term
    # alone, p * (F_e - <p, F>) with every F_e within a percent of 1/N
    ("f32_top1_balanced_aux", BASE_F32, dict(T=2049, d=128, d_ff=1032, N=3, k=1, r=16, alpha=32.0)),
    ("f32_top1_balanced_aux_topk", BASE_F32, dict(T=2049, d=128, d_ff=264, N=3, k=3, r=8)),
]


@pytest.mark.parametrize("name,base,over", SMALL_CASES, ids=[c[0] for c in SMALL_CASES])
def test_small_cases(name, base, over):
    cfg = synth.scaled(base, name=name, **over)
    host = synth.make_inputs(cfg)
    # livelier LoRA paths than the large-shape recipe so that a wrong rank-r term shows
    for n in ("B_gate", "B_up", "B_down"):
        host[n] = synth.round_to_bf16(host[n] * 4.0) if cfg.dtype == "bf16" else host[n] * 4.0
    res, fw, bw, _ = run_case(cfg, host, "topk" if cfg.k == 3 else "top1", d_aux=1.5)
    pu.compare_all(res, fw, bw, cfg)


def test_million_tokens():
    """A very long batch of narrow rows (two million pairs): row indices times row widths pass
    2^31 elements only in 64-bit arithmetic, the grouping runs as thousands of chunks, and the
    reductions over tokens are long.  Everything against the oracle, element by element."""
    cfg = synth.scaled(BASE_BF16, name="bf16_million", T=1000003, d=64, d_ff=136, N=8, k=2, r=8,
                       alpha=16.0)
    host = synth.make_inputs(cfg)
    res, fw, bw, _ = run_case(cfg, host, d_aux=1.5)
    pu.compare_all(res, fw, bw, cfg)


def test_unused_expert_and_untransposed_weights():
    cfg = synth.scaled(synth.CONFIGS["llama2_13b_skew"], name="bf16_unused", T=260, d=128,
                       d_ff=264, N=8, k=2, r=16)
    host = synth.make_inputs(cfg)
    host["W_router"][5, cfg.d - 1] = -60.0      # x[:, d-1] == 1: expert 5 is never kept
    host["W_router"] = synth.round_to_bf16(host["W_router"])
    res, fw, bw, _ = run_case(cfg, host, pretransposed=False)
    assert fw["counts"][5] == 0 and res["counts"][5] == 0
    pu.compare_all(res, fw, bw, cfg)
    for n in ("dA_gate", "dB_gate", "dA_up", "dB_up", "dA_down", "dB_down"):
        assert (res[n][5] == 0.0).all(), n


@pytest.mark.parametrize("variant", ["default", "long_batch", "shared", "vanilla", "dora"])
def test_deterministic_reruns(variant):
    """No atomics, fixed summation orders: a second run on the same buffers gives the same bits.
    long_batch goes through the multi-workgroup grouping passes."""
    over = dict(T=700, d=256, d_ff=1032, N=8, k=2, r=16)
    if variant == "long_batch":
        over = dict(T=4500, d=64, d_ff=136, N=8, k=2, r=8, alpha=16.0)
    cfg = synth.scaled(BASE_BF16, name="bf16_rerun_" + variant, **over)
    host = synth.make_inputs(cfg)
    kw = {}
    if variant in ("shared", "vanilla"):
        kw["schedule"] = B.SCHEDULE_SHARED if variant == "shared" else B.SCHEDULE_VANILLA
    if variant == "dora":
        kw["magnitudes"] = synth.make_magnitudes(cfg)
    m = MixLoraFFN(cfg, host, **kw)
    m.forward(); m.backward()
    a = m.results()
    m.forward(); m.backward()
    b = m.results()
    for n in a:
        assert np.array_equal(np.asarray(a[n]), np.asarray(b[n])), n


def test_caller_stream_and_forward_only_workspace():
    """Everything is enqueued on the stream the caller passes (here a non-default one, with the
    host not synchronising between the two calls), and a forward-only call needs only the
    forward workspace; results equal those of the default-stream run bit for bit."""
    cfg = synth.scaled(BASE_BF16, name="bf16_stream", T=520, d=256, d_ff=776, N=8, k=2, r=16)
    host = synth.make_inputs(cfg)
    m = MixLoraFFN(cfg, host)
    m.forward(); m.backward()
    a = m.results()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for t in (m.y, m.dx, m.topk_w, *m.g.values()):
        t.zero_()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        m.forward(stream=side)
        m.backward(stream=side)
    side.synchronize()
    b = m.results()
    for n in a:
        assert np.array_equal(np.asarray(a[n]), np.asarray(b[n])), n
    f = MixLoraFFN(cfg, host, with_backward=False)
    assert f.ws_bytes < m.ws_bytes
    f.forward()
    c = f.results()
    for n in c:
        assert np.array_equal(np.asarray(a[n]), np.asarray(c[n])), n


@pytest.mark.parametrize("variant", ["default", "long_batch", "shared", "vanilla", "dora"])
def test_graph_capture_and_replay(variant):
    """The call sequences allocate nothing and never synchronise, so forward + backward can be
    captured into a HIP graph.  Every replay (with eager work and synchronisations between the
    replays) must reproduce the eager result bit for bit; the same holds for the paper's two
    schedules, the weight-decomposed variant and the multi-workgroup grouping of long batches."""
    over = dict(T=384, d=256, d_ff=648, N=8, k=2, r=16)
    if variant == "long_batch":
        over = dict(T=4500, d=64, d_ff=136, N=8, k=2, r=8, alpha=16.0)
    cfg = synth.scaled(BASE_BF16, name="bf16_graph_" + variant, **over)
    host = synth.make_inputs(cfg)
    kw = {}
    if variant in ("shared", "vanilla"):
        kw["schedule"] = B.SCHEDULE_SHARED if variant == "shared" else B.SCHEDULE_VANILLA
    if variant == "dora":
        kw["magnitudes"] = synth.make_magnitudes(cfg)
    m = MixLoraFFN(cfg, host, **kw)
    m.forward(); m.backward()          # eager: also sets the kernels' one-time attributes
    ref = m.results()
    outputs = [m.y, m.dx, m.topk_w, *m.g.values()]
    if variant == "dora":
        outputs += list(m.gm.values())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        m.forward(stream=side)
        m.backward(stream=side)
        graph.capture_end()
    torch.cuda.synchronize()
    x0 = m.t["x"].clone()
    for rep in range(3):
        for t in outputs:
            t.zero_()
        # eager work of the program's own between the replays: another input through the same
        # workspace, then the original input restored
        m.t["x"].copy_(torch.roll(x0, 1, dims=0))
        m.forward()
        torch.cuda.synchronize()
        m.t["x"].copy_(x0)
        graph.replay()
        got = m.results()
        for n in ref:
            assert np.array_equal(np.asarray(ref[n]), np.asarray(got[n])), (rep, n)


def test_mfma_probe_is_plausible():
    sink = torch.empty(1 << 20, dtype=torch.float32, device="cuda:0")
    one = B.mixlora_mfma_probe(sink, sink.numel() * 4, 1, 4000)
    two = B.mixlora_mfma_probe(sink, sink.numel() * 4, 2, 4000)
    print(f"register-only bf16 MFMA: {one:.0f} TFLOP/s at 1 wave/SIMD, {two:.0f} at 2", flush=True)
    assert 300.0 < one < 2600.0 and 300.0 < two < 2600.0     # below the 2.5 PFLOP/s published peak
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_mfma_probe(sink, 1024, 2, 100)
    assert ei.value.code == -5


@pytest.mark.parametrize("mode", ["top1", "topk"])
def test_aux_loss_entry(mode):
    T, N, k = 5000, 16, 2
    rng = np.random.default_rng(7)
    z = rng.normal(size=(T, N)) * 1.3
    p = np.exp(z - z.max(axis=1, keepdims=True))
    p = (p / p.sum(axis=1, keepdims=True)).astype(np.float32)
    idx = np.argsort(-p, axis=1, kind="stable")[:, :k].astype(np.int32)
    dev = torch.device("cuda:0")
    tp, ti = torch.from_numpy(p).to(dev), torch.from_numpy(idx).to(dev)
    loss = torch.empty(1, device=dev)
    F = torch.empty(N, device=dev)
    P = torch.empty(N, device=dev)
    dp = torch.empty((T, N), device=dev)
    B.mixlora_aux_loss(tp, ti, T, N, k, 0.01, B.AUX_TOP1 if mode == "top1" else B.AUX_TOPK,
                       loss, F, P, dp)
    torch.cuda.synchronize()
    rl, rF, rP = orc.aux_loss(p, idx, N, 0.01, mode)
    rdp = orc.aux_loss_dprobs(p, idx, N, 0.01, mode)
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl)
    assert np.array_equal(F.cpu().numpy(), rF.astype(np.float32))   # counts / T: exact in fp32
    np.testing.assert_allclose(P.cpu().numpy(), rP, rtol=1e-5)
    np.testing.assert_allclose(dp.cpu().numpy(), rdp, rtol=1e-5)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_transpose_entry(dtype):
    rows, cols = 130, 257
    a = synth.round_to_bf16(np.random.default_rng(3).normal(size=(rows, cols)).astype(np.float32))
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    src = torch.from_numpy(a).to("cuda:0").to(td)
    dst = torch.empty((cols, rows), dtype=td, device="cuda:0")
    B.mixlora_transpose(src, dst, rows, cols, B.BF16 if dtype == "bf16" else B.F32)
    torch.cuda.synchronize()
    assert np.array_equal(dst.float().cpu().numpy(), a.T)


# ---- full-size workloads, in the launch configuration the bench times -----------------------
def test_llama2_7b_full_forward_backward():
    """Whole LLaMA-2-7B-shaped workload against the full oracle (every token, every gradient)."""
    cfg = synth.CONFIGS["llama2_7b"]
    t0 = time.time()
    host = synth.make_inputs(cfg)
    print(f"inputs {time.time() - t0:.1f}s", flush=True)
    t0 = time.time()
    res, fw, bw, _ = run_case(cfg, host)
    print(f"gpu + oracle {time.time() - t0:.1f}s", flush=True)
    pu.compare_all(res, fw, bw, cfg)


def full_size_case(cfg):
    """A full-size workload against the full oracle: every token's y and dx, every gradient
    with all grouped rows live, the auxiliary loss and its gradient (d_aux = 1)."""
    t0 = time.time()
    host = synth.make_inputs(cfg)
    print(f"inputs {time.time() - t0:.1f}s", flush=True)
    t0 = time.time()
    res, fw, bw, _ = run_case(cfg, host)
    print(f"gpu + oracle {time.time() - t0:.1f}s", flush=True)
    pu.compare_all(res, fw, bw, cfg)
    share = res["counts"] / res["counts"].sum()
    print("expert load share:", np.round(share, 3), flush=True)
    return res


@pytest.mark.timeout(1500)
def test_llama2_13b_skew_full_forward_backward():
    """LLaMA-2-13B shape, expert 0's logit raised by 1.5 (about 30 % of the pairs on one expert):
    the grouped stages and the gradient sums under load imbalance, whole batch."""
    res = full_size_case(synth.CONFIGS["llama2_13b_skew"])
    share0 = res["counts"][0] / res["counts"].sum()
    assert share0 > 0.22      # the skewed expert carries well above the uniform 12.5 %


@pytest.mark.timeout(1500)
def test_llama3_8b_clusters_full_forward_backward():
    """LLaMA-3-8B shape, 16 experts of rank 8, 16384 tokens in four clusters: more than 8192
    pairs (multi-workgroup grouping), N = 16 auxiliary gradient, whole batch."""
    full_size_case(synth.CONFIGS["llama3_8b_clusters"])
