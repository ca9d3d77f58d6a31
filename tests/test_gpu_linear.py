"""GPU parity of the plain LoRA linear (attention-projection form, Eq. 1) against the oracle."""
import numpy as np
import pytest

from oracle import mixlora_oracle as orc
from paper_2404_15159_amd import synth
from paper_2404_15159_amd.runner import LoraLinear

import parity_utils as pu

pytestmark = pytest.mark.gpu

CASES = [
    # name, T, d_in, d_out, r, dtype, pretransposed
    ("f32_small", 130, 72, 200, 8, "f32", True),
    ("f32_r16_untransposed", 97, 64, 136, 16, "f32", False),
    ("bf16_ragged", 300, 256, 520, 16, "bf16", True),
    ("bf16_r64", 257, 136, 264, 64, "bf16", True),
    ("bf16_r24_untransposed", 513, 192, 320, 24, "bf16", False),
    ("bf16_multi_tile", 1000, 512, 1288, 8, "bf16", True),
    ("bf16_few_rows", 17, 512, 704, 16, "bf16", True),
    ("bf16_one_row", 1, 64, 128, 8, "bf16", True),
]


@pytest.mark.parametrize("name,T,d_in,d_out,r,dtype,pre", CASES, ids=[c[0] for c in CASES])
def test_lora_linear_small(name, T, d_in, d_out, r, dtype, pre):
    s = 2.0
    host = synth.make_linear_inputs(T, d_in, d_out, r, dtype, seed=synth.SEED_BASE + 100 + len(name),
                                    b_std=0.08)
    print(f"\nlinear case {name}: T={T} d_in={d_in} d_out={d_out} r={r} {dtype}", flush=True)
    m = LoraLinear(T, d_in, d_out, r, s, dtype, host, pretransposed=pre)
    m.forward(); m.backward()
    res = m.results()
    y = orc.lora_linear_forward(host["x"], host["W"], host["A"], host["B"], s)
    g = orc.lora_linear_backward(host["x"], host["W"], host["A"], host["B"], s, host["dy"])
    tol = pu.TOL[dtype]
    rep = {"y": pu.assert_close("y", res["y"], y, tol)}
    for n in ("dx", "dA", "dB"):
        rep[n] = pu.assert_close(n, res[n], g[n], tol)
    print({k: tuple(f"{v:.2e}" for v in e) for k, e in rep.items()}, flush=True)
    # the LoRA path is really there: the frozen product alone is off by more than the tolerance
    base = host["x"].astype(np.float64) @ host["W"].astype(np.float64).T
    assert pu.rel_errors(base, y)[0] > 5 * tol


def test_lora_linear_full_size_attention_projection():
    """A q/k/v/o-sized projection of the LLaMA-2-7B shape (4096 -> 4096, rank 16, 4096 tokens),
    as bench.py --workload llama2_7b_attn_proj times it: sampled outputs and the full A/B
    gradients against the oracle."""
    T, d, r, s = 4096, 4096, 16, 2.0
    host = synth.make_linear_inputs(T, d, d, r, "bf16", seed=synth.SEED_BASE + 8)
    m = LoraLinear(T, d, d, r, s, "bf16", host)
    m.forward(); m.backward()
    res = m.results()
    rng = np.random.default_rng(4)
    rows = rng.choice(T, size=64, replace=False)
    y = orc.lora_linear_forward(host["x"][rows], host["W"], host["A"], host["B"], s)
    pu.assert_close("y", res["y"][rows], y, pu.TOL["bf16"])
    g = orc.lora_linear_backward(host["x"], host["W"], host["A"], host["B"], s, host["dy"])
    for n in ("dx", "dA", "dB"):
        pu.assert_close(n, res[n], g[n], pu.TOL["bf16"])


def test_adamw_step_matches_oracle():
    """Three AdamW steps on 100003 parameters: float32 master values and moments against the
    float64 oracle, and the bf16 copy equal to the rounded master values."""
    import torch
    from paper_2404_15159_amd import binding as B
    n = 100003
    rng = np.random.default_rng(21)
    p0 = rng.standard_normal(n).astype(np.float32)
    p = torch.from_numpy(p0.copy()).cuda()
    m = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    v = torch.zeros_like(m)
    low = torch.empty(n, dtype=torch.bfloat16, device="cuda:0")
    rp, rm, rv = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    # the C struct carries the hyper-parameters as float32: the oracle gets the same values
    lr, b1, b2, eps, wd = (float(np.float32(h)) for h in (2e-4, 0.9, 0.999, 1e-8, 0.01))
    for t in range(1, 4):
        g = (rng.standard_normal(n) * 0.3).astype(np.float32)
        gd = torch.from_numpy(g).cuda()
        B.mixlora_adamw_step(B.AdamW(lr, b1, b2, eps, wd, t), n, p, gd, m, v, low, B.BF16)
        rp, rm, rv = orc.adamw_step(rp, g, rm, rv, t, lr, b1, b2, eps, wd)
    torch.cuda.synchronize()
    pu.assert_close("param", p.cpu().numpy(), rp, 1e-6)
    pu.assert_close("m", m.cpu().numpy(), rm, 1e-6)
    pu.assert_close("v", v.cpu().numpy(), rv, 1e-6)
    assert torch.equal(low, p.to(torch.bfloat16))
    # the update really moved the parameters by about lr per step
    assert 1e-4 < np.abs(p.cpu().numpy() - p0).mean() < 1e-3
