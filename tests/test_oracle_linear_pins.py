"""Pins of the oracle's plain LoRA linear (the form MixLoRA puts on the attention projections,
Section 3.2 / Eq. 1) against things other than itself: the merged-weight identity, the B = 0
special case, torch autograd of the merged formulation and central finite differences."""
import numpy as np
import torch

from oracle import mixlora_oracle as orc


def _case(T=37, d_in=24, d_out=40, r=8, seed=3):
    rng = np.random.default_rng(seed)
    return dict(x=rng.standard_normal((T, d_in)), W=rng.standard_normal((d_out, d_in)) * 0.1,
                A=rng.standard_normal((r, d_in)) * 0.3, B=rng.standard_normal((d_out, r)) * 0.3,
                dy=rng.standard_normal((T, d_out)), s=2.0)


def test_merged_weight_identity():
    c = _case()
    y = orc.lora_linear_forward(c["x"], c["W"], c["A"], c["B"], c["s"])
    merged = c["W"] + c["s"] * (c["B"] @ c["A"])
    np.testing.assert_allclose(y, c["x"] @ merged.T, rtol=1e-12, atol=1e-12)


def test_zero_B_is_the_frozen_linear():
    c = _case()
    y = orc.lora_linear_forward(c["x"], c["W"], c["A"], np.zeros_like(c["B"]), c["s"])
    np.testing.assert_array_equal(y, c["x"] @ c["W"].T)
    g = orc.lora_linear_backward(c["x"], c["W"], c["A"], np.zeros_like(c["B"]), c["s"], c["dy"])
    np.testing.assert_array_equal(g["dA"], np.zeros_like(c["A"]))
    np.testing.assert_allclose(g["dx"], c["dy"] @ c["W"], rtol=1e-13)


def test_backward_matches_autograd_of_merged_weights():
    c = _case()
    t = {n: torch.tensor(c[n], dtype=torch.float64, requires_grad=n in ("x", "A", "B"))
         for n in ("x", "W", "A", "B", "dy")}
    y = t["x"] @ (t["W"] + c["s"] * (t["B"] @ t["A"])).T
    (y * t["dy"]).sum().backward()
    g = orc.lora_linear_backward(c["x"], c["W"], c["A"], c["B"], c["s"], c["dy"])
    np.testing.assert_allclose(g["dx"], t["x"].grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["dA"], t["A"].grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["dB"], t["B"].grad.numpy(), rtol=1e-11, atol=1e-12)


def test_backward_matches_finite_differences():
    c = _case(T=9, d_in=7, d_out=11, r=8)
    g = orc.lora_linear_backward(c["x"], c["W"], c["A"], c["B"], c["s"], c["dy"])

    def loss(**kw):
        a = dict(c); a.update(kw)
        return float((orc.lora_linear_forward(a["x"], a["W"], a["A"], a["B"], a["s"]) * c["dy"]).sum())

    h = 1e-6
    rng = np.random.default_rng(0)
    for name, key in (("x", "dx"), ("A", "dA"), ("B", "dB")):
        for _ in range(6):
            i = tuple(rng.integers(0, n) for n in c[name].shape)
            up, dn = c[name].copy(), c[name].copy()
            up[i] += h; dn[i] -= h
            fd = (loss(**{name: up}) - loss(**{name: dn})) / (2 * h)
            assert abs(fd - g[key][i]) <= 1e-6 * max(1.0, abs(fd)), (name, i)


def test_adamw_matches_torch_optimizer():
    """Five steps of the oracle's AdamW against torch.optim.AdamW (an independent implementation)
    with the paper's learning rate and a non-default weight decay."""
    rng = np.random.default_rng(9)
    p0 = rng.standard_normal(257)
    grads = [rng.standard_normal(257) * (0.1 + i) for i in range(5)]
    lr, b1, b2, eps, wd = 2e-4, 0.9, 0.999, 1e-8, 0.05
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t, g in enumerate(grads, start=1):
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = orc.adamw_step(p, g, m, v, t, lr, b1, b2, eps, wd)
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-15)
