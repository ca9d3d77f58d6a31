"""Pins of the multi-adapter oracle functions (CPU only).

The multi-adapter block (Section 3.3, optimisation II; outer loop of Algorithm 1) is checked
against things other than itself:
  * one adapter reduces to the single-adapter block;
  * M adapters equal ONE large block with M*N experts whose router is blocked by indicator
    channels appended to x (a token's logits for foreign experts are lowered by 1e4, so their
    probability is exactly 0 in float64) - computed with the single-adapter oracle;
  * adapters are independent (changing one adapter leaves the other's tokens bit-identical);
  * permuting the tokens permutes the per-token results and keeps the summed gradients;
  * an adapter without tokens gets zero gradients and zero loss.
"""
import numpy as np
import pytest

from oracle import mixlora_oracle as orc
from paper_2404_15159_amd import synth

NAMES = ("A_gate", "B_gate", "A_up", "B_up", "A_down", "B_down", "W_router")


def _case(M=3, pattern="round_robin", T=96, seq_len=8, **kw):
    base = synth.CONFIGS["tiny_f32"]
    cfg = synth.scaled(base, T=T, d=32, d_ff=56, N=4, k=2, r=8, M=M, seq_len=seq_len, b_std=0.3, **kw)
    host = synth.make_inputs(cfg)
    host = {n: v.astype(np.float64) for n, v in host.items()}
    host["W_router"] = host["W_router"] * 20.0      # spread the logits: no near-ties
    tm = synth.token_model(cfg, pattern)
    return cfg, host, tm


def test_single_adapter_reduces_to_block():
    cfg, host, tm = _case(M=1)
    Ws = synth.split_adapters(cfg, host)
    fw1 = orc.forward(host["x"], Ws[0], cfg.k, cfg.lora_scale, cfg.aux_coeff)
    fwm = orc.multi_forward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, cfg.aux_coeff)
    assert np.array_equal(fw1["y"], fwm["y"])
    assert np.array_equal(fw1["topk_idx"], fwm["topk_idx"])
    assert fwm["aux_loss"][0] == fw1["aux_loss"]
    bw1 = orc.backward(host["x"], Ws[0], cfg.k, cfg.lora_scale, host["dy"], 1.0, cfg.aux_coeff)
    bwm = orc.multi_backward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, host["dy"], None, cfg.aux_coeff)
    assert np.array_equal(bw1["dx"], bwm["dx"])
    for n in NAMES:
        assert np.array_equal(bw1["d" + n], bwm["grads"][0]["d" + n])


@pytest.mark.parametrize("pattern", ["round_robin", "uneven"])
def test_equals_one_large_block_with_blocked_router(pattern):
    """Append M indicator channels to x; expert (m, e) of the large block has router row
    [W_r^m[e], -c * (1 - onehot(m))], so a token of adapter m sees logit z for its own experts
    and z - c for all others.  Everything but the auxiliary loss (a per-adapter statistic)
    must then agree with the single-adapter oracle run on the large block."""
    cfg, host, tm = _case(M=3, pattern=pattern)
    M, N, d = cfg.M, cfg.N, cfg.d
    Ws = synth.split_adapters(cfg, host)
    T = cfg.T
    c = 1.0e4
    xa = np.concatenate([host["x"], np.eye(M)[tm]], axis=1)                 # [T, d+M]
    big = {}
    for n in ("W_gate", "W_up"):
        big[n] = np.concatenate([host[n], np.zeros((cfg.d_ff, M))], axis=1)
    big["W_down"] = np.concatenate([host["W_down"], np.zeros((M, cfg.d_ff))], axis=0)
    for n in ("A_gate", "A_up"):
        big[n] = np.concatenate([host[n], np.zeros((M * N, cfg.r, M))], axis=2)
    for n in ("B_gate", "B_up", "A_down"):
        big[n] = host[n]
    big["B_down"] = np.concatenate([host["B_down"], np.zeros((M * N, M, cfg.r))], axis=1)
    block = -c * (1.0 - np.repeat(np.eye(M), N, axis=0))                    # [M*N, M]
    big["W_router"] = np.concatenate([host["W_router"], block], axis=1)
    dya = np.concatenate([host["dy"], np.zeros((T, M))], axis=1)

    fwb = orc.forward(xa, big, cfg.k, cfg.lora_scale, 0.0)
    fwm = orc.multi_forward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, 0.0)
    np.testing.assert_allclose(fwm["y"], fwb["y"][:, :d], rtol=1e-12, atol=1e-13)
    assert np.array_equal(fwm["topk_idx"] + (tm * N)[:, None], fwb["topk_idx"])
    np.testing.assert_allclose(fwm["topk_w"], fwb["topk_w"], rtol=1e-12)
    assert np.array_equal(fwm["counts"].reshape(-1), fwb["counts"])

    bwb = orc.backward(xa, big, cfg.k, cfg.lora_scale, dya, 0.0, 0.0)
    bwm = orc.multi_backward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, host["dy"], None, 0.0)
    np.testing.assert_allclose(bwm["dx"], bwb["dx"][:, :d], rtol=1e-10, atol=1e-12)
    for n in NAMES:
        got = np.concatenate([g["d" + n] for g in bwm["grads"]], axis=0)
        ref = bwb["d" + n]
        if n in ("A_gate", "A_up", "W_router"):
            ref = ref[..., :d]
        if n == "B_down":
            ref = ref[:, :d, :]
        np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-12, err_msg=n)


def test_adapters_are_independent():
    cfg, host, tm = _case(M=2)
    Ws = synth.split_adapters(cfg, host)
    fw_a = orc.multi_forward(host["x"], tm, Ws, cfg.k, cfg.lora_scale)
    other = dict(Ws[1])
    other["B_gate"] = Ws[1]["B_gate"] * 3.0
    other["W_router"] = Ws[1]["W_router"][::-1].copy()
    fw_b = orc.multi_forward(host["x"], tm, [Ws[0], other], cfg.k, cfg.lora_scale)
    own = tm == 0
    assert np.array_equal(fw_a["y"][own], fw_b["y"][own])
    assert not np.allclose(fw_a["y"][~own], fw_b["y"][~own])
    assert fw_a["aux_loss"][0] == fw_b["aux_loss"][0]


def test_token_permutation_equivariance():
    cfg, host, tm = _case(M=3, pattern="uneven")
    Ws = synth.split_adapters(cfg, host)
    rng = np.random.default_rng(5)
    perm = rng.permutation(cfg.T)
    a = orc.multi_backward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, host["dy"])
    b = orc.multi_backward(host["x"][perm], tm[perm], Ws, cfg.k, cfg.lora_scale, host["dy"][perm])
    np.testing.assert_allclose(a["dx"][perm], b["dx"], rtol=1e-12, atol=1e-14)
    for m in range(cfg.M):
        for n in NAMES:
            np.testing.assert_allclose(a["grads"][m]["d" + n], b["grads"][m]["d" + n],
                                       rtol=1e-9, atol=1e-12)


def test_adapter_without_tokens():
    cfg, host, tm = _case(M=3, pattern="skip_last")
    assert not np.any(tm == 2)
    Ws = synth.split_adapters(cfg, host)
    fw = orc.multi_forward(host["x"], tm, Ws, cfg.k, cfg.lora_scale)
    assert fw["aux_loss"][2] == 0.0 and not fw["counts"][2].any()
    bw = orc.multi_backward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, host["dy"])
    for n in NAMES:
        assert not bw["grads"][2]["d" + n].any()
    # the two adapters that do have tokens see exactly the two-adapter problem
    fw2 = orc.multi_forward(host["x"], tm, Ws[:2], cfg.k, cfg.lora_scale)
    assert np.array_equal(fw["y"], fw2["y"])


def test_aux_loss_is_per_adapter_statistic():
    """Eq. 8-9 over the adapter's own tokens: with a router that sends every token of adapter m
    to expert 0 with probability ~1, F = P = e_0 and the loss is a * N."""
    cfg, host, tm = _case(M=2)
    Ws = synth.split_adapters(cfg, host)
    x = np.abs(host["x"]) + 0.1
    for Wm in Ws:
        wr = np.zeros_like(Wm["W_router"])
        wr[0] = 50.0
        Wm["W_router"] = wr
    fw = orc.multi_forward(x, tm, Ws, cfg.k, cfg.lora_scale, aux_coeff=0.01)
    np.testing.assert_allclose(fw["aux_loss"], 0.01 * cfg.N, rtol=1e-9)


def test_per_adapter_aux_upstream_gradient():
    """With dy = 0 and d_aux = the m-th unit vector the backward must return the gradient of
    adapter m's auxiliary loss alone: zero for the other adapters, and for adapter m the central
    finite difference of multi_forward's aux_loss[m] with respect to its router weights."""
    cfg, host, tm = _case(M=2, T=48, seq_len=4)
    Ws = synth.split_adapters(cfg, host)
    Ws = [dict(W) for W in Ws]
    for W in Ws:
        W["W_router"] = W["W_router"] * 0.2      # soft routing: the loss varies smoothly
    dy0 = np.zeros_like(host["dy"])
    coeff = 0.7
    for m in range(cfg.M):
        d_aux = np.zeros(cfg.M); d_aux[m] = 1.0
        bw = orc.multi_backward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, dy0, d_aux, coeff)
        other = 1 - m
        for n in NAMES:
            assert not bw["grads"][other]["d" + n].any(), n
        g = bw["grads"][m]["dW_router"]
        assert np.abs(g).max() > 0
        rng = np.random.default_rng(m)
        h = 1e-6
        for _ in range(6):
            i = (int(rng.integers(0, cfg.N)), int(rng.integers(0, cfg.d)))
            vals = []
            for sgn in (+1, -1):
                Wp = [dict(W) for W in Ws]
                wr = Wp[m]["W_router"].copy(); wr[i] += sgn * h
                Wp[m]["W_router"] = wr
                vals.append(orc.multi_forward(host["x"], tm, Wp, cfg.k, cfg.lora_scale, coeff)["aux_loss"][m])
            fd = (vals[0] - vals[1]) / (2 * h)
            assert abs(fd - g[i]) <= 1e-6 * max(1.0, abs(fd)) + 1e-9, (m, i, fd, g[i])
