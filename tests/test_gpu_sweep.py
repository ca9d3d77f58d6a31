"""Seeded random-shape sweep of every entry-point family against the oracle (small shapes: odd
token counts around the tile sizes, d and d_ff at every multiple-of-8 remainder class, ranks
8..64, 1..32 experts).

One tensor needs a scale of its own in bf16 when there are only a few tokens.  The router
gradient of a token is  dz_e = p_e (dp_e - <p, dp>)  with  dp_j = (dw_j - sum_i w_i dw_i) / sum_kept p
on the kept experts, where  dw_j = <dy_t, E_j(x_t)> = sum_c dy_tc o_jc  is the gradient of routing
weight j: dz is driven by DIFFERENCES of the dw_j, which for experts that share the frozen FFN
are nearly equal numbers.  bf16 storage of the shared projections and of the rank-r deltas
perturbs every dw_j by a few 1e-3 of the size of its terms (far inside the 2e-2 bar), but that
is 3 to 10 % of dw_0 - dw_1, and with fewer than 16 tokens nothing averages it out in
dW_router = sum_t dz_t x_t^T  (re-evaluating the definition on the CPU with only those roundings
applied gives the same 2.5e-2 and 1.0e-1 that the kernels show on the two single-token cases
of this sweep).  There the tensor is therefore held to the error that a tol-accurate dw
implies through the exact map dw -> dW_router:  with  |delta dw_tj| <= tol * rss_tj,
rss_tj = sqrt(sum_c (dy_tc o_jc)^2)  the root-sum-square of the terms of dw_tj, one has
|delta dz_te| <= 2 w_e max_j |delta dw_tj|, hence
|delta dW_router[e, c]| <= 2 tol sum_t max_j rss_tj |x_tc|   (plus tol * max |ref|).
fp32 storage keeps the flat 1e-5 bar at every token count."""
import numpy as np
import pytest

from oracle import mixlora_oracle as orc
from paper_2404_15159_amd import binding as B
from paper_2404_15159_amd import synth
from paper_2404_15159_amd.runner import MixLoraFFN

import parity_utils as pu

pytestmark = pytest.mark.gpu

KINDS = ("default", "shared", "vanilla", "dora", "multi", "f32")
MAG = ("m_gate", "m_up", "m_down")


def _draw(rng, ci):
    kind = KINDS[ci % len(KINDS)]
    N = int(rng.choice([1, 2, 3, 4, 5, 6, 8, 12, 16, 24, 32]))
    k = int(rng.integers(1, min(N, 4) + 1))
    r = int(rng.choice([1, 2, 4, 8, 12, 16, 24, 32, 40, 64]))
    rp = (r + 7) // 8 * 8   # the library's limit counts rank entries after padding to 8
    if N * rp > 512:
        r = 8
    T = int(rng.choice([1, 2, 7, 33, 64, 65, 127, 128, 129, 200, 255, 256, 257, 511, 700, 1025, 2049]))
    d = int(rng.choice([8, 16, 24, 64, 72, 128, 136, 192, 256, 264, 320, 512]))
    f = int(rng.choice([8, 16, 40, 64, 120, 128, 136, 256, 264, 504, 512, 520, 1032]))
    M = 1
    if kind == "multi":
        M = int(rng.choice([2, 3]))
        if M * N > 64 or M * N * ((r + 7) // 8 * 8) > 512:
            N, r, k = 4, 8, min(k, 4)
    return kind, dict(T=T, d=d, d_ff=f, N=N, k=k, r=r, alpha=2.0 * r, M=M, seq_len=max(1, T // 7))


def _dw_term_rss(fw, dy, T, k):
    """rss[t, j] = sqrt(sum_c (dy[t, c] * o[t, j, c])^2) from the oracle's kept expert outputs."""
    rss = np.zeros((T, k))
    dy = np.asarray(dy, dtype=np.float64)
    for sv in fw["saved"].values():
        tok, slot = sv["tok"], sv["slot"]
        rss[tok, slot] = np.sqrt(((dy[tok] * sv["o"]) ** 2).sum(axis=1))
    return rss


def _router_grad_bound(rss, x, tol):
    """[d] bound on |delta dW_router[e, :]| implied by a tol-accurate dw (module docstring)."""
    m = np.asarray(rss, dtype=np.float64).max(axis=1)            # [T]
    return 2.0 * tol * (m[:, None] * np.abs(np.asarray(x, dtype=np.float64))).sum(axis=0)


def _check_grads(res, ref, cfg, all_same, F=None, x_max=1.0, rss=None, x=None):
    tol = pu.TOL[cfg.dtype]
    for n in pu.GRAD_NAMES:
        if not (all_same or cfg.dtype == "bf16"):
            continue
        if n == "dW_router" and cfg.k == 1 and F is not None and np.ptp(F) == 0.0:
            # top-1 keeps weight 1, so only the auxiliary term reaches the router, and with
            # exactly equal F_e it is p * (F_e - <p, F>) = 0: the oracle's value is its own
            # float64 rounding noise, so the HIP result is held to an absolute bound instead
            assert np.abs(ref[n]).max() <= 1e-12 * x_max
            assert np.abs(res[n]).max() <= 1e-7 * cfg.aux_coeff * x_max, n
            continue
        if n == "dW_router" and cfg.T < 16 and cfg.dtype == "bf16":
            bound = _router_grad_bound(rss, x, tol)[None, :] + tol * np.abs(ref[n]).max()
            excess = np.abs(np.asarray(res[n], dtype=np.float64) - ref[n]) - bound
            assert (excess <= 0.0).all(), f"dW_router beyond the dw-implied bound by {excess.max():.3e}"
            continue
        pu.assert_close(n, res[n], ref[n], tol)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_shapes(seed):
    rng = np.random.default_rng(seed)
    for ci in range(36):
        kind, over = _draw(rng, ci)
        base = synth.CONFIGS["tiny_f32"] if kind == "f32" else synth.CONFIGS["llama2_7b"]
        cfg = synth.scaled(base, name=f"sweep{seed}_{ci}_{kind}", **over)
        print(f"case {ci} {kind}: {over}", flush=True)
        host = synth.make_inputs(cfg)
        for n in ("B_gate", "B_up", "B_down"):
            host[n] = synth.round_to_bf16(host[n] * 4.0) if cfg.dtype == "bf16" else host[n] * 4.0
        W = {n: host[n] for n in synth.WEIGHT_NAMES}
        tol = pu.TOL[cfg.dtype]
        if kind == "multi":
            tm = synth.token_model(cfg, "uneven")
            m = MixLoraFFN(cfg, host, token_model=tm)
            m.forward()
            m.backward()
            res = m.results()
            Ws = synth.split_adapters(cfg, host)
            fw = orc.multi_forward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, cfg.aux_coeff)
            bw = orc.multi_backward(host["x"], tm, Ws, cfg.k, cfg.lora_scale, host["dy"], None,
                                    cfg.aux_coeff)
            same = pu.check_routing(res, fw, cfg, 2e-5, token_model=tm)
            pu.assert_close("y", res["y"][same], fw["y"][same], tol)
            pu.assert_close("dx", res["dx"][same], bw["dx"][same], tol)
            ref = {n: np.concatenate([g[n] for g in bw["grads"]], axis=0) for n in pu.GRAD_NAMES}
            rss = np.zeros((cfg.T, cfg.k))
            if cfg.T < 16:   # terms of the routing-weight gradients, adapter by adapter
                for mi in range(cfg.M):
                    tok = np.nonzero(tm == mi)[0]
                    if tok.size:
                        fm = orc.forward(host["x"][tok], Ws[mi], cfg.k, cfg.lora_scale,
                                         cfg.aux_coeff, keep=True)
                        rss[tok] = _dw_term_rss(fm, host["dy"][tok], tok.size, cfg.k)
            _check_grads(res, ref, cfg, bool(same.all()), rss=rss, x=host["x"])
            continue
        if kind == "dora":
            mag = {n: [] for n in MAG}
            for e in range(cfg.N):
                nrm = orc.dora_row_norms(W, e, cfg.lora_scale)
                for nm in ("gate", "up", "down"):
                    mag["m_" + nm].append(nrm[nm] * rng.uniform(0.6, 1.4, nrm[nm].shape))
            mag = {n: np.stack(v).astype(np.float32) for n, v in mag.items()}
            m = MixLoraFFN(cfg, host, magnitudes=mag)
            bw = orc.dora_backward(host["x"], W, mag, cfg.k, cfg.lora_scale, host["dy"], 1.5,
                                   cfg.aux_coeff)
        else:
            sched = {"shared": B.SCHEDULE_SHARED, "vanilla": B.SCHEDULE_VANILLA}.get(
                kind, B.SCHEDULE_LINEAR_DOWN)
            m = MixLoraFFN(cfg, host, schedule=sched)
            bw = orc.backward(host["x"], W, cfg.k, cfg.lora_scale, host["dy"], 1.5, cfg.aux_coeff)
        m.forward()
        m.backward(d_aux=1.5)
        res = m.results()
        rep = pu.compare_all(res, bw["forward"], bw, cfg, check_grads=False, verbose=False)
        same = (res["topk_idx"] == bw["forward"]["topk_idx"]).all(axis=1)
        pu.assert_close("dx", res["dx"][same], bw["dx"][same], tol)
        _check_grads(res, bw, cfg, rep["routing_mismatch_tokens"] == 0, F=bw["forward"]["F"],
                     x_max=float(np.abs(host["x"]).max()),
                     rss=_dw_term_rss(bw["forward"], host["dy"], cfg.T, cfg.k), x=host["x"])
        if kind == "dora":
            for n in MAG:
                pu.assert_close("d" + n, res["d" + n], bw["d" + n], tol)
