"""Comparison rules shared by the GPU parity tests (HIP path vs CPU oracle).

Tolerances (stated by the task's acceptance bar): outputs and gradients within a maximum
relative error of 2e-2 for bf16 storage and 1e-5 for fp32 storage, measured per tensor both as
max|delta| / max|ref| and as the Frobenius ratio; routing indices and per-expert counts
bit-exact on tokens whose logit margins exceed 1e-3.
"""
from __future__ import annotations

import numpy as np

TOL = {"bf16": 2e-2, "f32": 1e-5}
MARGIN = 1e-3
GRAD_NAMES = ("dA_gate", "dB_gate", "dA_up", "dB_up", "dA_down", "dB_down", "dW_router")


def rel_errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values from the HIP path"
    den_inf = np.abs(ref).max()
    den_f = np.sqrt((ref * ref).sum())
    if den_inf == 0.0:
        return float(np.abs(got).max()), float(np.sqrt((got * got).sum()))
    d = got - ref
    return float(np.abs(d).max() / den_inf), float(np.sqrt((d * d).sum()) / den_f)


def assert_close(name, got, ref, tol):
    e_inf, e_f = rel_errors(got, ref)
    assert e_inf <= tol and e_f <= tol, f"{name}: max-rel {e_inf:.3e}, fro-rel {e_f:.3e} > {tol}"
    return e_inf, e_f


def routing_masks(logits, k):
    """From the oracle's float64 logits: tokens whose kept set is safe (gap between the k-th
    and (k+1)-th logit above the margin) and tokens whose slot order is safe too."""
    z = np.sort(logits, axis=1)[:, ::-1]
    N = z.shape[1]
    set_safe = np.ones(z.shape[0], bool) if k == N else (z[:, k - 1] - z[:, k]) > MARGIN
    gaps = z[:, :k - 1] - z[:, 1:k] if k > 1 else np.full((z.shape[0], 1), np.inf)
    order_safe = set_safe & (gaps.min(axis=1) > MARGIN)
    return set_safe, order_safe


def check_routing(res, ref, cfg, tol_w, token_model=None):
    """Returns the mask of tokens whose routing agrees completely with the oracle.  With several
    adapters (token_model given) the indices are those inside the token's adapter and the counts
    cover the M*N experts of all adapters."""
    k, N, T = cfg.k, cfg.N, cfg.T
    set_safe, order_safe = routing_masks(ref["logits"], k)
    gi, ri = res["topk_idx"].astype(np.int64), ref["topk_idx"]
    assert gi.shape == (T, k) and gi.min() >= 0 and gi.max() < N
    if token_model is not None:   # index among all experts from here on
        off = (np.asarray(token_model, dtype=np.int64) * N)[:, None]
        gi, ri = gi + off, ri + off
        N = N * cfg.M
    # bit-exact on margin-safe tokens: kept sets, and slot order where the order is safe too
    assert (np.sort(gi[set_safe], axis=1) == np.sort(ri[set_safe], axis=1)).all()
    assert (gi[order_safe] == ri[order_safe]).all()
    # no expert twice in a token; counts are exactly the histogram of the returned indices
    assert (np.diff(np.sort(gi, axis=1), axis=1) != 0).all()
    assert (res["counts"] == np.bincount(gi.reshape(-1), minlength=N)).all()
    assert res["counts"].sum() == k * T
    # counts over the safe tokens equal the oracle's over the same tokens
    assert (np.bincount(gi[set_safe].reshape(-1), minlength=N)
            == np.bincount(ri[set_safe].reshape(-1), minlength=N)).all()
    same = (gi == ri).all(axis=1)
    assert np.abs(res["topk_w"].sum(axis=1) - 1.0).max() < 1e-5
    if same.any():
        assert np.abs(res["topk_w"][same] - ref["topk_w"][same]).max() <= tol_w
    return same


def compare_all(res, fw, bw, cfg, check_grads=True, tol=None, verbose=True):
    """res: HIP results dict; fw/bw: oracle forward / backward dicts (bw may be None)."""
    tol = tol or TOL[cfg.dtype]
    report = {}
    same = check_routing(res, fw, cfg, 1e-5 if cfg.dtype == "f32" else 2e-5)
    report["routing_mismatch_tokens"] = int((~same).sum())
    report["y"] = assert_close("y", res["y"][same], fw["y"][same], tol)
    all_same = bool(same.all())
    if all_same:
        a = abs(res["aux_loss"] - fw["aux_loss"]) / abs(fw["aux_loss"])
        assert a <= 1e-5, f"aux_loss rel err {a}"
        report["aux_loss"] = a
    if bw is not None and check_grads:
        report["dx"] = assert_close("dx", res["dx"][same], bw["dx"][same], tol)
        for n in GRAD_NAMES:
            # a token routed differently (possible only inside the margin) perturbs the summed
            # gradients slightly; the tolerance is only meaningful when routing agrees
            if all_same or cfg.dtype == "bf16":
                report[n] = assert_close(n, res[n], bw[n], tol)
    if verbose:
        print({k: (tuple(f"{x:.2e}" for x in v) if isinstance(v, tuple) else v)
               for k, v in report.items()}, flush=True)
    return report
