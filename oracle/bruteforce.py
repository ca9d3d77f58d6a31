"""Scalar-loop evaluation of the MixLoRA block on tiny inputs.  TEST INFRASTRUCTURE ONLY.

Written independently of mixlora_oracle.py (pure Python floats, no NumPy
arithmetic) to pin it: every expert's three matrices are first merged as in
Eq. 1 (W' = W + s B A, formed element by element), then each token is pushed
through its kept experts one scalar at a time (Eq. 6 with the SwiGLU FFN of
Section 3.3), with the router of Eq. 7 and the renormalisation of Algorithm 1.
Cost grows as T*k*d*d_ff Python operations: use only for T, d, d_ff of a few
tens at most.
"""
from __future__ import annotations

import math


def _merged(Wb, A, B, s):
    """Wb [o][i], A [r][i], B [o][r] -> Wb + s * B A as nested lists."""
    o_n, i_n, r_n = len(Wb), len(Wb[0]), len(A)
    out = []
    for o in range(o_n):
        row = []
        for i in range(i_n):
            acc = 0.0
            for q in range(r_n):
                acc += B[o][q] * A[q][i]
            row.append(Wb[o][i] + s * acc)
        out.append(row)
    return out


def _matvec(M, v):
    return [math.fsum(M[o][i] * v[i] for i in range(len(v))) for o in range(len(M))]


def forward(x, W, k, s, aux_coeff=0.01, aux_mode="top1"):
    """x: nested list [T][d]; W: dict of nested lists with the block's layouts.
    Returns dict(y, topk_idx, topk_w, probs, counts, aux_loss)."""
    T = len(x)
    N = len(W["W_router"])
    merged = []
    for e in range(N):
        merged.append((
            _merged(W["W_gate"], W["A_gate"][e], W["B_gate"][e], s),
            _merged(W["W_up"], W["A_up"][e], W["B_up"][e], s),
            _merged(W["W_down"], W["A_down"][e], W["B_down"][e], s),
        ))
    ys, idxs, ws, probs = [], [], [], []
    counts = [0] * N
    first = [0] * N
    for t in range(T):
        z = _matvec(W["W_router"], x[t])
        zmax = max(z)
        ez = [math.exp(v - zmax) for v in z]
        tot = math.fsum(ez)
        p = [v / tot for v in ez]
        # k largest logits, ties to the lowest expert index, descending order
        chosen = sorted(range(N), key=lambda e: (-z[e], e))[:k]
        ksum = math.fsum(p[e] for e in chosen)
        wt = [p[e] / ksum for e in chosen]
        y = [0.0] * len(x[t])
        for e, we in zip(chosen, wt):
            Wg, Wu, Wd = merged[e]
            g = _matvec(Wg, x[t])
            u = _matvec(Wu, x[t])
            a = [gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)]
            o = _matvec(Wd, a)
            for i in range(len(y)):
                y[i] += we * o[i]
            counts[e] += 1
        first[chosen[0]] += 1
        ys.append(y)
        idxs.append(chosen)
        ws.append(wt)
        probs.append(p)
    if aux_mode == "top1":
        F = [c / T for c in first]
    else:
        F = [c / (T * k) for c in counts]
    P = [math.fsum(probs[t][e] for t in range(T)) / T for e in range(N)]
    loss = aux_coeff * N * math.fsum(F[e] * P[e] for e in range(N))
    return dict(y=ys, topk_idx=idxs, topk_w=ws, probs=probs, counts=counts, aux_loss=loss)
