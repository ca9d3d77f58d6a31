"""CPU oracle for the MixLoRA feed-forward block.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
file; the product path never does.  It shares no code with the HIP library.

It is the plain definition of the block written out in float64 NumPy:

* Router (Top-K router paragraph, Eq. 7, and the Norm step of Algorithm 1):
  logits z = W_r x, probabilities p = softmax(z), keep the k largest, divide the
  kept probabilities by their sum.
* Expert (Eq. 1 and Eq. 6, with the SwiGLU shape given in Section 3.3): expert e
  is the frozen FFN  W_down(SiLU(W_gate x) * W_up x)  in which each of the three
  projections has its own low-rank update  W + s B_e A_e  (s = alpha / r, the
  appendix hyper-parameter table).
* Block output (Eq. 2 / Eq. 6): y_t = sum over the kept experts of
  weight * expert output.  The residual add of Eq. 5 is outside this block.
* Auxiliary loss (Eq. 8 and Eq. 9): L = a N sum_i F_i P_i.
* Backward: the reverse-mode derivative of the above with the three base
  matrices frozen and A, B, W_r and x receiving gradients (the paper does not
  print it; it is derived here and pinned by finite differences in the tests).

Every expert is evaluated from the definition on the tokens routed to it
(base projection and low-rank update computed per expert); nothing of
Algorithm 1's shared-projection schedule or of the HIP path's grouping is used.

Readings of the paper where it is silent or inconsistent (listed in full in the
design notes): top-k selection is on the logits with ties going to the lowest
expert index; slots are ordered by descending logit; F_i of Eq. 9 counts the
first-choice expert ("top1", as printed) or all k choices divided by k
("topk"); P_i uses the full softmax; no gradient flows through F_i.

* Several adapters on one frozen base (Section 3.3, "Optimizing Multi-MixLoRA
  Training and Inference (II)", outer loop of Algorithm 1): every token belongs
  to one adapter and is routed and processed by that adapter's router and
  experts only; multi_forward / multi_backward are that definition, adapter by
  adapter, on top of the single-adapter functions.

* Plain LoRA linear (Eq. 1 with the scale of the hyper-parameter table), which the method puts
  on the attention projections (Section 3.2): y = x W^T + s (x A^T) B^T, W frozen;
  lora_linear_forward / lora_linear_backward, pinned in tests/test_oracle_linear_pins.py.

* AdamW (the optimiser of the appendix hyper-parameter table; decoupled weight decay):
  adamw_step, pinned against torch.optim.AdamW in tests/test_oracle_linear_pins.py.

* Weight-decomposed experts ("MixDoRA", named in the experiment setup; the paper prints no
  formula for it, so this is a reading: every expert projection follows the cited
  weight-decomposition method): W'_e = diag(m_e / n_e) (W + s B_e A_e) with a trainable
  magnitude m_e per output feature and n_e the row norms of W + s B_e A_e, which that method
  treats as a constant in the backward pass.  Parity unpinned with respect to the paper (it
  prints nothing to pin to); pinned to that definition: dora_forward / dora_backward, in
  tests/test_oracle_dora_pins.py (m = n reduces to the LoRA block, explicit merged weights,
  homogeneity in m, autograd with the norm detached, finite differences for dm and dx).

Pinned by tests/test_oracle_pins.py (dense-FFN special case, k = N mixture,
merged-weight identity, brute-force loops, closed-form auxiliary losses,
finite differences, autograd of an independent formulation) and, for the
multi-adapter functions, tests/test_oracle_multi_pins.py (one adapter reduces
to the single-adapter block, equality with one large block whose router is
blocked by indicator channels, independence of the adapters, token-order
equivariance, empty adapter).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


def sigmoid(v):
    return 1.0 / (1.0 + np.exp(-v))


def router(x, W_router, k):
    """Eq. 7 + Norm of Algorithm 1.  Returns z, p [T,N]; idx [T,k]; w [T,k]."""
    x = _f64(x)
    W_router = _f64(W_router)
    z = x @ W_router.T
    zmax = z.max(axis=1, keepdims=True)
    ez = np.exp(z - zmax)
    p = ez / ez.sum(axis=1, keepdims=True)
    # stable sort of -z: largest logit first, equal logits keep ascending expert index
    order = np.argsort(-z, axis=1, kind="stable")
    idx = order[:, :k].astype(np.int64)
    kept = np.take_along_axis(p, idx, axis=1)
    w = kept / kept.sum(axis=1, keepdims=True)
    return z, p, idx, w


def aux_loss(probs, topk_idx, N, coeff, mode="top1"):
    """Eq. 8-9.  Returns (loss, F [N], P [N])."""
    probs = _f64(probs)
    topk_idx = np.asarray(topk_idx)
    T = probs.shape[0]
    if mode == "top1":
        F = np.bincount(topk_idx[:, 0], minlength=N).astype(F64) / T
    elif mode == "topk":
        F = np.bincount(topk_idx.reshape(-1), minlength=N).astype(F64) / (T * topk_idx.shape[1])
    else:
        raise ValueError(mode)
    P = probs.sum(axis=0) / T
    return coeff * N * float((F * P).sum()), F, P


def aux_loss_dprobs(probs, topk_idx, N, coeff, mode="top1"):
    """d L_aux / d probs [T,N]; F_i is piecewise constant so only P_i carries gradient."""
    T = np.asarray(probs).shape[0]
    _, F, _ = aux_loss(probs, topk_idx, N, coeff, mode)
    return np.broadcast_to(coeff * N * F / T, (T, N)).copy()


def expert_forward(xe, W, e, s):
    """One expert (Eq. 1 on each projection, SwiGLU of Section 3.3) on rows xe [n,d]."""
    pg = xe @ W["A_gate"][e].T                       # [n,r]
    pu = xe @ W["A_up"][e].T
    g = xe @ W["W_gate"].T + s * (pg @ W["B_gate"][e].T)   # [n,f]
    u = xe @ W["W_up"].T + s * (pu @ W["B_up"][e].T)
    a = g * sigmoid(g) * u
    q = a @ W["A_down"][e].T                         # [n,r]
    o = a @ W["W_down"].T + s * (q @ W["B_down"][e].T)     # [n,d]
    return dict(pg=pg, pu=pu, g=g, u=u, a=a, q=q, o=o)


def forward(x, W, k, lora_scale, aux_coeff=0.01, aux_mode="top1", keep=False):
    """Whole block.  W: dict of arrays (any float dtype).  Returns a dict with
    y [T,d], probs, logits, topk_idx, topk_w, counts [N], aux_loss, F, P
    (and the per-expert intermediates when keep=True)."""
    x = _f64(x)
    W = {n: _f64(v) for n, v in W.items()}
    T, d = x.shape
    N = W["W_router"].shape[0]
    z, p, idx, w = router(x, W["W_router"], k)
    y = np.zeros((T, d), dtype=F64)
    counts = np.zeros(N, dtype=np.int64)
    saved = {}
    for e in range(N):
        tok, slot = np.nonzero(idx == e)
        counts[e] = tok.size
        if tok.size == 0:
            continue
        res = expert_forward(x[tok], W, e, lora_scale)
        np.add.at(y, tok, w[tok, slot][:, None] * res["o"])
        if keep:
            res["tok"], res["slot"] = tok, slot
            saved[e] = res
    loss, F, P = aux_loss(p, idx, N, aux_coeff, aux_mode)
    out = dict(y=y, logits=z, probs=p, topk_idx=idx, topk_w=w, counts=counts,
               aux_loss=loss, F=F, P=P)
    if keep:
        out["saved"] = saved
    return out


def backward(x, W, k, lora_scale, dy, d_aux=1.0, aux_coeff=0.01, aux_mode="top1"):
    """Gradients of  <y, dy> + d_aux * L_aux  with W_gate, W_up, W_down frozen.

    Returns dict: dx [T,d], dA_gate/dA_up [N,r,d], dB_gate/dB_up [N,f,r],
    dA_down [N,r,f], dB_down [N,d,r], dW_router [N,d], plus dw [T,k] and dz [T,N]."""
    x = _f64(x)
    dy = _f64(dy)
    W = {n: _f64(v) for n, v in W.items()}
    s = lora_scale
    fw = forward(x, W, k, s, aux_coeff, aux_mode, keep=True)
    T, d = x.shape
    N = W["W_router"].shape[0]
    p, idx, w = fw["probs"], fw["topk_idx"], fw["topk_w"]
    G = {n: np.zeros_like(W[n]) for n in
         ("A_gate", "B_gate", "A_up", "B_up", "A_down", "B_down", "W_router")}
    dx = np.zeros_like(x)
    dw = np.zeros((T, k), dtype=F64)
    for e, sv in fw["saved"].items():
        tok, slot = sv["tok"], sv["slot"]
        xe, dye = x[tok], dy[tok]
        dw[tok, slot] = (dye * sv["o"]).sum(axis=1)
        do = w[tok, slot][:, None] * dye                     # [n,d]
        # down projection  o = a W_d^T + s (a A_d^T) B_d^T
        G["B_down"][e] = s * (do.T @ sv["q"])                # [d,r]
        v = do @ W["B_down"][e]                              # [n,r]
        G["A_down"][e] = s * (v.T @ sv["a"])                 # [r,f]
        da = do @ W["W_down"] + s * (v @ W["A_down"][e])     # [n,f]
        # a = g sigmoid(g) u
        g, u = sv["g"], sv["u"]
        sg = sigmoid(g)
        dg = da * u * sg * (1.0 + g * (1.0 - sg))
        du = da * g * sg
        # gate / up projections
        G["B_gate"][e] = s * (dg.T @ sv["pg"])               # [f,r]
        tg = dg @ W["B_gate"][e]                             # [n,r]
        G["A_gate"][e] = s * (tg.T @ xe)                     # [r,d]
        G["B_up"][e] = s * (du.T @ sv["pu"])
        tu = du @ W["B_up"][e]
        G["A_up"][e] = s * (tu.T @ xe)
        dxe = dg @ W["W_gate"] + du @ W["W_up"] + s * (tg @ W["A_gate"][e]) \
            + s * (tu @ W["A_up"][e])
        np.add.at(dx, tok, dxe)
    # router: w = p_S / sum(p_S) on the kept set, zero elsewhere
    kept = np.take_along_axis(p, idx, axis=1)
    ssum = kept.sum(axis=1, keepdims=True)
    dkept = (dw - (w * dw).sum(axis=1, keepdims=True)) / ssum
    dp = np.zeros((T, N), dtype=F64)
    np.put_along_axis(dp, idx, dkept, axis=1)
    dp += d_aux * aux_loss_dprobs(p, idx, N, aux_coeff, aux_mode)
    dz = p * (dp - (p * dp).sum(axis=1, keepdims=True))
    G["W_router"] = dz.T @ x
    dx += dz @ W["W_router"]
    out = {"d" + n: v for n, v in G.items()}
    out.update(dx=dx, dw=dw, dz=dz, forward=fw)
    return out


def multi_forward(x, token_model, Ws, k, lora_scale, aux_coeff=0.01, aux_mode="top1"):
    """M adapters sharing the frozen base (Section 3.3, optimisation II; outer loop of
    Algorithm 1).  token_model [T] gives the adapter of every token; Ws is a list of M weight
    dicts with identical W_gate / W_up / W_down.  Adapter m sees only its own tokens.

    Returns y [T,d]; topk_idx [T,k] (expert index inside the token's adapter), topk_w [T,k];
    probs, logits [T,N] over the token's own adapter's experts; counts [M,N]; aux_loss [M] (Eq. 8-9 per
    adapter over its own tokens; 0 for an adapter without tokens)."""
    x = _f64(x)
    token_model = np.asarray(token_model)
    M = len(Ws)
    T, d = x.shape
    N = np.asarray(Ws[0]["W_router"]).shape[0]
    y = np.zeros((T, d), dtype=F64)
    idx = np.zeros((T, k), dtype=np.int64)
    w = np.zeros((T, k), dtype=F64)
    probs = np.zeros((T, N), dtype=F64)
    logits = np.zeros((T, N), dtype=F64)
    counts = np.zeros((M, N), dtype=np.int64)
    aux = np.zeros(M, dtype=F64)
    for m in range(M):
        tok = np.nonzero(token_model == m)[0]
        if tok.size == 0:
            continue
        fw = forward(x[tok], Ws[m], k, lora_scale, aux_coeff, aux_mode)
        y[tok] = fw["y"]
        idx[tok] = fw["topk_idx"]
        w[tok] = fw["topk_w"]
        probs[tok] = fw["probs"]
        logits[tok] = fw["logits"]
        counts[m] = fw["counts"]
        aux[m] = fw["aux_loss"]
    return dict(y=y, topk_idx=idx, topk_w=w, probs=probs, logits=logits, counts=counts,
                aux_loss=aux)


def multi_backward(x, token_model, Ws, k, lora_scale, dy, d_aux=None, aux_coeff=0.01,
                   aux_mode="top1"):
    """Gradients of  <y, dy> + sum_m d_aux[m] * L_aux[m]  for the M-adapter block.

    Returns dx [T,d] and, per adapter, the gradient dicts of `backward` in the list "grads"
    (all zeros for an adapter without tokens); dz [T,N] over the token's own adapter."""
    x = _f64(x)
    dy = _f64(dy)
    token_model = np.asarray(token_model)
    M = len(Ws)
    d_aux = np.ones(M) if d_aux is None else np.asarray(d_aux, dtype=F64)
    N = np.asarray(Ws[0]["W_router"]).shape[0]
    dx = np.zeros_like(x)
    dz = np.zeros((x.shape[0], N), dtype=F64)
    grads = []
    names = ("A_gate", "B_gate", "A_up", "B_up", "A_down", "B_down", "W_router")
    for m in range(M):
        tok = np.nonzero(token_model == m)[0]
        if tok.size == 0:
            grads.append({"d" + n: np.zeros_like(_f64(Ws[m][n])) for n in names})
            continue
        bw = backward(x[tok], Ws[m], k, lora_scale, dy[tok], float(d_aux[m]), aux_coeff, aux_mode)
        dx[tok] = bw["dx"]
        dz[tok] = bw["dz"]
        grads.append({"d" + n: bw["d" + n] for n in names})
    return dict(dx=dx, dz=dz, grads=grads)


def lora_linear_forward(x, W, A, B, lora_scale):
    """Eq. 1 with scale: y = x W^T + s (x A^T) B^T.  x [T,d_in], W [d_out,d_in] (frozen),
    A [r,d_in], B [d_out,r].  Returns y [T,d_out]."""
    x, W, A, B = _f64(x), _f64(W), _f64(A), _f64(B)
    return x @ W.T + lora_scale * ((x @ A.T) @ B.T)


def lora_linear_backward(x, W, A, B, lora_scale, dy):
    """Gradients of <y, dy> with W frozen: dx [T,d_in], dA [r,d_in], dB [d_out,r]."""
    x, W, A, B, dy = _f64(x), _f64(W), _f64(A), _f64(B), _f64(dy)
    p = x @ A.T                      # [T,r]
    v = dy @ B                       # [T,r]
    dx = dy @ W + lora_scale * (v @ A)
    dA = lora_scale * (v.T @ x)
    dB = lora_scale * (dy.T @ p)
    return dict(dx=dx, dA=dA, dB=dB)


def adamw_step(p, g, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """One AdamW update (decoupled weight decay); step is 1-based.  Returns (p, m, v)."""
    p, g, m, v = _f64(p), _f64(g), _f64(m), _f64(v)
    p = p * (1.0 - lr * weight_decay)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    p = p - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


# ---- weight-decomposed experts (reading of "MixDoRA", see the header) ---------------------------
DORA_PROJ = (("gate", "W_gate", "A_gate", "B_gate"), ("up", "W_up", "A_up", "B_up"),
             ("down", "W_down", "A_down", "B_down"))


def dora_row_norms(W, e, s):
    """n_e per projection: L2 norm over the input dimension of every row of W + s B_e A_e."""
    out = {}
    for name, wn, an, bn in DORA_PROJ:
        V = _f64(W[wn]) + s * (_f64(W[bn][e]) @ _f64(W[an][e]))
        out[name] = np.sqrt((V * V).sum(axis=1))
    return out


def dora_magnitude(mag, nm, e):
    """Magnitude vector of projection nm for expert e.  Two readings of the variant (the paper
    prints no formula): a magnitude per expert, arrays [N, out]; or ONE magnitude per projection
    used by every expert, m_e = m, arrays [out] - the reading under which the "# Params" columns of
    the rank study and of the main results stay the same for MixLoRA and MixDoRA."""
    m = _f64(mag["m_" + nm])
    return m[e] if m.ndim == 2 else m


def dora_expert_forward(xe, W, mag, e, s):
    """One weight-decomposed expert on rows xe [n,d]: every projection's output feature j is
    (m_e[j] / n_e[j]) * ((W + s B_e A_e) x)[j].  mag: dict m_gate/m_up [N,f], m_down [N,d], or
    [f], [f], [d] for magnitudes shared by the experts."""
    n = dora_row_norms(W, e, s)
    cg, cu, cd = (dora_magnitude(mag, nm, e) / n[nm] for nm in ("gate", "up", "down"))
    pg = xe @ W["A_gate"][e].T
    pu = xe @ W["A_up"][e].T
    vg = xe @ W["W_gate"].T + s * (pg @ W["B_gate"][e].T)
    vu = xe @ W["W_up"].T + s * (pu @ W["B_up"][e].T)
    g, u = cg * vg, cu * vu
    a = g * sigmoid(g) * u
    q = a @ W["A_down"][e].T
    vd = a @ W["W_down"].T + s * (q @ W["B_down"][e].T)
    o = cd * vd
    return dict(pg=pg, pu=pu, vg=vg, vu=vu, g=g, u=u, a=a, q=q, vd=vd, o=o, cg=cg, cu=cu, cd=cd,
                n=n)


def dora_forward(x, W, mag, k, lora_scale, aux_coeff=0.01, aux_mode="top1", keep=False):
    """The block with weight-decomposed experts; routing, combination and auxiliary loss as in
    forward().  Returns the same dict."""
    x = _f64(x)
    W = {n: _f64(v) for n, v in W.items()}
    T, d = x.shape
    N = W["W_router"].shape[0]
    z, p, idx, w = router(x, W["W_router"], k)
    y = np.zeros((T, d), dtype=F64)
    counts = np.zeros(N, dtype=np.int64)
    saved = {}
    for e in range(N):
        tok, slot = np.nonzero(idx == e)
        counts[e] = tok.size
        if tok.size == 0:
            continue
        res = dora_expert_forward(x[tok], W, mag, e, lora_scale)
        np.add.at(y, tok, w[tok, slot][:, None] * res["o"])
        if keep:
            res["tok"], res["slot"] = tok, slot
            saved[e] = res
    loss, F, P = aux_loss(p, idx, N, aux_coeff, aux_mode)
    out = dict(y=y, logits=z, probs=p, topk_idx=idx, topk_w=w, counts=counts,
               aux_loss=loss, F=F, P=P)
    if keep:
        out["saved"] = saved
    return out


def dora_backward(x, W, mag, k, lora_scale, dy, d_aux=1.0, aux_coeff=0.01, aux_mode="top1"):
    """Gradients of <y, dy> + d_aux * L_aux for the weight-decomposed block: base matrices
    frozen, the row norms n_e held constant (no gradient flows through them), gradients for
    A, B, the magnitudes (dm_gate/dm_up [N,f], dm_down [N,d]; with shared magnitudes [f], [f],
    [d]: every expert's term lands on the same vector, so the terms add up), W_router and x."""
    x = _f64(x)
    dy = _f64(dy)
    W = {n: _f64(v) for n, v in W.items()}
    s = lora_scale
    fw = dora_forward(x, W, mag, k, s, aux_coeff, aux_mode, keep=True)
    T, d = x.shape
    N = W["W_router"].shape[0]
    p, idx, w = fw["probs"], fw["topk_idx"], fw["topk_w"]
    G = {n: np.zeros_like(W[n]) for n in
         ("A_gate", "B_gate", "A_up", "B_up", "A_down", "B_down", "W_router")}
    dm = {"m_" + nm: np.zeros_like(_f64(mag["m_" + nm])) for nm in ("gate", "up", "down")}
    dx = np.zeros_like(x)
    dw = np.zeros((T, k), dtype=F64)
    for e, sv in fw["saved"].items():
        tok, slot = sv["tok"], sv["slot"]
        xe, dye = x[tok], dy[tok]
        dw[tok, slot] = (dye * sv["o"]).sum(axis=1)
        do = w[tok, slot][:, None] * dye
        # o = cd * vd,  cd = m_down / n_down
        def add_dm(nm, term):   # per expert: row e; shared: the one vector
            if dm["m_" + nm].ndim == 2:
                dm["m_" + nm][e] = term
            else:
                dm["m_" + nm] += term
        add_dm("down", (do * sv["vd"]).sum(axis=0) / sv["n"]["down"])
        dvd = do * sv["cd"]
        G["B_down"][e] = s * (dvd.T @ sv["q"])
        v = dvd @ W["B_down"][e]
        G["A_down"][e] = s * (v.T @ sv["a"])
        da = dvd @ W["W_down"] + s * (v @ W["A_down"][e])
        g, u = sv["g"], sv["u"]
        sg = sigmoid(g)
        dg = da * u * sg * (1.0 + g * (1.0 - sg))
        du = da * g * sg
        add_dm("gate", (dg * sv["vg"]).sum(axis=0) / sv["n"]["gate"])
        add_dm("up", (du * sv["vu"]).sum(axis=0) / sv["n"]["up"])
        dvg, dvu = dg * sv["cg"], du * sv["cu"]
        G["B_gate"][e] = s * (dvg.T @ sv["pg"])
        tg = dvg @ W["B_gate"][e]
        G["A_gate"][e] = s * (tg.T @ xe)
        G["B_up"][e] = s * (dvu.T @ sv["pu"])
        tu = dvu @ W["B_up"][e]
        G["A_up"][e] = s * (tu.T @ xe)
        dxe = dvg @ W["W_gate"] + dvu @ W["W_up"] + s * (tg @ W["A_gate"][e]) \
            + s * (tu @ W["A_up"][e])
        np.add.at(dx, tok, dxe)
    kept = np.take_along_axis(p, idx, axis=1)
    ssum = kept.sum(axis=1, keepdims=True)
    dkept = (dw - (w * dw).sum(axis=1, keepdims=True)) / ssum
    dp = np.zeros((T, N), dtype=F64)
    np.put_along_axis(dp, idx, dkept, axis=1)
    dp += d_aux * aux_loss_dprobs(p, idx, N, aux_coeff, aux_mode)
    dz = p * (dp - (p * dp).sum(axis=1, keepdims=True))
    G["W_router"] = dz.T @ x
    dx += dz @ W["W_router"]
    out = {"d" + n: v for n, v in G.items()}
    out.update({"d" + n: v for n, v in dm.items()})
    out.update(dx=dx, dw=dw, dz=dz, forward=fw)
    return out
