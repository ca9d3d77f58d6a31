"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, sizes its
workspace sensibly and rejects bad arguments on the host before any HIP call."""
import ctypes as C
import os
import re

import pytest

from paper_2404_15159_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2404_15159_amd import build
        build.build(verbose=False)
    return B.load()


def test_exports_match_header(lib):
    text = open(os.path.join(ROOT, "include", "mixlora.h")).read()
    declared = set(re.findall(r"MIXLORA_API\s+[\w\s\*]+?\b(mixlora_\w+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert B.mixlora_version() >= 100


def dims(**kw):
    base = dict(T=4096, d=4096, d_ff=11008, N=8, k=2, r=16, lora_scale=2.0)
    base.update(kw)
    return B.make_dims(**base)


def test_workspace_bytes(lib):
    d = dims()
    fwd, bwd = B.mixlora_workspace_bytes(d, False), B.mixlora_workspace_bytes(d, True)
    # forward keeps G, U [T,f], the grouped activations [kT,f] and their combination [T,f]
    assert fwd >= 5 * 4096 * 11008 * 2
    assert bwd > fwd
    assert bwd < 8 << 30
    assert B.mixlora_workspace_bytes(dims(T=8192), True) > bwd
    # ranks off the multiples of 8 run on zero-padded banks held in the workspace
    assert B.mixlora_workspace_bytes(dims(r=2), True) > B.mixlora_workspace_bytes(dims(r=8), True)
    assert B.mixlora_workspace_bytes(dims(r=12), False) > B.mixlora_workspace_bytes(dims(r=16), False)
    for bad in (dict(k=0), dict(k=9), dict(N=65), dict(r=0), dict(r=65), dict(N=64, r=12), dict(d=4100),
                dict(d_ff=11004), dict(T=0), dict(dtype=7), dict(aux_mode=3), dict(N=64, r=16),
                dict(T=1 << 23, k=2)):
        assert B.mixlora_workspace_bytes(dims(**bad), True) == 0, bad


FAKE = 0x10000   # a non-null, 16-byte aligned value that is never dereferenced on these paths


def fake_weights(**kw):
    t = {n: FAKE for n in B.WEIGHT_FIELDS[:10]}
    t.update(kw)
    return B.make_weights(t)


def fwd_args(**kw):
    a = dict(x=FAKE, y=FAKE, topk_idx=FAKE, topk_w=FAKE, expert_counts=FAKE, aux_loss=FAKE,
             workspace=FAKE, workspace_bytes=1 << 40)
    a.update(kw)
    return a


def fwd_code(d, w, **kw):
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_ffn_forward(d, w, stream=0, **fwd_args(**kw))
    return ei.value.code


def test_forward_argument_errors(lib):
    assert fwd_code(dims(k=3, N=2), fake_weights()) == -2
    assert fwd_code(dims(dtype=5), fake_weights()) == -3
    assert fwd_code(dims(), fake_weights(W_up=None)) == -1
    assert fwd_code(dims(), fake_weights(B_down=FAKE + 4)) == -4
    assert fwd_code(dims(), fake_weights(), y=None) == -1
    assert fwd_code(dims(), fake_weights(), x=FAKE + 8) == -4
    assert fwd_code(dims(), fake_weights(), workspace_bytes=1024) == -5


def test_forward_static_argument_errors(lib):
    """The forward that keeps its workspace in the library's static device array: the size limit
    and the argument checks are host-side, before any HIP call."""
    def code(d, w, **kw):
        a = fwd_args(**kw)
        a.pop("workspace"), a.pop("workspace_bytes")
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_ffn_forward_static(d, w, stream=0, **a)
        return ei.value.code

    assert B.mixlora_workspace_bytes(dims(), False) > B.STATIC_SCRATCH_BYTES
    assert code(dims(), fake_weights()) == -7                     # 4096 tokens: beyond the array
    assert B.mixlora_workspace_bytes(dims(T=128), False) <= B.STATIC_SCRATCH_BYTES
    assert code(dims(T=128, k=9), fake_weights()) == -2
    assert code(dims(T=128), fake_weights(A_up=None)) == -1
    assert code(dims(T=128), fake_weights(), y=FAKE + 4) == -4
    text = open(os.path.join(ROOT, "include", "mixlora.h")).read()
    m = re.search(r"#define MIXLORA_STATIC_SCRATCH_BYTES \((\d+) \* 1024 \* 1024\)", text)
    assert m and int(m.group(1)) * 1024 * 1024 == B.STATIC_SCRATCH_BYTES


def test_backward_argument_errors(lib):
    g = B.make_grads({n: FAKE for n in B.GRAD_FIELDS})

    def code(d=None, w=None, grads=g, **kw):
        a = dict(x=FAKE, dy=FAKE, d_aux=1.0, workspace=FAKE, workspace_bytes=1 << 40, dx=FAKE)
        a.update(kw)
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_ffn_backward(d or dims(), w or fake_weights(), grads=grads, stream=0, **a)
        return ei.value.code

    assert code(d=dims(r=0)) == -2
    assert code(dy=None) == -1
    assert code(grads=B.make_grads({n: FAKE for n in B.GRAD_FIELDS[:-1]})) == -1
    assert code(dx=FAKE + 2) == -4
    assert code(w=fake_weights(W_gate_T=FAKE + 1)) == -4
    fwd_only = B.mixlora_workspace_bytes(dims(), False)
    assert code(workspace_bytes=fwd_only) == -5


def test_schedule_entry_points(lib):
    """The paper's own schedules: workspace grows with the per-pair rows, bad schedules / dtypes /
    workspaces are rejected on the host."""
    d = dims()
    ws = [B.mixlora_schedule_workspace_bytes(d, sch, True)
          for sch in (B.SCHEDULE_LINEAR_DOWN, B.SCHEDULE_SHARED, B.SCHEDULE_VANILLA)]
    assert ws[0] == B.mixlora_workspace_bytes(d, True)
    assert ws[0] < ws[1] < ws[2]
    # shared: the down projection's output and its backward input exist per pair row [kT, d]
    assert ws[1] - ws[0] >= 2 * (2 * 4096) * 4096 * 2
    # unshared: also the gathered token rows [kT, d] and their gradient [kT, d]
    assert ws[2] - ws[1] >= 2 * (2 * 4096) * 4096 * 2
    assert B.mixlora_schedule_workspace_bytes(d, 3, True) == 0
    assert B.mixlora_schedule_workspace_bytes(d, -1, True) == 0
    assert B.mixlora_schedule_workspace_bytes(dims(dtype=B.F32), B.SCHEDULE_SHARED, True) == 0
    assert B.mixlora_schedule_workspace_bytes(dims(dtype=B.F32), B.SCHEDULE_LINEAR_DOWN, True) > 0

    def fcode(dd, sch, **kw):
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_ffn_forward_schedule(dd, sch, fake_weights(), stream=0, **fwd_args(**kw))
        return ei.value.code

    assert fcode(d, 5) == -2
    assert fcode(dims(dtype=B.F32), B.SCHEDULE_VANILLA) == -3
    assert fcode(d, B.SCHEDULE_SHARED, y=None) == -1
    assert fcode(d, B.SCHEDULE_VANILLA, workspace_bytes=B.mixlora_workspace_bytes(d, False)) == -5
    g = B.make_grads({n: FAKE for n in B.GRAD_FIELDS})
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_ffn_backward_schedule(d, B.SCHEDULE_VANILLA, fake_weights(), FAKE, FAKE, 1.0, FAKE,
                                        ws[0], FAKE, g, stream=0)
    assert ei.value.code == -5
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_ffn_backward_schedule(d, 9, fake_weights(), FAKE, FAKE, 1.0, FAKE, 1 << 40, FAKE,
                                        g, stream=0)
    assert ei.value.code == -2


def test_dora_entry_points(lib):
    """Weight-decomposed expert variant: bf16 only, magnitudes and their gradients required."""
    d = dims()
    ws = B.mixlora_dora_workspace_bytes(d, True)
    assert ws > B.mixlora_schedule_workspace_bytes(d, B.SCHEDULE_SHARED, True)
    assert B.mixlora_dora_workspace_bytes(d, False) < ws
    assert B.mixlora_dora_workspace_bytes(dims(dtype=B.F32), True) == 0
    assert B.mixlora_dora_workspace_bytes(dims(r=65), True) == 0
    mags = B.make_dora({n: FAKE for n in B.DORA_FIELDS})

    def fcode(dd=d, dora=mags, **kw):
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_dora_forward(dd, fake_weights(), dora, stream=0, **fwd_args(**kw))
        return ei.value.code

    assert fcode(dd=dims(dtype=B.F32)) == -3
    assert fcode(dora=B.make_dora({"m_gate": FAKE, "m_up": FAKE})) == -1
    assert fcode(dora=B.make_dora({"m_gate": FAKE, "m_up": FAKE, "m_down": FAKE + 4})) == -4
    assert fcode(x=None) == -1
    assert fcode(workspace_bytes=B.mixlora_dora_workspace_bytes(d, False) - 256) == -5
    g = B.make_grads({n: FAKE for n in B.GRAD_FIELDS})
    dg = B.make_dora_grads({n: FAKE for n in B.DORA_GRAD_FIELDS})

    def bcode(dgrads=dg, ws_bytes=1 << 40):
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_dora_backward(d, fake_weights(), mags, FAKE, FAKE, 1.0, FAKE, ws_bytes, FAKE, g,
                                    dgrads, stream=0)
        return ei.value.code

    assert bcode(dgrads=B.make_dora_grads({"dm_gate": FAKE})) == -1
    assert bcode(dgrads=B.make_dora_grads({n: FAKE + 2 for n in B.DORA_GRAD_FIELDS})) == -4
    assert bcode(ws_bytes=B.mixlora_dora_workspace_bytes(d, False)) == -5


def test_aux_and_transpose_argument_errors(lib):
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_aux_loss(FAKE, FAKE, 16, 4, 5, 0.01, 0, FAKE, stream=0)
    assert ei.value.code == -2
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_aux_loss(FAKE, None, 16, 4, 2, 0.01, 0, FAKE, stream=0)
    assert ei.value.code == -1
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_aux_loss(FAKE, FAKE, 16, 4, 2, 0.01, 9, FAKE, stream=0)
    assert ei.value.code == -3
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_transpose(FAKE, FAKE, 0, 4, 1, stream=0)
    assert ei.value.code == -2
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_transpose(FAKE, FAKE, 4, 4, 3, stream=0)
    assert ei.value.code == -3


def test_multi_adapter_argument_errors(lib):
    d = dims()
    assert B.mixlora_multi_workspace_bytes(d, 1, True) == B.mixlora_workspace_bytes(d, True)
    assert B.mixlora_multi_workspace_bytes(d, 2, True) == B.mixlora_workspace_bytes(dims(N=16), True)
    for M in (0, -1, 9):          # 9 * 8 experts > 64
        assert B.mixlora_multi_workspace_bytes(d, M, True) == 0
    assert B.mixlora_multi_workspace_bytes(d, 5, True) == 0          # 5 * 8 * 16 > 512 rank columns
    assert B.mixlora_multi_workspace_bytes(dims(N=2, k=3), 4, True) == 0   # k > experts per adapter

    def fcode(d_, multi, w=None, **kw):
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_multi_forward(d_, multi, w or fake_weights(), stream=0, **fwd_args(**kw))
        return ei.value.code

    assert fcode(d, B.make_multi(0, FAKE)) == -2
    assert fcode(d, B.make_multi(9, FAKE)) == -2
    assert fcode(d, B.make_multi(2, None)) == -1
    assert fcode(dims(N=2, k=3), B.make_multi(4, FAKE)) == -2
    assert fcode(d, B.make_multi(2, FAKE), y=None) == -1
    assert fcode(d, B.make_multi(2, FAKE), workspace_bytes=1024) == -5
    g = B.make_grads({n: FAKE for n in B.GRAD_FIELDS})
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_multi_backward(d, B.make_multi(2, FAKE, (1.0, 2.0)), fake_weights(), FAKE, None,
                                 FAKE, 1 << 40, FAKE, g, stream=0)
    assert ei.value.code == -1
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_multi_backward(d, B.make_multi(2, FAKE), fake_weights(), FAKE, FAKE, FAKE,
                                 B.mixlora_multi_workspace_bytes(d, 2, False), FAKE, g, stream=0)
    assert ei.value.code == -5


def test_lora_linear_argument_errors(lib):
    def ld(**kw):
        a = dict(T=4096, d_in=4096, d_out=4096, r=16, lora_scale=2.0, dtype=B.BF16)
        a.update(kw)
        return B.LinearDims(a["T"], a["d_in"], a["d_out"], a["r"], a["lora_scale"], a["dtype"])

    fwd, bwd = (B.mixlora_lora_linear_workspace_bytes(ld(), f) for f in (False, True))
    assert 4096 * 16 * 4 <= fwd < bwd
    for bad in (dict(T=0), dict(r=0), dict(r=72), dict(d_in=4100), dict(d_out=4), dict(dtype=3)):
        assert B.mixlora_lora_linear_workspace_bytes(ld(**bad), True) == 0, bad

    def fcode(d_, **kw):
        a = dict(W=FAKE, A=FAKE, B_=FAKE, x=FAKE, y=FAKE, workspace=FAKE, workspace_bytes=1 << 40)
        a.update(kw)
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_lora_linear_forward(d_, stream=0, **a)
        return ei.value.code

    assert fcode(ld(r=65)) == -2
    assert fcode(ld(dtype=9)) == -3
    assert fcode(ld(), A=None) == -1
    assert fcode(ld(), x=FAKE + 4) == -4
    assert fcode(ld(), workspace_bytes=16) == -5

    def bcode(d_, **kw):
        a = dict(W=FAKE, W_T=None, A=FAKE, B_=FAKE, x=FAKE, dy=FAKE, workspace=FAKE,
                 workspace_bytes=1 << 40, dx=FAKE, dA=FAKE, dB=FAKE)
        a.update(kw)
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_lora_linear_backward(d_, stream=0, **a)
        return ei.value.code

    assert bcode(ld(d_in=12)) == -2
    assert bcode(ld(), dB=None) == -1
    assert bcode(ld(), W_T=FAKE + 2) == -4
    assert bcode(ld(), workspace_bytes=fwd) == -5


def test_adamw_argument_errors(lib):
    ok = dict(lr=2e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1)

    def code(n=16, param=FAKE, lowp=None, lowp_dtype=B.BF16, **kw):
        a = dict(ok); a.update(kw)
        h = B.AdamW(a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"], a["step"])
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_adamw_step(h, n, param, FAKE, FAKE, FAKE, lowp, lowp_dtype, stream=0)
        return ei.value.code

    assert code(param=None) == -1
    assert code(n=0) == -2
    assert code(step=0) == -2
    assert code(beta1=1.0) == -2
    assert code(eps=0.0) == -2
    assert code(lowp=FAKE, lowp_dtype=5) == -3


def test_mfma_probe_argument_errors(lib):
    for kw, code in ((dict(sink=None), -1), (dict(waves_per_simd=0), -2), (dict(waves_per_simd=3), -2),
                     (dict(iters=0), -2)):
        a = dict(sink=FAKE, sink_bytes=1 << 30, waves_per_simd=1, iters=10)
        a.update(kw)
        with pytest.raises(B.MixLoraError) as ei:
            B.mixlora_mfma_probe(stream=0, **a)
        assert ei.value.code == code, kw


def test_binding_refuses_missing_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        B.load()
