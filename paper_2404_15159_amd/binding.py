"""Thin ctypes binding over libmixlora.so: argument marshalling only.

Every step of the block runs inside the library's HIP kernels; PyTorch is used here for
device memory (tensors' data_ptr) and the current stream's handle.  The functions carry the
same names as the C entry points (see include/mixlora.h for the full contract).
There is no CPU fallback: load() raises if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
# MIXLORA_LIB: another build of the same library (e.g. the host-sanitizer build of build.py)
LIB_PATH = os.environ.get("MIXLORA_LIB") or os.path.join(HERE, "libmixlora.so")

F32, BF16 = 0, 1
AUX_TOP1, AUX_TOPK = 0, 1
SCHEDULE_LINEAR_DOWN, SCHEDULE_SHARED, SCHEDULE_VANILLA = 0, 1, 2
STATUS = {0: "OK", -1: "E_NULL", -2: "E_SHAPE", -3: "E_DTYPE", -4: "E_ALIGN", -5: "E_WORKSPACE",
          -6: "E_HIP", -7: "E_SCRATCH"}
STATIC_SCRATCH_BYTES = 40 * 1024 * 1024

EXPORTS = ("mixlora_workspace_bytes", "mixlora_ffn_forward", "mixlora_ffn_backward",
           "mixlora_aux_loss", "mixlora_transpose", "mixlora_version",
           "mixlora_profile_begin", "mixlora_profile_end", "mixlora_profile_kind",
           "mixlora_multi_workspace_bytes", "mixlora_multi_forward", "mixlora_multi_backward",
           "mixlora_mfma_probe", "mixlora_lora_linear_workspace_bytes",
           "mixlora_lora_linear_forward", "mixlora_lora_linear_backward", "mixlora_adamw_step",
           "mixlora_schedule_workspace_bytes", "mixlora_ffn_forward_schedule",
           "mixlora_ffn_backward_schedule", "mixlora_dora_workspace_bytes",
           "mixlora_dora_forward", "mixlora_dora_backward", "mixlora_ffn_forward_static")


class Dims(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("d_ff", C.c_int32), ("N", C.c_int32),
                ("k", C.c_int32), ("r", C.c_int32), ("lora_scale", C.c_float),
                ("aux_coeff", C.c_float), ("aux_mode", C.c_int32), ("dtype", C.c_int32)]


WEIGHT_FIELDS = ("W_gate", "W_up", "W_down", "A_gate", "B_gate", "A_up", "B_up", "A_down",
                 "B_down", "W_router", "W_gate_T", "W_up_T", "W_down_T")
GRAD_FIELDS = ("dA_gate", "dB_gate", "dA_up", "dB_up", "dA_down", "dB_down", "dW_router")


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class Grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in GRAD_FIELDS]


class LinearDims(C.Structure):
    _fields_ = [("T", C.c_int32), ("d_in", C.c_int32), ("d_out", C.c_int32), ("r", C.c_int32),
                ("lora_scale", C.c_float), ("dtype", C.c_int32)]


class AdamW(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("step", C.c_int32)]


DORA_FIELDS = ("m_gate", "m_up", "m_down")
DORA_GRAD_FIELDS = ("dm_gate", "dm_up", "dm_down")


class Dora(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in DORA_FIELDS] + [("shared", C.c_int32)]


class DoraGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in DORA_GRAD_FIELDS]


class Multi(C.Structure):
    _fields_ = [("M", C.c_int32), ("token_model", C.c_void_p), ("d_aux", C.POINTER(C.c_float))]


class MixLoraError(RuntimeError):
    def __init__(self, fn: str, code: int):
        super().__init__(f"{fn} returned {code} ({STATUS.get(code, '?')})")
        self.code = code


_lib = None


def load():
    """Load the HIP library (once).  Raises if it is missing: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not built; run `python -m paper_2404_15159_amd.build`")
    # The device pointers callers pass come from PyTorch, which ships its own copy of the HIP
    # runtime.  It has to be in the process before this library is, so that both use the same
    # runtime: loaded the other way round the process ends up with two, and every launch on a
    # torch tensor fails with MIXLORA_E_HIP.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    lib.mixlora_workspace_bytes.restype = sz
    lib.mixlora_workspace_bytes.argtypes = [C.POINTER(Dims), C.c_int]
    lib.mixlora_ffn_forward.restype = C.c_int
    lib.mixlora_ffn_forward.argtypes = [C.POINTER(Dims), C.POINTER(Weights), vp, vp, vp, vp, vp,
                                        vp, vp, sz, vp]
    lib.mixlora_ffn_forward_static.restype = C.c_int
    lib.mixlora_ffn_forward_static.argtypes = [C.POINTER(Dims), C.POINTER(Weights), vp, vp, vp, vp,
                                               vp, vp, vp]
    lib.mixlora_ffn_backward.restype = C.c_int
    lib.mixlora_ffn_backward.argtypes = [C.POINTER(Dims), C.POINTER(Weights), vp, vp, f32, vp, sz,
                                         vp, C.POINTER(Grads), vp]
    lib.mixlora_schedule_workspace_bytes.restype = sz
    lib.mixlora_schedule_workspace_bytes.argtypes = [C.POINTER(Dims), i32, C.c_int]
    lib.mixlora_ffn_forward_schedule.restype = C.c_int
    lib.mixlora_ffn_forward_schedule.argtypes = [C.POINTER(Dims), i32, C.POINTER(Weights), vp, vp,
                                                 vp, vp, vp, vp, vp, sz, vp]
    lib.mixlora_ffn_backward_schedule.restype = C.c_int
    lib.mixlora_ffn_backward_schedule.argtypes = [C.POINTER(Dims), i32, C.POINTER(Weights), vp, vp,
                                                  f32, vp, sz, vp, C.POINTER(Grads), vp]
    lib.mixlora_dora_workspace_bytes.restype = sz
    lib.mixlora_dora_workspace_bytes.argtypes = [C.POINTER(Dims), C.c_int]
    lib.mixlora_dora_forward.restype = C.c_int
    lib.mixlora_dora_forward.argtypes = [C.POINTER(Dims), C.POINTER(Weights), C.POINTER(Dora), vp, vp,
                                         vp, vp, vp, vp, vp, sz, vp]
    lib.mixlora_dora_backward.restype = C.c_int
    lib.mixlora_dora_backward.argtypes = [C.POINTER(Dims), C.POINTER(Weights), C.POINTER(Dora), vp, vp,
                                          f32, vp, sz, vp, C.POINTER(Grads), C.POINTER(DoraGrads), vp]
    lib.mixlora_aux_loss.restype = C.c_int
    lib.mixlora_aux_loss.argtypes = [vp, vp, i32, i32, i32, f32, i32, vp, vp, vp, vp, vp]
    lib.mixlora_transpose.restype = C.c_int
    lib.mixlora_transpose.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.mixlora_version.restype = C.c_int
    lib.mixlora_version.argtypes = []
    lib.mixlora_profile_begin.restype = C.c_int
    lib.mixlora_profile_begin.argtypes = [i32]
    lib.mixlora_profile_end.restype = C.c_int
    lib.mixlora_profile_end.argtypes = [C.POINTER(C.c_double), C.POINTER(i32),
                                        C.POINTER(C.c_double)]
    lib.mixlora_profile_kind.restype = C.c_int
    lib.mixlora_profile_kind.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(i32),
                                         C.POINTER(C.c_double)]
    lib.mixlora_multi_workspace_bytes.restype = sz
    lib.mixlora_multi_workspace_bytes.argtypes = [C.POINTER(Dims), i32, C.c_int]
    lib.mixlora_multi_forward.restype = C.c_int
    lib.mixlora_multi_forward.argtypes = [C.POINTER(Dims), C.POINTER(Multi), C.POINTER(Weights), vp,
                                          vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mixlora_multi_backward.restype = C.c_int
    lib.mixlora_multi_backward.argtypes = [C.POINTER(Dims), C.POINTER(Multi), C.POINTER(Weights),
                                           vp, vp, vp, sz, vp, C.POINTER(Grads), vp]
    lib.mixlora_lora_linear_workspace_bytes.restype = sz
    lib.mixlora_lora_linear_workspace_bytes.argtypes = [C.POINTER(LinearDims), C.c_int]
    lib.mixlora_lora_linear_forward.restype = C.c_int
    lib.mixlora_lora_linear_forward.argtypes = [C.POINTER(LinearDims), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mixlora_lora_linear_backward.restype = C.c_int
    lib.mixlora_lora_linear_backward.argtypes = [C.POINTER(LinearDims), vp, vp, vp, vp, vp, vp, vp,
                                                 sz, vp, vp, vp, vp]
    lib.mixlora_adamw_step.restype = C.c_int
    lib.mixlora_adamw_step.argtypes = [C.POINTER(AdamW), C.c_int64, vp, vp, vp, vp, vp, i32, vp]
    lib.mixlora_mfma_probe.restype = C.c_int
    lib.mixlora_mfma_probe.argtypes = [vp, sz, i32, i32, C.POINTER(C.c_double), vp]
    _lib = lib
    return lib


def make_dims(T, d, d_ff, N, k, r, lora_scale, aux_coeff=0.01, aux_mode=AUX_TOP1, dtype=BF16):
    return Dims(T, d, d_ff, N, k, r, lora_scale, aux_coeff, aux_mode, dtype)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def make_weights(tensors: Dict[str, object]) -> Weights:
    """tensors: name -> device tensor (or raw pointer); the three *_T entries are optional."""
    w = Weights()
    for n in WEIGHT_FIELDS:
        setattr(w, n, _ptr(tensors.get(n)))
    return w


def make_grads(tensors: Dict[str, object]) -> Grads:
    g = Grads()
    for n in GRAD_FIELDS:
        setattr(g, n, _ptr(tensors.get(n)))
    return g


def mixlora_workspace_bytes(dims: Dims, for_backward: bool) -> int:
    return int(load().mixlora_workspace_bytes(C.byref(dims), int(bool(for_backward))))


def mixlora_ffn_forward(dims: Dims, weights: Weights, x, y, topk_idx, topk_w, expert_counts,
                        aux_loss, workspace, workspace_bytes: int, stream=None) -> None:
    rc = load().mixlora_ffn_forward(C.byref(dims), C.byref(weights), _ptr(x), _ptr(y),
                                    _ptr(topk_idx), _ptr(topk_w), _ptr(expert_counts),
                                    _ptr(aux_loss), _ptr(workspace), workspace_bytes,
                                    _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_ffn_forward", rc)


def mixlora_ffn_forward_static(dims: Dims, weights: Weights, x, y, topk_idx, topk_w,
                               expert_counts, aux_loss, stream=None) -> None:
    rc = load().mixlora_ffn_forward_static(C.byref(dims), C.byref(weights), _ptr(x), _ptr(y),
                                           _ptr(topk_idx), _ptr(topk_w), _ptr(expert_counts),
                                           _ptr(aux_loss), _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_ffn_forward_static", rc)


def mixlora_ffn_backward(dims: Dims, weights: Weights, x, dy, d_aux: float, workspace,
                         workspace_bytes: int, dx, grads: Grads, stream=None) -> None:
    rc = load().mixlora_ffn_backward(C.byref(dims), C.byref(weights), _ptr(x), _ptr(dy),
                                     float(d_aux), _ptr(workspace), workspace_bytes, _ptr(dx),
                                     C.byref(grads), _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_ffn_backward", rc)


def mixlora_schedule_workspace_bytes(dims: Dims, schedule: int, for_backward: bool) -> int:
    return int(load().mixlora_schedule_workspace_bytes(C.byref(dims), int(schedule),
                                                       int(bool(for_backward))))


def mixlora_ffn_forward_schedule(dims: Dims, schedule: int, weights: Weights, x, y, topk_idx,
                                 topk_w, expert_counts, aux_loss, workspace,
                                 workspace_bytes: int, stream=None) -> None:
    rc = load().mixlora_ffn_forward_schedule(C.byref(dims), int(schedule), C.byref(weights),
                                             _ptr(x), _ptr(y), _ptr(topk_idx), _ptr(topk_w),
                                             _ptr(expert_counts), _ptr(aux_loss), _ptr(workspace),
                                             workspace_bytes, _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_ffn_forward_schedule", rc)


def mixlora_ffn_backward_schedule(dims: Dims, schedule: int, weights: Weights, x, dy,
                                  d_aux: float, workspace, workspace_bytes: int, dx,
                                  grads: Grads, stream=None) -> None:
    rc = load().mixlora_ffn_backward_schedule(C.byref(dims), int(schedule), C.byref(weights),
                                              _ptr(x), _ptr(dy), float(d_aux), _ptr(workspace),
                                              workspace_bytes, _ptr(dx), C.byref(grads),
                                              _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_ffn_backward_schedule", rc)


def make_dora(tensors: Dict[str, object], shared: bool = False) -> Dora:
    """shared: one magnitude vector per projection ([d_ff], [d_ff], [d]) used by every expert."""
    d = Dora()
    for n in DORA_FIELDS:
        setattr(d, n, _ptr(tensors.get(n)))
    d.shared = int(shared)
    return d


def make_dora_grads(tensors: Dict[str, object]) -> DoraGrads:
    g = DoraGrads()
    for n in DORA_GRAD_FIELDS:
        setattr(g, n, _ptr(tensors.get(n)))
    return g


def mixlora_dora_workspace_bytes(dims: Dims, for_backward: bool) -> int:
    return int(load().mixlora_dora_workspace_bytes(C.byref(dims), int(bool(for_backward))))


def mixlora_dora_forward(dims: Dims, weights: Weights, dora: Dora, x, y, topk_idx, topk_w,
                         expert_counts, aux_loss, workspace, workspace_bytes: int,
                         stream=None) -> None:
    rc = load().mixlora_dora_forward(C.byref(dims), C.byref(weights), C.byref(dora), _ptr(x),
                                     _ptr(y), _ptr(topk_idx), _ptr(topk_w), _ptr(expert_counts),
                                     _ptr(aux_loss), _ptr(workspace), workspace_bytes,
                                     _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_dora_forward", rc)


def mixlora_dora_backward(dims: Dims, weights: Weights, dora: Dora, x, dy, d_aux: float, workspace,
                          workspace_bytes: int, dx, grads: Grads, dora_grads: DoraGrads,
                          stream=None) -> None:
    rc = load().mixlora_dora_backward(C.byref(dims), C.byref(weights), C.byref(dora), _ptr(x),
                                      _ptr(dy), float(d_aux), _ptr(workspace), workspace_bytes,
                                      _ptr(dx), C.byref(grads), C.byref(dora_grads),
                                      _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_dora_backward", rc)


def make_multi(M: int, token_model, d_aux=None) -> Multi:
    """token_model: device int32 tensor [T] (or raw pointer); d_aux: M host floats or None."""
    m = Multi()
    m.M = M
    m.token_model = _ptr(token_model)
    if d_aux is not None:
        arr = (C.c_float * M)(*[float(v) for v in d_aux])
        m._keep = arr                       # keeps the host array alive with the struct
        m.d_aux = C.cast(arr, C.POINTER(C.c_float))
    return m


def mixlora_multi_workspace_bytes(dims: Dims, M: int, for_backward: bool) -> int:
    return int(load().mixlora_multi_workspace_bytes(C.byref(dims), M, int(bool(for_backward))))


def mixlora_multi_forward(dims: Dims, multi: Multi, weights: Weights, x, y, topk_idx, topk_w,
                          expert_counts, aux_loss, workspace, workspace_bytes: int,
                          stream=None) -> None:
    rc = load().mixlora_multi_forward(C.byref(dims), C.byref(multi), C.byref(weights), _ptr(x),
                                      _ptr(y), _ptr(topk_idx), _ptr(topk_w), _ptr(expert_counts),
                                      _ptr(aux_loss), _ptr(workspace), workspace_bytes,
                                      _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_multi_forward", rc)


def mixlora_multi_backward(dims: Dims, multi: Multi, weights: Weights, x, dy, workspace,
                           workspace_bytes: int, dx, grads: Grads, stream=None) -> None:
    rc = load().mixlora_multi_backward(C.byref(dims), C.byref(multi), C.byref(weights), _ptr(x),
                                       _ptr(dy), _ptr(workspace), workspace_bytes, _ptr(dx),
                                       C.byref(grads), _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_multi_backward", rc)


def mixlora_aux_loss(probs, topk_idx, T: int, N: int, k: int, coeff: float, mode: int, loss,
                     F=None, P=None, dprobs=None, stream=None) -> None:
    rc = load().mixlora_aux_loss(_ptr(probs), _ptr(topk_idx), T, N, k, float(coeff), mode,
                                 _ptr(loss), _ptr(F), _ptr(P), _ptr(dprobs), _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_aux_loss", rc)


def mixlora_transpose(src, dst, rows: int, cols: int, dtype: int, stream=None) -> None:
    rc = load().mixlora_transpose(_ptr(src), _ptr(dst), rows, cols, dtype, _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_transpose", rc)


def mixlora_version() -> int:
    return int(load().mixlora_version())


def mixlora_lora_linear_workspace_bytes(dims: LinearDims, for_backward: bool) -> int:
    return int(load().mixlora_lora_linear_workspace_bytes(C.byref(dims), int(bool(for_backward))))


def mixlora_lora_linear_forward(dims: LinearDims, W, A, B_, x, y, workspace, workspace_bytes: int,
                                stream=None) -> None:
    rc = load().mixlora_lora_linear_forward(C.byref(dims), _ptr(W), _ptr(A), _ptr(B_), _ptr(x),
                                            _ptr(y), _ptr(workspace), workspace_bytes,
                                            _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_lora_linear_forward", rc)


def mixlora_lora_linear_backward(dims: LinearDims, W, W_T, A, B_, x, dy, workspace,
                                 workspace_bytes: int, dx, dA, dB, stream=None) -> None:
    rc = load().mixlora_lora_linear_backward(C.byref(dims), _ptr(W), _ptr(W_T), _ptr(A), _ptr(B_),
                                             _ptr(x), _ptr(dy), _ptr(workspace), workspace_bytes,
                                             _ptr(dx), _ptr(dA), _ptr(dB), _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_lora_linear_backward", rc)


def mixlora_adamw_step(h: AdamW, n: int, param, grad, m, v, lowp=None, lowp_dtype: int = BF16,
                       stream=None) -> None:
    rc = load().mixlora_adamw_step(C.byref(h), n, _ptr(param), _ptr(grad), _ptr(m), _ptr(v),
                                   _ptr(lowp), lowp_dtype, _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_adamw_step", rc)


def mixlora_mfma_probe(sink, sink_bytes: int, waves_per_simd: int, iters: int, stream=None) -> float:
    """TFLOP/s of a register-only bf16 MFMA loop on pseudo-random operands (waits for the GPU)."""
    v = C.c_double()
    rc = load().mixlora_mfma_probe(_ptr(sink), sink_bytes, waves_per_simd, iters, C.byref(v),
                                   _stream(stream))
    if rc != 0:
        raise MixLoraError("mixlora_mfma_probe", rc)
    return v.value


def mixlora_profile_begin(max_launches: int) -> None:
    rc = load().mixlora_profile_begin(max_launches)
    if rc != 0:
        raise MixLoraError("mixlora_profile_begin", rc)


def mixlora_profile_end():
    """Returns (summed kernel ms, launches, executed flops) of the large-tile GEMM kernel."""
    ms, n, fl = C.c_double(), C.c_int32(), C.c_double()
    rc = load().mixlora_profile_end(C.byref(ms), C.byref(n), C.byref(fl))
    if rc != 0:
        raise MixLoraError("mixlora_profile_end", rc)
    return ms.value, n.value, fl.value


PROFILE_KINDS = ("gemm", "fused_forward", "fused_backward", "combine", "gradient_sums", "routing",
                 "other")


def mixlora_profile_kind(kind: int):
    """After mixlora_profile_end: (summed ms, launches, declared work) of one kind of launch
    (index into PROFILE_KINDS; work is FLOPs for kind 0, algorithmic bytes otherwise)."""
    ms, n, wk = C.c_double(), C.c_int32(), C.c_double()
    rc = load().mixlora_profile_kind(int(kind), C.byref(ms), C.byref(n), C.byref(wk))
    if rc != 0:
        raise MixLoraError("mixlora_profile_kind", rc)
    return ms.value, n.value, wk.value
