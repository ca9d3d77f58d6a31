"""Device-side plumbing around the binding: owns the tensors of one MixLoRA FFN problem.

No arithmetic of the method happens here: tensors are allocated with PyTorch, pointers are
handed to the C ABI, and results are read back.  Used by the GPU tests, the smoke check and
bench.py.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as B
from . import synth


def _tdtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


class MixLoraFFN:
    """One problem instance on cuda:0: weights, workspace and output buffers."""

    def __init__(self, cfg: synth.Config, host: Dict[str, np.ndarray], aux_mode: int = B.AUX_TOP1,
                 pretransposed: bool = True, with_backward: bool = True, device: str = "cuda:0",
                 token_model: Optional[np.ndarray] = None, d_aux=None,
                 schedule: int = B.SCHEDULE_LINEAR_DOWN,
                 magnitudes: Optional[Dict[str, np.ndarray]] = None):
        """With cfg.M > 1 (several adapters on one frozen base) token_model [T] is required and
        the multi-adapter entry points are used; the banks then hold M*N experts.  A schedule
        other than SCHEDULE_LINEAR_DOWN goes through the *_schedule entry points (one adapter).
        magnitudes (m_gate, m_up [N,d_ff], m_down [N,d], float32) selects the weight-decomposed
        expert variant and its entry points."""
        B.load()
        self.cfg = cfg
        self.schedule = int(schedule)
        if self.schedule != B.SCHEDULE_LINEAR_DOWN and cfg.M > 1:
            raise ValueError("the paper's schedules are built for one adapter")
        self.dora = None
        if magnitudes is not None and (cfg.M > 1 or self.schedule != B.SCHEDULE_LINEAR_DOWN):
            raise ValueError("weight-decomposed experts: one adapter, default schedule argument")
        self.M = cfg.M
        if (cfg.M > 1) != (token_model is not None):
            raise ValueError("token_model goes with cfg.M > 1")
        self.dev = torch.device(device)
        self.with_backward = with_backward
        td = _tdtype(cfg.dtype)
        self.dims = B.make_dims(cfg.T, cfg.d, cfg.d_ff, cfg.N, cfg.k, cfg.r, cfg.lora_scale,
                                cfg.aux_coeff, aux_mode, B.BF16 if cfg.dtype == "bf16" else B.F32)
        self.t: Dict[str, torch.Tensor] = {}
        for n in synth.WEIGHT_NAMES + ("x",) + (("dy",) if with_backward and "dy" in host else ()):
            self.t[n] = torch.from_numpy(np.ascontiguousarray(host[n])).to(self.dev).to(td).contiguous()
        T, d, f, N, k, r = cfg.T, cfg.d, cfg.d_ff, cfg.N * cfg.M, cfg.k, cfg.r
        self.multi = None
        if cfg.M > 1:
            self.token_model = torch.from_numpy(np.ascontiguousarray(token_model, dtype=np.int32)).to(self.dev)
            self.multi = B.make_multi(cfg.M, self.token_model, d_aux)
        if with_backward and pretransposed:
            for n, (rows, cols) in (("W_gate", (f, d)), ("W_up", (f, d)), ("W_down", (d, f))):
                out = torch.empty((cols, rows), dtype=td, device=self.dev)
                B.mixlora_transpose(self.t[n], out, rows, cols, self.dims.dtype)
                self.t[n + "_T"] = out
        self.weights = B.make_weights(self.t)
        if magnitudes is not None:
            self.mag = {n: torch.from_numpy(np.ascontiguousarray(magnitudes[n], dtype=np.float32)).to(self.dev)
                        for n in B.DORA_FIELDS}
            # 1-D magnitude vectors: one per projection, shared by the experts
            self.dora = B.make_dora(self.mag, shared=self.mag["m_gate"].dim() == 1)
            self.ws_bytes = B.mixlora_dora_workspace_bytes(self.dims, with_backward)
        elif self.schedule != B.SCHEDULE_LINEAR_DOWN:
            self.ws_bytes = B.mixlora_schedule_workspace_bytes(self.dims, self.schedule, with_backward)
        else:
            self.ws_bytes = (B.mixlora_multi_workspace_bytes(self.dims, cfg.M, with_backward)
                             if self.multi else B.mixlora_workspace_bytes(self.dims, with_backward))
        if self.ws_bytes == 0:
            raise ValueError("dims rejected by mixlora_workspace_bytes")
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        self.y = torch.empty((T, d), dtype=td, device=self.dev)
        self.topk_idx = torch.empty((T, k), dtype=torch.int32, device=self.dev)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, device=self.dev)
        self.counts = torch.empty((N,), dtype=torch.int32, device=self.dev)
        self.aux = torch.empty((cfg.M,), dtype=torch.float32, device=self.dev)
        if with_backward:
            self.dx = torch.empty((T, d), dtype=td, device=self.dev)
            shapes = dict(dA_gate=(N, r, d), dB_gate=(N, f, r), dA_up=(N, r, d), dB_up=(N, f, r),
                          dA_down=(N, r, f), dB_down=(N, d, r), dW_router=(N, d))
            self.g = {n: torch.empty(s, dtype=torch.float32, device=self.dev)
                      for n, s in shapes.items()}
            self.grads = B.make_grads(self.g)
            if self.dora is not None:
                self.gm = {"d" + n: torch.empty_like(self.mag[n]) for n in B.DORA_FIELDS}
                self.dora_grads = B.make_dora_grads(self.gm)

    def forward(self, x: Optional[torch.Tensor] = None, stream=None) -> None:
        if self.multi:
            B.mixlora_multi_forward(self.dims, self.multi, self.weights,
                                    self.t["x"] if x is None else x, self.y, self.topk_idx,
                                    self.topk_w, self.counts, self.aux, self.workspace,
                                    self.ws_bytes, stream)
            return
        if self.dora is not None:
            B.mixlora_dora_forward(self.dims, self.weights, self.dora,
                                   self.t["x"] if x is None else x, self.y, self.topk_idx,
                                   self.topk_w, self.counts, self.aux, self.workspace,
                                   self.ws_bytes, stream)
            return
        if self.schedule != B.SCHEDULE_LINEAR_DOWN:
            B.mixlora_ffn_forward_schedule(self.dims, self.schedule, self.weights,
                                           self.t["x"] if x is None else x, self.y, self.topk_idx,
                                           self.topk_w, self.counts, self.aux, self.workspace,
                                           self.ws_bytes, stream)
            return
        B.mixlora_ffn_forward(self.dims, self.weights, self.t["x"] if x is None else x, self.y,
                              self.topk_idx, self.topk_w, self.counts, self.aux, self.workspace,
                              self.ws_bytes, stream)

    def backward(self, dy: Optional[torch.Tensor] = None, d_aux: float = 1.0, stream=None) -> None:
        if self.multi:   # per-adapter upstream gradients were given at construction
            B.mixlora_multi_backward(self.dims, self.multi, self.weights, self.t["x"],
                                     self.t["dy"] if dy is None else dy, self.workspace,
                                     self.ws_bytes, self.dx, self.grads, stream)
            return
        if self.dora is not None:
            B.mixlora_dora_backward(self.dims, self.weights, self.dora, self.t["x"],
                                    self.t["dy"] if dy is None else dy, d_aux, self.workspace,
                                    self.ws_bytes, self.dx, self.grads, self.dora_grads, stream)
            return
        if self.schedule != B.SCHEDULE_LINEAR_DOWN:
            B.mixlora_ffn_backward_schedule(self.dims, self.schedule, self.weights, self.t["x"],
                                            self.t["dy"] if dy is None else dy, d_aux,
                                            self.workspace, self.ws_bytes, self.dx, self.grads, stream)
            return
        B.mixlora_ffn_backward(self.dims, self.weights, self.t["x"],
                               self.t["dy"] if dy is None else dy, d_aux, self.workspace,
                               self.ws_bytes, self.dx, self.grads, stream)

    def results(self) -> Dict[str, np.ndarray]:
        torch.cuda.synchronize()
        out = dict(y=self.y.float().cpu().numpy(), topk_idx=self.topk_idx.cpu().numpy(),
                   topk_w=self.topk_w.cpu().numpy(), counts=self.counts.cpu().numpy(),
                   aux_loss=(self.aux.cpu().numpy() if self.multi else float(self.aux.cpu().item())))
        if self.with_backward:
            out["dx"] = self.dx.float().cpu().numpy()
            for n, v in self.g.items():
                out[n] = v.cpu().numpy()
            if self.dora is not None:
                for n, v in self.gm.items():
                    out[n] = v.cpu().numpy()
        return out


class LoraLinear:
    """One plain LoRA linear problem (the attention-projection form) on cuda:0."""

    def __init__(self, T: int, d_in: int, d_out: int, r: int, lora_scale: float, dtype: str,
                 host: Dict[str, np.ndarray], pretransposed: bool = True, device: str = "cuda:0"):
        B.load()
        self.dev = torch.device(device)
        td = _tdtype(dtype)
        code = B.BF16 if dtype == "bf16" else B.F32
        self.dims = B.LinearDims(T, d_in, d_out, r, lora_scale, code)
        self.t = {n: torch.from_numpy(np.ascontiguousarray(host[n])).to(self.dev).to(td).contiguous()
                  for n in ("x", "W", "A", "B", "dy")}
        self.W_T = None
        if pretransposed:
            self.W_T = torch.empty((d_in, d_out), dtype=td, device=self.dev)
            B.mixlora_transpose(self.t["W"], self.W_T, d_out, d_in, code)
        self.ws_bytes = B.mixlora_lora_linear_workspace_bytes(self.dims, True)
        if self.ws_bytes == 0:
            raise ValueError("dims rejected by mixlora_lora_linear_workspace_bytes")
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        self.y = torch.empty((T, d_out), dtype=td, device=self.dev)
        self.dx = torch.empty((T, d_in), dtype=td, device=self.dev)
        self.dA = torch.empty((r, d_in), dtype=torch.float32, device=self.dev)
        self.dB = torch.empty((d_out, r), dtype=torch.float32, device=self.dev)

    def forward(self, stream=None) -> None:
        B.mixlora_lora_linear_forward(self.dims, self.t["W"], self.t["A"], self.t["B"], self.t["x"],
                                      self.y, self.workspace, self.ws_bytes, stream)

    def backward(self, stream=None) -> None:
        B.mixlora_lora_linear_backward(self.dims, self.t["W"], self.W_T, self.t["A"], self.t["B"],
                                       self.t["x"], self.t["dy"], self.workspace, self.ws_bytes,
                                       self.dx, self.dA, self.dB, stream)

    def results(self) -> Dict[str, np.ndarray]:
        torch.cuda.synchronize()
        return dict(y=self.y.float().cpu().numpy(), dx=self.dx.float().cpu().numpy(),
                    dA=self.dA.cpu().numpy(), dB=self.dB.cpu().numpy())
