"""Seeded synthetic inputs for the MixLoRA FFN block.

This module holds no arithmetic of the method itself: it only draws random
tensors of the shapes, value distributions and routing structure of the
LLaMA-shaped fine-tuning workloads (hyper-parameter table of the appendix:
rank 16, alpha 32, 8 experts, top-2), and rounds them to the storage dtype.
Both the CPU oracle's tests and the HIP path's tests/bench consume the arrays
produced here; neither side's code is imported.

Random numbers come from a counter-based generator (splitmix64 of
``(seed, tensor, element)`` followed by Box-Muller) so the values do not
depend on the NumPy version or on the order in which tensors are requested.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np

SEED_BASE = 240415159

TENSOR_ORDER = (
    "x", "W_gate", "W_up", "W_down", "A_gate", "B_gate", "A_up", "B_up",
    "A_down", "B_down", "W_router", "dy", "aux",
)

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * _C1
    z = (z ^ (z >> np.uint64(27))) * _C2
    return z ^ (z >> np.uint64(31))


def _stream_key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix(np.array([np.uint64(seed) * _GOLDEN + np.uint64(stream + 1) * _C2],
                          dtype=np.uint64))
    return k[0]


def uniform01(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n doubles in the open interval (0, 1); element i depends only on (seed, stream, i)."""
    key = _stream_key(seed, stream)
    out = np.empty(n, dtype=np.float64)
    chunk = 1 << 22
    with np.errstate(over="ignore"):
        for lo in range(0, n, chunk):
            hi = min(n, lo + chunk)
            ctr = np.arange(lo + offset, hi + offset, dtype=np.uint64)
            bits = _mix(key + ctr * _GOLDEN)
            out[lo:hi] = ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / (1 << 53))
    return out


def normal(seed: int, stream: int, n: int) -> np.ndarray:
    """n standard normal doubles via Box-Muller on counters (2i, 2i+1)."""
    out = np.empty(n, dtype=np.float64)
    chunk = 1 << 22
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        u = uniform01(seed, stream, 2 * (hi - lo), offset=2 * lo)
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        out[lo:hi] = r * np.cos(2.0 * math.pi * u[1::2])
    return out


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array holding the nearest-even bfloat16 value of each element."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array of bf16-representable values -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    index: int            # position in the workload list; seed = SEED_BASE + index
    T: int
    d: int
    d_ff: int
    N: int
    k: int
    r: int
    alpha: float
    dtype: str            # "f32" or "bf16"
    b_std: float          # std of the LoRA B banks
    aux_coeff: float = 0.01
    backward: bool = True
    structure: str = "uniform"   # "uniform" | "skew0" | "clusters4"
    seq_len: int = 1024
    M: int = 1            # adapters sharing the frozen base; banks then hold M*N experts

    @property
    def lora_scale(self) -> float:
        return self.alpha / self.r

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index


CONFIGS = {
    "tiny_f32": Config("tiny_f32", 1, T=256, d=128, d_ff=344, N=8, k=2, r=8, alpha=16.0,
                       dtype="f32", b_std=0.02, seq_len=256),
    "llama2_7b_fwd": Config("llama2_7b_fwd", 2, T=4096, d=4096, d_ff=11008, N=8, k=2, r=16,
                            alpha=32.0, dtype="bf16", b_std=0.01, backward=False),
    "llama2_7b": Config("llama2_7b", 3, T=4096, d=4096, d_ff=11008, N=8, k=2, r=16,
                        alpha=32.0, dtype="bf16", b_std=0.01),
    "llama2_13b_skew": Config("llama2_13b_skew", 4, T=8192, d=5120, d_ff=13824, N=8, k=2, r=16,
                              alpha=32.0, dtype="bf16", b_std=0.01, structure="skew0"),
    "llama3_8b_clusters": Config("llama3_8b_clusters", 5, T=16384, d=4096, d_ff=14336, N=16, k=2,
                                 r=8, alpha=16.0, dtype="bf16", b_std=0.01,
                                 structure="clusters4"),
    # decode-shaped forward: 64 sequences, one new token each (weight-read-bound regime)
    "llama2_7b_decode": Config("llama2_7b_decode", 7, T=64, d=4096, d_ff=11008, N=8, k=2, r=16,
                               alpha=32.0, dtype="bf16", b_std=0.01, backward=False, seq_len=1),
    # two adapters trained together on one frozen base (the multi-adapter setting of the
    # paper's efficiency table): 4 sequences of 1024 tokens, alternating between the adapters
    "llama2_7b_multi2": Config("llama2_7b_multi2", 6, T=4096, d=4096, d_ff=11008, N=8, k=2, r=16,
                               alpha=32.0, dtype="bf16", b_std=0.01, M=2),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of cfg with some dimensions replaced (used for small parity cases)."""
    return dataclasses.replace(cfg, **kw)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    a = a.astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


def make_inputs(cfg: Config, only: Optional[tuple] = None) -> Dict[str, np.ndarray]:
    """Draw every tensor of one workload.

    Returns fp32 arrays whose values are exactly representable in cfg.dtype:
      x [T,d], W_gate/W_up [d_ff,d], W_down [d,d_ff], A_gate/A_up [N,r,d],
      B_gate/B_up [N,d_ff,r], A_down [N,r,d_ff], B_down [N,d,r], W_router [N,d],
      dy [T,d].  With cfg.M adapters the banks and the router hold M*N experts, adapter m's
      expert e at index m*N + e.
    Distributions: x, dy ~ N(0,1); frozen W ~ N(0,0.02^2); A ~ U(+-1/sqrt(fan_in));
    B ~ N(0,b_std^2) (non-zero so that every LoRA path is exercised);
    W_router ~ N(0,0.02^2).
    Structure:
      skew0     - last channel of x is the constant 1 and W_router[0,d-1] is raised by
                  1.5, i.e. expert 0's logit gets exactly +1.5 (skewed expert load);
      clusters4 - sequence s (seq_len tokens) belongs to cluster s mod 4 and its tokens
                  are shifted by 0.5 * (random sign vector of the cluster).
    """
    T, d, f, N, r = cfg.T, cfg.d, cfg.d_ff, cfg.N * cfg.M, cfg.r
    seed = cfg.seed
    sid = {n: i for i, n in enumerate(TENSOR_ORDER)}
    want = set(only) if only is not None else set(TENSOR_ORDER)
    out: Dict[str, np.ndarray] = {}

    def nrm(name, shape, std):
        n = int(np.prod(shape))
        return (normal(seed, sid[name], n) * std).reshape(shape)

    def uni(name, shape, bound):
        n = int(np.prod(shape))
        return ((uniform01(seed, sid[name], n) * 2.0 - 1.0) * bound).reshape(shape)

    if "x" in want:
        x = nrm("x", (T, d), 1.0)
        if cfg.structure == "skew0":
            x[:, d - 1] = 1.0
        elif cfg.structure == "clusters4":
            signs = np.where(uniform01(seed, sid["aux"], 4 * d) < 0.5, -1.0, 1.0).reshape(4, d)
            cluster = (np.arange(T) // cfg.seq_len) % 4
            x += 0.5 * signs[cluster]
        out["x"] = _store(x, cfg.dtype)
    for name, shape in (("W_gate", (f, d)), ("W_up", (f, d)), ("W_down", (d, f))):
        if name in want:
            out[name] = _store(nrm(name, shape, 0.02), cfg.dtype)
    for name, shape, fan_in in (("A_gate", (N, r, d), d), ("A_up", (N, r, d), d),
                                ("A_down", (N, r, f), f)):
        if name in want:
            out[name] = _store(uni(name, shape, 1.0 / math.sqrt(fan_in)), cfg.dtype)
    for name, shape in (("B_gate", (N, f, r)), ("B_up", (N, f, r)), ("B_down", (N, d, r))):
        if name in want:
            out[name] = _store(nrm(name, shape, cfg.b_std), cfg.dtype)
    if "W_router" in want:
        wr = nrm("W_router", (N, d), 0.02)
        if cfg.structure == "skew0":
            wr[0, d - 1] += 1.5
        out["W_router"] = _store(wr, cfg.dtype)
    if "dy" in want:
        out["dy"] = _store(nrm("dy", (T, d), 1.0), cfg.dtype)
    return out


WEIGHT_NAMES = ("W_gate", "W_up", "W_down", "A_gate", "B_gate", "A_up", "B_up",
                "A_down", "B_down", "W_router")


def make_magnitudes(cfg: Config) -> Dict[str, np.ndarray]:
    """Magnitude vectors of the weight-decomposed expert variant, float32: m_gate, m_up [N,d_ff],
    m_down [N,d].  Drawn as U(0.8, 1.2) times 0.02 * sqrt(fan_in), the expected row norm of a
    frozen matrix of the recipe above, so the factors magnitude / norm scatter around one."""
    N, d, f = cfg.N, cfg.d, cfg.d_ff
    out = {}
    for i, (name, shape, fan_in) in enumerate((("m_gate", (N, f), d), ("m_up", (N, f), d),
                                               ("m_down", (N, d), f))):
        u = uniform01(cfg.seed + 7919, i, int(np.prod(shape))).reshape(shape)
        out[name] = ((0.8 + 0.4 * u) * 0.02 * math.sqrt(fan_in)).astype(np.float32)
    return out


def token_model(cfg: Config, pattern: str = "round_robin") -> np.ndarray:
    """Adapter of every token, int32 [T].  Whole sequences (cfg.seq_len tokens) belong to one
    adapter, as in a batch that mixes the training sequences of several adapters.
      round_robin - sequence s goes to adapter s mod M;
      uneven      - adapter 0 gets every second sequence, the others share the rest in turn;
      skip_last   - round robin over the first M-1 adapters: the last adapter gets no token."""
    seq = np.arange(cfg.T) // cfg.seq_len
    M = cfg.M
    if pattern == "round_robin":
        m = seq % M
    elif pattern == "uneven":
        m = np.where(seq % 2 == 0, 0, 1 + (seq // 2) % max(M - 1, 1)) if M > 1 else seq * 0
    elif pattern == "skip_last":
        m = seq % max(M - 1, 1)
    else:
        raise ValueError(pattern)
    return m.astype(np.int32)


def split_adapters(cfg: Config, host: Dict[str, np.ndarray]):
    """The M per-adapter weight dicts (views) of a multi-adapter input set."""
    N = cfg.N
    out = []
    for m in range(cfg.M):
        Wm = {n: host[n] for n in ("W_gate", "W_up", "W_down")}
        for n in ("A_gate", "B_gate", "A_up", "B_up", "A_down", "B_down", "W_router"):
            Wm[n] = host[n][m * N:(m + 1) * N]
        out.append(Wm)
    return out


def make_linear_inputs(T: int, d_in: int, d_out: int, r: int, dtype: str, seed: int,
                       b_std: float = 0.01) -> Dict[str, np.ndarray]:
    """Tensors of one plain LoRA linear (an attention projection with its adapter): x [T,d_in],
    W [d_out,d_in] ~ N(0,0.02^2), A [r,d_in] ~ U(+-1/sqrt(d_in)), B [d_out,r] ~ N(0,b_std^2),
    dy [T,d_out]; same generator and rounding as make_inputs."""
    out = {}
    out["x"] = _store((normal(seed, 0, T * d_in)).reshape(T, d_in), dtype)
    out["W"] = _store((normal(seed, 1, d_out * d_in) * 0.02).reshape(d_out, d_in), dtype)
    out["A"] = _store(((uniform01(seed, 4, r * d_in) * 2.0 - 1.0) / math.sqrt(d_in)).reshape(r, d_in), dtype)
    out["B"] = _store((normal(seed, 5, d_out * r) * b_std).reshape(d_out, r), dtype)
    out["dy"] = _store((normal(seed, 11, T * d_out)).reshape(T, d_out), dtype)
    return out
