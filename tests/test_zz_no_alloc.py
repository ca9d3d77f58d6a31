"""The forward entry point that allocates nothing (its workspace is a static device array inside
the library) against the ordinary forward entry point, through the C ABI: same kernels, so every
output must be bit-identical.  Two calls in a row share the array; the second is a smaller input,
so whatever the first call left behind must not leak into it."""
import numpy as np
import pytest
import torch

from paper_2404_15159_amd import binding as B
from paper_2404_15159_amd import synth
from paper_2404_15159_amd.runner import MixLoraFFN

pytestmark = pytest.mark.gpu

BASE = synth.CONFIGS["llama2_7b"]


def _static_forward(m):
    """Run mixlora_ffn_forward_static on the runner's inputs; returns fresh output tensors."""
    dev = m.t["x"].device
    cfg = m.cfg
    y = torch.full_like(m.y, float("nan"))
    idx = torch.full((cfg.T, cfg.k), -1, dtype=torch.int32, device=dev)
    w = torch.full((cfg.T, cfg.k), float("nan"), dtype=torch.float32, device=dev)
    counts = torch.full((cfg.N,), -1, dtype=torch.int32, device=dev)
    aux = torch.full((1,), float("nan"), dtype=torch.float32, device=dev)
    B.mixlora_ffn_forward_static(m.dims, m.weights, m.t["x"], y, idx, w, counts, aux)
    torch.cuda.synchronize()
    return dict(y=y.float().cpu().numpy(), topk_idx=idx.cpu().numpy(), topk_w=w.cpu().numpy(),
                counts=counts.cpu().numpy(), aux_loss=float(aux.item()))


def test_static_forward_matches_forward_twice():
    shapes = [dict(T=128, d=512, d_ff=1408, N=8, k=2, r=16),      # K-split down projection
              dict(T=37, d=256, d_ff=520, N=4, k=2, r=8, alpha=16.0)]   # smaller, ragged
    for i, over in enumerate(shapes):
        cfg = synth.scaled(BASE, name=f"static{i}", **over)
        print(f"case {cfg.name}: {over}", flush=True)
        host = synth.make_inputs(cfg)
        m = MixLoraFFN(cfg, host, with_backward=False)
        assert m.ws_bytes <= B.STATIC_SCRATCH_BYTES
        m.forward()
        ref = m.results()
        got = _static_forward(m)
        for n in ("y", "topk_idx", "topk_w", "counts"):
            assert np.array_equal(np.asarray(ref[n]), got[n]), (cfg.name, n)
        assert ref["aux_loss"] == got["aux_loss"]


def test_static_forward_rejects_large_problems():
    cfg = synth.scaled(BASE, name="static_big", T=2048, d=1024, d_ff=4096)
    dims = B.make_dims(cfg.T, cfg.d, cfg.d_ff, cfg.N, cfg.k, cfg.r, cfg.lora_scale)
    assert B.mixlora_workspace_bytes(dims, False) > B.STATIC_SCRATCH_BYTES
    fake = 0x10000
    w = B.make_weights({n: fake for n in B.WEIGHT_FIELDS[:10]})
    with pytest.raises(B.MixLoraError) as ei:
        B.mixlora_ffn_forward_static(dims, w, fake, fake, fake, fake, fake, fake, stream=0)
    assert ei.value.code == -7
