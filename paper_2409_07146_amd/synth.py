"""Seeded synthetic inputs shaped like the paper's GSA workloads.

This module only draws random tensors; it holds none of the operator's
arithmetic and is the one piece shared by the GPU path's tests/benchmarks and
by the CPU oracle's tests.  The paper trains language models whose activations
are not available here, so tensors with the paper's shapes (m = 64 slots,
4 heads, model widths 2048 / 2560, 2K-16K contexts; Section 4 and the
experimental-setup appendix) stand in for them:

    q, k, v ~ N(0,1)/sqrt(d_k), rounded once to the I/O dtype
    g = logsigmoid(N(0,1)) / tau with tau = 8   (the layer's gate
        alpha = sigmoid(W x)^(1/tau), Section 3.3, in log space), fp32
    dO ~ N(0,1) rounded to the I/O dtype;  initial memories ~ N(0, std^2), fp32

Draw order from one CPU generator: q, k, v, gate logits, dO, K0, V0.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import torch


@dataclass(frozen=True)
class GsaConfig:
    name: str
    B: int
    T: int
    H: int
    d_k: int
    d_v: int
    m: int
    dtype: str = "bf16"            # "bf16" or "f32": dtype of q,k,v,o,dO,dq,dk,dv
    backward: bool = True
    cu_seqlens: Optional[Tuple[int, ...]] = None   # packed sequences (then B == 1)
    init_state_std: float = 0.0    # 0 => zero initial memories (the paper's default)
    seed: int = 0
    tau: float = 8.0

    @property
    def n_seqs(self) -> int:
        return self.B if self.cu_seqlens is None else len(self.cu_seqlens) - 1

    @property
    def tokens(self) -> int:
        return self.B * self.T


# The five workloads this repository is measured and checked on.
CONFIGS = {
    "tiny_f32": GsaConfig("tiny_f32", B=1, T=256, H=1, d_k=64, d_v=64, m=16, dtype="f32",
                          backward=False, seed=0),
    "fwd_d128": GsaConfig("fwd_d128", B=8, T=2048, H=4, d_k=128, d_v=128, m=64, backward=False,
                          seed=1),
    "layer_1p3b": GsaConfig("layer_1p3b", B=8, T=2048, H=4, d_k=512, d_v=512, m=64, seed=2),
    "layer_2p7b": GsaConfig("layer_2p7b", B=8, T=2048, H=4, d_k=640, d_v=640, m=64, seed=3),
    "packed_16k": GsaConfig("packed_16k", B=1, T=16384, H=4, d_k=512, d_v=512, m=64,
                            cu_seqlens=(0, 8192, 12288, 14336, 16384), seed=4),
}

# Shape variants beyond the five workloads (the ablation table of Section 4 varies the number of slots;
# the experimental-setup appendix gives the 2.7B model 5 heads of 512).
VARIANTS = {
    "layer_1p3b_m32": GsaConfig("layer_1p3b_m32", B=8, T=2048, H=4, d_k=512, d_v=512, m=32, seed=12),
    "layer_1p3b_m128": GsaConfig("layer_1p3b_m128", B=8, T=2048, H=4, d_k=512, d_v=512, m=128, seed=13),
    "layer_2p7b_h5": GsaConfig("layer_2p7b_h5", B=8, T=2048, H=5, d_k=512, d_v=512, m=64, seed=14),
}

# Decode workload: 512 steps at batch 64 from random memories ~ N(0, 0.1^2).
DECODE = dict(B=64, H=4, d_k=512, d_v=512, m=64, steps=512, state_std=0.1, seed=5)


def torch_dtype(name: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "f32": torch.float32}[name]


def make_inputs(cfg: GsaConfig, seed: Optional[int] = None):
    """Returns a dict of CPU tensors: q,k,v,dO in cfg.dtype; g,K0,V0 fp32
    (K0,V0 are None when cfg.init_state_std == 0); cu_seqlens int32 or None."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(cfg.seed if seed is None else seed)
    dt = torch_dtype(cfg.dtype)
    B, T, H = cfg.B, cfg.T, cfg.H
    inv = cfg.d_k ** -0.5

    def draw(*shape):
        return torch.randn(*shape, generator=gen, dtype=torch.float32)

    q = (draw(B, T, H, cfg.d_k) * inv).to(dt)
    k = (draw(B, T, H, cfg.d_k) * inv).to(dt)
    v = (draw(B, T, H, cfg.d_v) * inv).to(dt)
    g = torch.nn.functional.logsigmoid(draw(B, T, H, cfg.m)) / cfg.tau
    dO = draw(B, T, H, cfg.d_v).to(dt)
    K0 = V0 = None
    if cfg.init_state_std > 0:
        K0 = draw(cfg.n_seqs, H, cfg.m, cfg.d_k) * cfg.init_state_std
        V0 = draw(cfg.n_seqs, H, cfg.m, cfg.d_v) * cfg.init_state_std
    cu = None if cfg.cu_seqlens is None else torch.tensor(cfg.cu_seqlens, dtype=torch.int32)
    return dict(q=q, k=k, v=v, g=g.contiguous(), dO=dO, K0=K0, V0=V0, cu_seqlens=cu)


def make_decode_inputs(B, H, d_k, d_v, m, steps, state_std=0.1, seed=5, dtype="bf16", tau=8.0):
    """Random memories and a stream of per-step q,k,v,g.
    Returns K,V [B,H,m,d] fp32 and q,k [steps,B,H,d_k], v [steps,B,H,d_v] (dtype),
    g [steps,B,H,m] fp32."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    dt = torch_dtype(dtype)
    inv = d_k ** -0.5
    K = torch.randn(B, H, m, d_k, generator=gen) * state_std
    V = torch.randn(B, H, m, d_v, generator=gen) * state_std
    q = (torch.randn(steps, B, H, d_k, generator=gen) * inv).to(dt)
    k = (torch.randn(steps, B, H, d_k, generator=gen) * inv).to(dt)
    v = (torch.randn(steps, B, H, d_v, generator=gen) * inv).to(dt)
    g = torch.nn.functional.logsigmoid(torch.randn(steps, B, H, m, generator=gen)) / tau
    return dict(K=K, V=V, q=q, k=k, v=v, g=g.contiguous())
