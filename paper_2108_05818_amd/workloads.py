"""Seeded synthetic workloads: tensor lists and input values.

This module serves both the HIP path's callers and the tests' oracle.  It
holds shapes and random draws only -- none of the method's arithmetic (no
layout rule, no Adam, no overflow test).  The tensor lists stand in for the
paper's GPT-2-like models (Evaluation, Table "Model Config."): the paper's
checkpoints and data are not needed because the update is data-oblivious
apart from inf/nan.

Value recipe (sigma = standard deviation):
  param fp32  ~ N(0, 0.02)
  grad  fp16  = round_to_nearest_even_fp16( N(0, 1e-3) * loss_scale )
  momentum = variance = 0 at step 0
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

Mi = 1 << 20


def gpt_tensor_list(layers: int, hidden: int, vocab: int, seq: int) -> List[Tuple[str, int]]:
    """GPT-2 module order ("order of model initialization"): token and position
    embeddings, then per layer LayerNorm, fused QKV, attention projection,
    LayerNorm, MLP up (4h), MLP down; final LayerNorm.  Output head tied."""
    h = hidden
    out = [("wte", vocab * h), ("wpe", seq * h)]
    for l in range(layers):
        out += [
            (f"l{l}.ln1.w", h), (f"l{l}.ln1.b", h),
            (f"l{l}.qkv.w", 3 * h * h), (f"l{l}.qkv.b", 3 * h),
            (f"l{l}.proj.w", h * h), (f"l{l}.proj.b", h),
            (f"l{l}.ln2.w", h), (f"l{l}.ln2.b", h),
            (f"l{l}.fc.w", 4 * h * h), (f"l{l}.fc.b", 4 * h),
            (f"l{l}.fcproj.w", 4 * h * h), (f"l{l}.fcproj.b", h),
        ]
    out += [("lnf.w", h), ("lnf.b", h)]
    return out


def ragged_sizes(n: int = 5000, lo: int = 1, hi: int = 4 * Mi, seed: int = 3000) -> List[int]:
    """n tensor sizes, log-uniform in [lo, hi]."""
    rng = np.random.default_rng(seed)
    u = rng.uniform(np.log(lo), np.log(hi), size=n)
    s = np.floor(np.exp(u)).astype(np.int64)
    return [int(x) for x in np.clip(s, lo, hi)]


@dataclass
class Workload:
    name: str
    numel: List[int]
    chunk_elems: int
    loss_scale: float
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    adamw_mode: int = 0
    steps: int = 10
    seed: int = 0
    host_fraction: float = 0.0          # share of chunks whose fp32 states start in pinned host memory
    budget_jitter: float = 0.0          # +-fraction by which the HBM budget moves per step
    inject_prob: float = 0.0            # per-step probability of planting an inf/nan in one grad
    growth_interval: int = 2000
    names: Optional[List[str]] = field(default=None, repr=False)

    @property
    def n_elems(self) -> int:
        return int(sum(self.numel))


def _gpt(name, layers, hidden, vocab, seq, **kw) -> Workload:
    tl = gpt_tensor_list(layers, hidden, vocab, seq)
    return Workload(name=name, numel=[n for _, n in tl], names=[s for s, _ in tl], **kw)


def config1_tiny() -> Workload:
    return _gpt("tiny-gpt-L2-h64", 2, 64, 1000, 128, chunk_elems=65536, loss_scale=1024.0,
                steps=10, seed=1000)


def config2_gpt1b(layers: int = 20) -> Workload:
    return _gpt(f"gpt-1.1b-L{layers}-h2048", layers, 2048, 50257, 1024, chunk_elems=32 * Mi,
                loss_scale=65536.0, steps=20, seed=2000)


def config3_ragged(n: int = 5000, hi: int = 4 * Mi, chunk_elems: int = 16 * Mi) -> Workload:
    return Workload(name=f"ragged-{n}", numel=ragged_sizes(n, 1, hi, 3000), chunk_elems=chunk_elems,
                    loss_scale=65536.0, steps=200, seed=3000, inject_prob=0.01, growth_interval=50)


def config4_gpt12b(layers: int = 40) -> Workload:
    return _gpt(f"gpt-12.6b-L{layers}-h5120", layers, 5120, 50257, 1024, chunk_elems=64 * Mi,
                loss_scale=65536.0, steps=5, seed=4000, host_fraction=0.4)


def config5_gpt20b(layers: int = 44) -> Workload:
    return _gpt(f"gpt-20b-L{layers}-h6144", layers, 6144, 50257, 1024, chunk_elems=64 * Mi,
                loss_scale=65536.0, steps=10, seed=5000, host_fraction=0.7, budget_jitter=0.3)


# ------------------------------------------------------------------ numpy draws

def params_np(n: int, seed: int) -> np.ndarray:
    """fp32 params ~ N(0, 0.02)."""
    rng = np.random.default_rng([seed, 1])
    return (rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)).astype(np.float32)


def grads_f16_np(n: int, seed: int, loss_scale: float) -> np.ndarray:
    """Scaled fp16 grads as uint16 bit patterns."""
    rng = np.random.default_rng([seed, 2])
    g = rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3) * np.float32(loss_scale)
    return g.astype(np.float16).view(np.uint16)


def specials_f16() -> np.ndarray:
    """fp16 bit patterns that are inf or nan: +-inf, quiet and signalling nans."""
    return np.array([0x7C00, 0xFC00, 0x7E00, 0xFE00, 0x7D00, 0x7C01, 0xFFFF], dtype=np.uint16)


def budget_fraction(step: int, base: float, jitter: float, seed: int = 5000) -> float:
    """Share of chunks that may keep fp32 states in HBM at `step`: base*(1+jitter*u), u~U(-1,1)."""
    rng = np.random.default_rng(seed + step)
    u = rng.uniform(-1.0, 1.0)
    return float(min(1.0, max(0.0, base * (1.0 + jitter * u))))


# ------------------------------------------------------------------ torch draws (device side, large sizes)

def params_torch(n: int, seed: int, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed * 2 + 1)
    return torch.randn(n, generator=g, device=device, dtype=torch.float32).mul_(0.02)


def grads_f16_torch(n: int, seed: int, loss_scale: float, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed * 2 + 2)
    x = torch.randn(n, generator=g, device=device, dtype=torch.float32).mul_(1e-3 * loss_scale)
    return x.to(torch.float16)
