"""Seeded synthetic inputs for the GSA forward path.

This module only draws random tensors of the right shape, dtype and value
distribution; it holds none of the method's arithmetic and is the one piece
shared by the GPU tests, the benchmark and the CPU checker.  The shapes follow
the paper's 1.7B model (Sec. 7.1: 16 query heads, 4 key-value heads, head
dimension 128) and its indexer defaults (Sec. 4.1: H^I = 4, d^I = 64).
"""
from dataclasses import dataclass, replace
import math

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Lq: int
    Lk: int
    q_offset: int
    H: int
    H_kv: int
    d_h: int
    HI: int
    dI: int
    dtype: str            # "f32" or "bf16"
    k_base: int
    k_min: int
    k_max: int
    k_fixed: int = 0      # > 0: controller off
    gate_std: float = 1.0
    heavy_frac: float = 0.0   # fraction of tokens whose indexer key is scaled
    heavy_scale: float = 1.0
    seed: int = 0
    indexer_act: str = "sigmoid"   # "relu": the ungated indexer of the comparison variants

    @property
    def k_cap(self):
        return self.k_fixed if self.k_fixed > 0 else self.k_max

    def with_(self, **kw):
        return replace(self, **kw)


def _kbase(k_min, k_max):
    return int(math.floor(math.sqrt(k_min * k_max)))


# The five benchmark configurations (tiny fp32; 1.7B-shaped layer at 8K; 32K skewed; 128K prefill; 128K decode).
C1_FIXED = Workload("C1-fixed", 1, 512, 512, 0, 4, 4, 64, 4, 32, "f32", 64, 32, 128, k_fixed=64, seed=0)
C1 = Workload("C1-adaptive", 1, 512, 512, 0, 4, 4, 64, 4, 32, "f32", _kbase(32, 128), 32, 128, seed=0)
C2 = Workload("C2-8k", 1, 8192, 8192, 0, 16, 4, 128, 4, 64, "bf16", _kbase(512, 2048), 512, 2048, seed=1002)
C3 = Workload("C3-32k-skewed", 2, 32768, 32768, 0, 16, 4, 128, 4, 64, "bf16", _kbase(1024, 2048), 1024, 2048,
              heavy_frac=0.05, heavy_scale=4.0, seed=1003)
C4 = Workload("C4-128k-prefill", 1, 131072, 131072, 0, 16, 4, 128, 4, 64, "bf16", _kbase(1024, 4096), 1024, 4096,
              gate_std=2.0, seed=1004)
C5 = Workload("C5-128k-decode", 64, 1, 131072, 131071, 16, 4, 128, 4, 64, "bf16", _kbase(1024, 2048), 1024, 2048,
              seed=1005)
CONFIGS = {w.name: w for w in (C1_FIXED, C1, C2, C3, C4, C5)}

_TENSOR_ORDER = ("Q", "K", "V", "g1", "g2", "qI", "kI", "w", "heavy")


def torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(device, seed, name):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 131 + _TENSOR_ORDER.index(name))
    return g


def _normal(shape, std, dtype, device, gen, chunk_elems=1 << 28):
    """N(0, std) drawn in fp32 and rounded to dtype, in chunks so that the fp32 staging stays small."""
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    n = flat.numel()
    for lo in range(0, n, chunk_elems):
        hi = min(n, lo + chunk_elems)
        x = torch.randn(hi - lo, dtype=torch.float32, device=device, generator=gen)
        if std != 1.0:
            x *= std
        flat[lo:hi] = x.to(dtype)
    return out


def make_inputs(wl, device="cpu", with_bias=False):
    """Draw every input tensor of the path for one workload.

    Returns a dict: Q [B,Lq,H,d_h], K/V/g2 [B,Lk,H_kv,d_h], g1 [B,Lq,H,d_h],
    qI [B,Lq,HI,dI], kI [B,Lk,dI] in the workload dtype; w [B,Lq,HI] fp32 in
    (0,1); bI [HI] fp32 or None.
    """
    dt = torch_dtype(wl.dtype)
    dev = torch.device(device)
    t = {}
    t["Q"] = _normal((wl.B, wl.Lq, wl.H, wl.d_h), 1.0, dt, dev, _gen(dev, wl.seed, "Q"))
    t["K"] = _normal((wl.B, wl.Lk, wl.H_kv, wl.d_h), 1.0, dt, dev, _gen(dev, wl.seed, "K"))
    t["V"] = _normal((wl.B, wl.Lk, wl.H_kv, wl.d_h), 1.0, dt, dev, _gen(dev, wl.seed, "V"))
    t["g1"] = _normal((wl.B, wl.Lq, wl.H, wl.d_h), wl.gate_std, dt, dev, _gen(dev, wl.seed, "g1"))
    t["g2"] = _normal((wl.B, wl.Lk, wl.H_kv, wl.d_h), wl.gate_std, dt, dev, _gen(dev, wl.seed, "g2"))
    t["qI"] = _normal((wl.B, wl.Lq, wl.HI, wl.dI), 1.0, dt, dev, _gen(dev, wl.seed, "qI"))
    kI = torch.randn((wl.B, wl.Lk, wl.dI), dtype=torch.float32, device=dev, generator=_gen(dev, wl.seed, "kI"))
    if wl.heavy_frac > 0.0:
        # a seeded subset of exactly floor(frac * Lk) token positions per sequence gets its whole key scaled
        n_heavy = int(math.floor(wl.heavy_frac * wl.Lk))
        gh = _gen(dev, wl.seed, "heavy")
        for b in range(wl.B):
            perm = torch.randperm(wl.Lk, device=dev, generator=gh)[:n_heavy]
            kI[b, perm] *= wl.heavy_scale
    t["kI"] = kI.to(dt)
    w = torch.rand((wl.B, wl.Lq, wl.HI), dtype=torch.float32, device=dev, generator=_gen(dev, wl.seed, "w"))
    t["w"] = w.clamp_(2.0 ** -24, 1.0 - 2.0 ** -24)
    if with_bias:
        t["bI"] = torch.linspace(-1.0, 1.0, wl.HI, dtype=torch.float32, device=dev)
    else:
        t["bI"] = None
    return t
