"""Seeded synthetic inputs for the Keyformer hot path.

This module only makes INPUTS: random Q/K/V tensors shaped like the paper's
GPT-J / Cerebras-GPT / MPT attention layers (Sec. 4: the three model families;
Sec. 4.2: the paper's own performance runs also used synthetic padded prompts),
the per-sequence noise seeds and the per-head ALiBi slopes.  It holds none of
the method's arithmetic and is imported by both the GPU tests/bench and the
oracle-side tests; the GPU library and the oracle do not import each other.

They stand in for the paper's datasets (CNN/DailyMail, GovReport, SODA), which
are not used anywhere in this repository.

Recipe: every element i.i.d. N(0,1) from a torch generator seeded per (base
seed, stream, layer), rounded to the workload's dtype.  "Heavy hitter" tokens:
round(outlier_frac*n) prompt key rows per unit, chosen by a seeded permutation,
are multiplied by outlier_scale; each generated key is scaled with probability
outlier_frac.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch

BASE_SEED = 20240309


@dataclass(frozen=True)
class Workload:
    name: str
    L: int
    B: int
    H: int
    d: int
    dtype: str  # "f32" | "bf16" | "f16"
    n: int      # prompt length
    k: int      # KV budget
    w: int      # recent window
    T: int      # decode steps
    tau_init: float = 1.0
    tau_end: float = 2.0
    outlier_frac: float = 0.0
    outlier_scale: float = 4.0
    alibi: bool = False
    H_full: int = 0      # head count the ALiBi slopes are derived for (0 = H)
    base_seed: int = BASE_SEED

    @property
    def units(self) -> int:
        return self.L * self.B * self.H

    @property
    def torch_dtype(self):
        return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[self.dtype]

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def scale(self) -> float:
        return float(np.float32(1.0) / np.sqrt(np.float32(self.d)))

    def slice(self, L=None, B=None, H=None, T=None, n=None, k=None, w=None, name=None):
        """Same per-unit shape, fewer units / steps (a parity slice)."""
        return replace(self, L=L or self.L, B=B or self.B, H=H or self.H, T=T or self.T,
                       n=n or self.n, k=k or self.k, w=self.w if w is None else w,
                       H_full=self.H_full or self.H,
                       name=name or (self.name + "-slice"))


CONFIGS = {
    "tiny": Workload("tiny", L=1, B=1, H=2, d=64, dtype="f32", n=128, k=64, w=16, T=32),
    "gptj": Workload("gptj", L=28, B=1, H=16, d=256, dtype="bf16", n=2048, k=1024, w=205, T=512,
                     outlier_frac=0.01),
    "mpt": Workload("mpt", L=32, B=8, H=32, d=128, dtype="bf16", n=4096, k=2048, w=410, T=1024,
                    alibi=True),
    "long": Workload("long", L=32, B=1, H=32, d=128, dtype="bf16", n=32768, k=9830, w=1966, T=2048,
                     outlier_frac=0.005),
    "batched": Workload("batched", L=32, B=64, H=32, d=128, dtype="bf16", n=2048, k=1024, w=205,
                        T=1024),
}


def staging_layers(wl: Workload, budget_bytes: float = 12e9) -> int:
    """Layers of the prompt (Q, K and V of n tokens each) staged per prompt-scoring call: as many as fit
    the byte budget, so that the n-token prompts of all layers never have to be resident at once."""
    layer_bytes = 3 * wl.B * wl.H * wl.n * wl.d * wl.elem_bytes
    return max(1, min(wl.L, int(budget_bytes // layer_bytes)))


def alibi_slopes(wl: Workload):
    """Per-head slopes 2^(-8h/H), h = 1..H (first wl.H of them), or None."""
    if not wl.alibi:
        return None
    Hf = wl.H_full or wl.H
    h = np.arange(1, Hf + 1, dtype=np.float64)
    return (2.0 ** (-8.0 * h / Hf)).astype(np.float32)[: wl.H].copy()


def noise_seeds(wl: Workload) -> np.ndarray:
    """One 64-bit noise seed per sequence: base ^ b."""
    return (np.uint64(wl.base_seed) ^ np.arange(wl.B, dtype=np.uint64)).astype(np.uint64)


def _gen(wl: Workload, stream: int, layer: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((wl.base_seed * 1000003 + stream * 7919 + layer) & 0x7FFFFFFFFFFFFFFF)
    return g


def prompt_layer(wl: Workload, layer: int, device="cpu"):
    """Q, K, V of one layer's prompt: each [B,H,n,d] in the workload dtype."""
    g = _gen(wl, 1, layer, device)
    shp = (wl.B, wl.H, wl.n, wl.d)
    Q = torch.randn(shp, generator=g, device=device, dtype=torch.float32)
    K = torch.randn(shp, generator=g, device=device, dtype=torch.float32)
    V = torch.randn(shp, generator=g, device=device, dtype=torch.float32)
    n_out = int(round(wl.outlier_frac * wl.n))
    if n_out > 0:
        r = torch.rand((wl.B, wl.H, wl.n), generator=g, device=device)
        idx = torch.argsort(r, dim=-1)[..., :n_out]  # a seeded permutation's head
        mult = torch.ones((wl.B, wl.H, wl.n), device=device)
        mult.scatter_(-1, idx, wl.outlier_scale)
        K = K * mult[..., None]
    dt = wl.torch_dtype
    return Q.to(dt), K.to(dt), V.to(dt)


def decode_inputs(wl: Workload, t: int, device="cpu"):
    """q, k_new, v_new of decode step t (1-based): each [L,B,H,d]."""
    g = _gen(wl, 2, t, device)
    shp = (wl.L, wl.B, wl.H, wl.d)
    q = torch.randn(shp, generator=g, device=device, dtype=torch.float32)
    k = torch.randn(shp, generator=g, device=device, dtype=torch.float32)
    v = torch.randn(shp, generator=g, device=device, dtype=torch.float32)
    if wl.outlier_frac > 0:
        r = torch.rand(shp[:3], generator=g, device=device)
        k = k * torch.where(r < wl.outlier_frac, wl.outlier_scale, 1.0)[..., None]
    dt = wl.torch_dtype
    return q.to(dt), k.to(dt), v.to(dt)


def to_oracle(t: torch.Tensor) -> np.ndarray:
    """Host numpy view the oracle reads: float32 as is, bf16 as uint16 bits."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def from_oracle(a: np.ndarray) -> torch.Tensor:
    """Inverse of to_oracle (uint16 -> bf16 tensor)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
    return torch.from_numpy(a.copy())


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    """Exact numeric value of oracle-format data, for test-side arithmetic."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)
