"""Seeded synthetic inputs for the Contextual Token Sparsity hot path.

This module only PREPARES INPUTS (random draws, the Q/K projections with RoPE that stand in for a
trained Llama-shaped layer, heavy-key scaling, rounding to bf16).  It holds none of the method's
arithmetic -- no scoring, selection, gather or scatter -- and is the one piece of code that both the
HIP path's callers and the CPU oracle's callers use, so that both see the same bit patterns.

The paper fine-tunes on real text with trained weights (Sec. 6.1); neither is available here, so
each configuration takes the shapes, dtypes and value distributions of a Llama-shaped layer and
adds the column structure the paper reports for attention maps (Sec. 3: a few token columns dominate)
by scaling the keys of a few positions.

Draw order for a configuration (numpy ``default_rng(seed)``): X, Wq, Wk, W, heavy positions or
Zipf multipliers, G.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Optional, Sequence

import numpy as np
import torch

SEED_BASE = 20250109


@dataclass(frozen=True)
class LayerConfig:
    name: str
    S: int            # tokens
    H: int            # query heads
    H_kv: int         # key/value heads
    d: int            # head_dim
    C: int            # hidden size (GEMM K dimension)
    N: int            # consumer GEMM output width
    dtype: str        # "f32" | "bf16"
    L: int            # segment length
    ratio: float      # keep ratio
    heavy: str        # "fixed16" | "frac1pct" | "zipf"
    direct_qk: bool   # Q,K drawn directly (True) or projected from X with RoPE (False)
    backward: bool    # config includes the scatter-add of gathered-GEMM gradients
    index: int        # 1-based position in the benchmark's config list (seed offset)

    @property
    def k(self) -> int:
        v = math.ceil(self.ratio * self.L - 1e-9)
        return max(1, min(self.L, v))

    @property
    def n_seg(self) -> int:
        return (self.S + self.L - 1) // self.L

    @property
    def M(self) -> int:
        full, tail = divmod(self.S, self.L)
        m = full * self.k
        if tail:
            m += max(1, min(tail, -(-self.k * tail // self.L)))
        return m

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index


CONFIGS = {
    "C1": LayerConfig("C1", 1024, 4, 4, 64, 256, 256, "f32", 128, 0.5, "fixed16", True, False, 1),
    "C2": LayerConfig("C2", 4096, 32, 32, 128, 4096, 11008, "bf16", 512, 0.5, "frac1pct", False, False, 2),
    "C3": LayerConfig("C3", 8192, 32, 32, 128, 4096, 11008, "bf16", 512, 0.4, "frac1pct", False, True, 3),
    "C4": LayerConfig("C4", 16384, 32, 8, 128, 4096, 14336, "bf16", 1024, 0.5, "frac1pct", False, False, 4),
    "C5": LayerConfig("C5", 32768, 32, 32, 128, 4096, 11008, "bf16", 1024, 0.3, "zipf", False, True, 5),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of a configuration with some fields replaced (smaller S, fewer heads, ...)."""
    return replace(cfg, **kw)


# ---------------------------------------------------------------------------------- helpers

def to_bf16_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 torch tensor (any device) -> numpy uint16 array of the same bit patterns."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def as_numpy(t: torch.Tensor) -> np.ndarray:
    """Tensor -> numpy array the oracle accepts (float32, int32, or uint16 bf16 bits)."""
    if t.dtype == torch.bfloat16:
        return to_bf16_bits(t)
    return t.detach().cpu().contiguous().numpy()


def _normal(rng: np.random.Generator, shape, std: float = 1.0) -> torch.Tensor:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return torch.from_numpy(a)


def _rope(x: torch.Tensor, base: float = 10000.0) -> torch.Tensor:
    """Rotary position embedding, rotate-half convention, position = token index.  x: [S,h,d] fp32."""
    S, _, d = x.shape
    half = d // 2
    inv_freq = 1.0 / (base ** (torch.arange(0, half, dtype=torch.float64, device=x.device) / half))
    ang = torch.arange(S, dtype=torch.float64, device=x.device)[:, None] * inv_freq[None, :]
    cos = torch.cos(ang).to(torch.float32)[:, None, :]
    sin = torch.sin(ang).to(torch.float32)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)


def key_multipliers(cfg: LayerConfig, rng: np.random.Generator) -> np.ndarray:
    """Per-token key-norm multiplier [S] float32: the heavy-key structure of a configuration."""
    mult = np.ones(cfg.S, dtype=np.float32)
    if cfg.heavy == "fixed16":
        pos = rng.choice(cfg.S, size=min(16, cfg.S), replace=False)
        mult[pos] = 4.0
    elif cfg.heavy == "frac1pct":
        n = max(1, int(round(0.01 * cfg.S)))
        pos = rng.choice(cfg.S, size=n, replace=False)
        mult[pos] = 4.0
    elif cfg.heavy == "zipf":
        z = rng.zipf(1.1, size=cfg.S)
        mult = np.clip(z, 1, 4).astype(np.float32)
    elif cfg.heavy != "none":
        raise ValueError(cfg.heavy)
    return mult


def make_layer(cfg: LayerConfig, *, seed: Optional[int] = None, heads: Optional[Sequence[int]] = None,
               want_gemm: bool = True, want_grad: Optional[bool] = None, device: str = "cpu") -> dict:
    """Build the tensors of one layer.

    Returns a dict of torch tensors on ``device``: ``Q`` [S,h,d], ``K`` [S,h_kv,d] (bf16 or fp32),
    ``X`` [S,C], ``W`` [N,C] (if ``want_gemm``), ``G`` [M,C] (if ``want_grad``), ``mult`` [S] fp32.
    ``heads`` restricts Q to the listed query heads and K to the KV heads they read (a cheap
    slice for large-S checks; the draws are unchanged, so head h holds the same values either way).
    ``device`` only chooses where the projection matmuls run; the draws are always made on the host.
    """
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    want_grad = cfg.backward if want_grad is None else want_grad
    out: dict = {"cfg": cfg}
    hsel = list(range(cfg.H)) if heads is None else list(heads)
    group = cfg.H // cfg.H_kv
    kvsel = sorted({h // group for h in hsel})
    # the slice must keep the GQA mapping "query head i reads KV head floor(i * h_kv / h)" valid
    if len(hsel) % len(kvsel) or any(h // group != kvsel[i * len(kvsel) // len(hsel)] for i, h in enumerate(hsel)):
        raise ValueError("head subset must keep whole, ordered GQA groups")

    if cfg.direct_qk:
        q = _normal(rng, (cfg.S, cfg.H, cfg.d))
        k = _normal(rng, (cfg.S, cfg.H_kv, cfg.d))
        _v = _normal(rng, (cfg.S, cfg.H_kv, cfg.d))  # drawn for fidelity to the configuration; unused
        X = _normal(rng, (cfg.S, cfg.C))
        W = _normal(rng, (cfg.N, cfg.C), 0.02)
        mult = key_multipliers(cfg, rng)
        q = q[:, hsel]
        k = k[:, kvsel] * torch.from_numpy(mult)[:, None, None]
    else:
        X = _normal(rng, (cfg.S, cfg.C))
        Wq = _normal(rng, (cfg.H * cfg.d, cfg.C), 0.02)
        Wk = _normal(rng, (cfg.H_kv * cfg.d, cfg.C), 0.02)
        W = _normal(rng, (cfg.N, cfg.C), 0.02)  # always drawn, so later draws do not depend on want_gemm
        mult = key_multipliers(cfg, rng)
        rows_q = torch.cat([torch.arange(h * cfg.d, (h + 1) * cfg.d) for h in hsel])
        rows_k = torch.cat([torch.arange(g * cfg.d, (g + 1) * cfg.d) for g in kvsel])
        Xd = X.to(device)
        q = (Xd @ Wq[rows_q].to(device).T).view(cfg.S, len(hsel), cfg.d)
        k = (Xd @ Wk[rows_k].to(device).T).view(cfg.S, len(kvsel), cfg.d)
        q = _rope(q)
        k = _rope(k) * torch.from_numpy(mult).to(device)[:, None, None]
        del Xd
    out["Q"] = q.to(tdt).contiguous().to(device)
    out["K"] = k.to(tdt).contiguous().to(device)
    out["mult"] = torch.from_numpy(mult)
    if want_gemm:
        out["X"] = X.to(tdt).to(device)
        out["W"] = W.to(tdt).to(device)
    if want_grad:
        out["G"] = _normal(rng, (cfg.M, cfg.C)).to(tdt).to(device)
    return out


def tiny_qk(S: int, H: int, H_kv: int, d: int, dtype: str, seed: int, heavy: int = 0):
    """Small direct-draw Q,K for edge-case tests: N(0,1) entries, ``heavy`` key rows scaled by 4."""
    rng = np.random.default_rng(seed)
    q = _normal(rng, (S, H, d))
    k = _normal(rng, (S, H_kv, d))
    if heavy:
        pos = rng.choice(S, size=min(heavy, S), replace=False)
        k[pos] *= 4.0
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    return q.to(tdt), k.to(tdt)
