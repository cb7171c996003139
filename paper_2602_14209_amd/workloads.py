"""Seeded synthetic workloads for the MAGE hot path (inputs only, no method arithmetic).

Stand-ins for the paper's LongBench / NIAH runs (Sec. 5), whose items, models and
weights are not available: shapes are those of the evaluated families (B=32,
k in {256,512,1024}, 8K-128K context, GQA) and the value structure concentrates
attention mass on a few "heavy-hitter" keys, the regime in which a top-k budget
captures most of the mass.  Both the CPU oracle (through the tests) and the HIP
path consume the arrays produced here; bf16 workloads are rounded to bf16 on the
host (round-to-nearest-even) and handed out both as bf16 bit patterns (uint16)
and as the exactly equal float32 values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" | "bf16"
    Hq: int
    Hkv: int
    d: int
    L: int
    B: int
    ks: Tuple[int, ...]   # budgets k evaluated on this workload
    T: int                # denoising steps per block
    layers: int = 1
    heavy_frac: float = 0.0   # fraction of cache positions (per KV head) whose key row is scaled
    heavy_scale: float = 1.0
    drift: float = 0.0        # rise of the mean logit from j=0 to j=L-1 (0 = none)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def k(self) -> int:
        return self.ks[0] if len(self.ks) == 1 else self.ks[len(self.ks) // 2]

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS: Dict[str, Workload] = {
    "c0": Workload("c0", "f32", Hq=4, Hkv=1, d=64, L=2048, B=4, ks=(64,), T=4),
    "c1": Workload("c1", "bf16", Hq=28, Hkv=4, d=128, L=8192, B=32, ks=(512,), T=8,
                   heavy_frac=0.01, heavy_scale=4.0),
    "c2": Workload("c2", "bf16", Hq=32, Hkv=8, d=128, L=32768, B=32, ks=(512,), T=8,
                   heavy_frac=0.01, heavy_scale=4.0),
    "c3": Workload("c3", "bf16", Hq=28, Hkv=4, d=128, L=65536, B=32, ks=(512,), T=8, layers=28,
                   heavy_frac=0.01, heavy_scale=4.0),
    "c4": Workload("c4", "bf16", Hq=32, Hkv=8, d=128, L=131072, B=32, ks=(256, 512, 1024), T=16,
                   heavy_frac=0.005, heavy_scale=4.0, drift=2.0),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the exactly equal float32 values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def layer_seed(base_seed: int, cfg_index: int, layer: int) -> int:
    return int(base_seed) + 1000 * int(cfg_index) + int(layer)


def make_layer(w: Workload, seed: int, steps: int | None = None) -> Dict[str, np.ndarray]:
    """One layer's inputs for one block.

    Returns float32 arrays (bf16-representable when ``w.dtype == "bf16"``):
      q      [T,B,Hq,d]   q[0] = Q1 (All-[MASK] step), q[t] = Q1 + 0.3 N(0,1)
      k_blk  [T,B,Hkv,d]  in-block keys, fresh per step
      v_blk  [T,B,Hkv,d]
      k_cache, v_cache [L,Hkv,d]
      heavy  [Hkv, n_heavy] int64 positions of the scaled key rows (diagnostic)
    """
    T = w.T if steps is None else int(steps)
    rng = np.random.default_rng(seed)
    f32 = np.float32
    q_mask = rng.standard_normal((w.Hq, w.d), dtype=f32)
    q1 = q_mask[None, :, :] + f32(0.1) * rng.standard_normal((w.B, w.Hq, w.d), dtype=f32)
    q = np.empty((T, w.B, w.Hq, w.d), f32)
    q[0] = q1
    for t in range(1, T):
        q[t] = q1 + f32(0.3) * rng.standard_normal((w.B, w.Hq, w.d), dtype=f32)
    k_blk = rng.standard_normal((T, w.B, w.Hkv, w.d), dtype=f32)
    v_blk = rng.standard_normal((T, w.B, w.Hkv, w.d), dtype=f32)
    k_cache = rng.standard_normal((w.L, w.Hkv, w.d), dtype=f32)
    v_cache = rng.standard_normal((w.L, w.Hkv, w.d), dtype=f32)

    n_heavy = int(round(w.heavy_frac * w.L))
    heavy = np.empty((w.Hkv, n_heavy), np.int64)
    for h in range(w.Hkv):
        pos = np.sort(rng.choice(w.L, size=n_heavy, replace=False)) if n_heavy else np.empty((0,), np.int64)
        heavy[h] = pos
        if n_heavy:
            k_cache[pos, h, :] *= f32(w.heavy_scale)
    if w.drift != 0.0:
        # recency bias: K[j,h,:] += gamma_h * (j/L) * u_h, u_h the unit vector of the group-mean
        # q_mask, gamma_h chosen so that the mean logit rises by `drift` from j=0 to j=L-1.
        ramp = (np.arange(w.L, dtype=np.float64) / w.L).astype(f32)
        for h in range(w.Hkv):
            qbar = q_mask[h * w.G:(h + 1) * w.G].astype(np.float64).mean(axis=0)
            nrm = float(np.linalg.norm(qbar))
            gamma = w.drift * np.sqrt(w.d) / nrm
            k_cache[:, h, :] += ramp[:, None] * (gamma * qbar / nrm).astype(f32)[None, :]

    out = {"q": q, "k_blk": k_blk, "v_blk": v_blk, "k_cache": k_cache, "v_cache": v_cache}
    if w.dtype == "bf16":
        out = {n: bf16_to_f32(round_to_bf16(a)) for n, a in out.items()}
    elif w.dtype != "f32":
        raise ValueError(f"unknown dtype {w.dtype}")
    out["heavy"] = heavy
    return out


def device_bits(a: np.ndarray, dtype: str) -> np.ndarray:
    """The array as the device consumes it: float32 as is, bf16 as uint16 bit patterns."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        bits = round_to_bf16(a)
        if not np.array_equal(bf16_to_f32(bits), np.asarray(a, dtype=np.float32)):
            raise ValueError("array is not bf16-representable")
        return bits
    raise ValueError(f"unknown dtype {dtype}")


def make_layer_device(w: Workload, seed: int, device="cuda", steps: int | None = None):
    """The recipe of :func:`make_layer`, drawn on the device with torch's seeded generator (used by
    the benchmark, where 28 layers of 128K-token caches would take minutes to draw on the host).
    Returns torch tensors of the workload's dtype with the same names and shapes."""
    import torch

    T = w.T if steps is None else int(steps)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    def randn(*shape):
        return torch.randn(*shape, generator=g, device=device, dtype=torch.float32)

    q_mask = randn(w.Hq, w.d)
    q1 = q_mask[None] + 0.1 * randn(w.B, w.Hq, w.d)
    q = torch.empty((T, w.B, w.Hq, w.d), device=device, dtype=torch.float32)
    q[0] = q1
    for t in range(1, T):
        q[t] = q1 + 0.3 * randn(w.B, w.Hq, w.d)
    k_blk = randn(T, w.B, w.Hkv, w.d)
    v_blk = randn(T, w.B, w.Hkv, w.d)
    k_cache = torch.empty((w.L, w.Hkv, w.d), device=device, dtype=dt)
    v_cache = torch.empty((w.L, w.Hkv, w.d), device=device, dtype=dt)
    n_heavy = int(round(w.heavy_frac * w.L))
    chunk = 16384
    heavy_mask = torch.zeros((w.L, w.Hkv), device=device, dtype=torch.bool)
    for h in range(w.Hkv):
        if n_heavy:
            pos = torch.randperm(w.L, generator=g, device=device)[:n_heavy]
            heavy_mask[pos, h] = True
    dirs = None
    if w.drift != 0.0:
        qbar = q_mask.view(w.Hkv, w.G, w.d).double().mean(dim=1)
        nrm = qbar.norm(dim=1, keepdim=True)
        dirs = ((w.drift * (w.d ** 0.5) / nrm) * (qbar / nrm)).float()          # gamma_h * u_h, [Hkv,d]
    for j0 in range(0, w.L, chunk):
        j1 = min(w.L, j0 + chunk)
        kk = randn(j1 - j0, w.Hkv, w.d)
        kk = torch.where(heavy_mask[j0:j1, :, None], kk * w.heavy_scale, kk)
        if dirs is not None:
            ramp = (torch.arange(j0, j1, device=device, dtype=torch.float64) / w.L).float()
            kk = kk + ramp[:, None, None] * dirs[None]
        k_cache[j0:j1] = kk.to(dt)
        v_cache[j0:j1] = randn(j1 - j0, w.Hkv, w.d).to(dt)
    return {"q": q.to(dt), "k_blk": k_blk.to(dt), "v_blk": v_blk.to(dt), "k_cache": k_cache, "v_cache": v_cache}


def algorithmic_bytes(w: Workload, k: int) -> Dict[str, int]:
    """Bytes each entry point must move per call (one layer, one block), the figure the roofline
    fractions are computed from: inputs read once, outputs written once, nothing else."""
    esz = 2 if w.dtype == "bf16" else 4
    q = w.B * w.Hq * w.d * esz
    out = w.B * w.Hq * w.d * 4
    blk = 2 * w.B * w.Hkv * w.d * esz
    cache_k = w.L * w.Hkv * w.d * esz
    return {
        "sparse_attn": 2 * w.Hkv * k * w.d * esz + 4 * w.Hkv * k + q + blk + out,
        "exact_attn": 2 * cache_k + q + blk + out,
        "select": 2 * cache_k + 2 * q + 2 * 4 * w.Hkv * w.L + 4 * w.Hkv * k,   # K twice; alpha written + read
    }
