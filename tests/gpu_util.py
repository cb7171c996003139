"""Helpers shared by the GPU parity tests: upload workloads, call the C ABI, compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

from paper_2602_14209_amd import binding as mb
from paper_2602_14209_amd.workloads import device_bits

ATOL = {"bf16": 2e-2, "f32": 1e-4}        # max-abs tolerance on attention outputs (spec bar)
TIE_BAND = 1e-6                           # index mismatches excused within this relative band of the k-th score


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    bits = device_bits(a, dtype)
    if dtype == "bf16":
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(bits).cuda()


class Problem:
    """Device-side buffers of one (layer, block) problem plus the C-ABI shape."""

    def __init__(self, q, k_cache, v_cache, k_blk, v_blk, k, dtype):
        B, Hq, d = q.shape
        L, Hkv, _ = k_cache.shape
        self.dtype = dtype
        self.dims = (B, Hq, Hkv, d, L, k)
        self.shape = mb.make_shape(B, Hq, Hkv, d, L, k, dtype)
        self.q = to_device(q, dtype)
        self.kc = to_device(k_cache, dtype)
        self.vc = to_device(v_cache, dtype)
        self.kb = None if k_blk is None else to_device(k_blk, dtype)
        self.vb = None if v_blk is None else to_device(v_blk, dtype)
        self.ws = mb.alloc_workspace(self.shape)
        self.out = torch.full((B, Hq, d), float("nan"), dtype=torch.float32, device="cuda")
        self.lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device="cuda")
        self.idx = torch.full((Hkv, k), -1, dtype=torch.int32, device="cuda")
        self.alpha = torch.full((Hkv, L), float("nan"), dtype=torch.float32, device="cuda")

    def set_q(self, q):
        self.q = to_device(q, self.dtype)

    def set_blk(self, k_blk, v_blk):
        self.kb = to_device(k_blk, self.dtype)
        self.vb = to_device(v_blk, self.dtype)

    def select(self, with_alpha=True):
        mb.check(mb.mage_select(self.shape, self.q, self.kc, self.idx, self.alpha if with_alpha else None, self.ws),
                 "mage_select")
        torch.cuda.synchronize()
        return self.idx.cpu().numpy(), (self.alpha.cpu().numpy() if with_alpha else None)

    def block_probs(self):
        B, Hq, Hkv, d, L, k = self.dims
        pbar = torch.empty((Hq, L), dtype=torch.float32, device="cuda")
        mb.check(mb.mage_block_probs(self.shape, self.q, self.kc, pbar, self.ws), "mage_block_probs")
        torch.cuda.synchronize()
        return pbar.cpu().numpy()

    def step1(self):
        mb.check(mb.mage_step1(self.shape, self.q, self.kc, self.vc, self.kb, self.vb, self.out, self.lse, self.idx,
                               self.alpha, self.ws), "mage_step1")
        torch.cuda.synchronize()
        return self.out.cpu().numpy(), self.lse.cpu().numpy(), self.idx.cpu().numpy(), self.alpha.cpu().numpy()

    def exact(self):
        mb.check(mb.mage_exact_attn(self.shape, self.q, self.kc, self.vc, self.kb, self.vb, self.out, self.lse, self.ws),
                 "mage_exact_attn")
        torch.cuda.synchronize()
        return self.out.cpu().numpy(), self.lse.cpu().numpy()

    def sparse(self, idx: np.ndarray):
        idx_d = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).cuda()
        mb.check(mb.mage_sparse_attn(self.shape, self.q, self.kc, self.vc, idx_d, self.kb, self.vb, self.out, self.lse,
                                     self.ws), "mage_sparse_attn")
        torch.cuda.synchronize()
        return self.out.cpu().numpy(), self.lse.cpu().numpy()


def check_index_sets(idx_gpu: np.ndarray, idx_ref: np.ndarray, alpha32_ref: np.ndarray, L: int):
    """Bit-exact sets, except entries whose ORACLE fp32 score is within TIE_BAND (relative) of the
    oracle's k-th largest score of that head.  Returns the number of excused entries."""
    Hkv, k = idx_ref.shape
    assert idx_gpu.shape == idx_ref.shape and idx_gpu.dtype == np.int32
    excused = 0
    for h in range(Hkv):
        g = idx_gpu[h]
        assert g.min() >= 0 and g.max() < L, f"head {h}: index out of range"
        assert np.all(np.diff(g) > 0), f"head {h}: indices not strictly ascending"
        if np.array_equal(g, idx_ref[h]):
            continue
        kth = float(np.sort(alpha32_ref[h])[::-1][k - 1])
        diff = np.setxor1d(g, idx_ref[h])
        rel = np.abs(alpha32_ref[h, diff].astype(np.float64) - kth) / kth
        srt = np.sort(alpha32_ref[h])[::-1]
        margin = (srt[k - 1] - srt[k]) / srt[k - 1] if k < L else float("inf")
        assert np.all(rel <= TIE_BAND), (
            f"head {h}: {diff.size} mismatching indices, worst relative distance to the k-th score {rel.max():.3e} "
            f"(band {TIE_BAND}); oracle margin at rank k {margin:.3e}")
        excused += diff.size
    return excused


def check_alpha(alpha_gpu: np.ndarray, alpha_ref: np.ndarray, rtol=2e-4):
    assert np.all(np.isfinite(alpha_gpu)) and np.all(alpha_gpu >= 0)
    np.testing.assert_allclose(alpha_gpu.sum(axis=1, dtype=np.float64), 1.0, atol=1e-4)
    floor = alpha_ref.max(axis=1, keepdims=True) * 1e-6
    err = np.abs(alpha_gpu - alpha_ref) / (alpha_ref + floor)
    assert err.max() <= rtol, f"alpha relative error {err.max():.3e} > {rtol}"


def check_out(out_gpu, out_ref, lse_gpu, lse_ref, dtype):
    assert np.all(np.isfinite(out_gpu)), "non-finite attention output"
    err = np.abs(out_gpu.astype(np.float64) - out_ref.astype(np.float64)).max()
    assert err <= ATOL[dtype], f"attention max-abs error {err:.3e} > {ATOL[dtype]}"
    if lse_gpu is not None:
        lerr = np.abs(lse_gpu.astype(np.float64) - lse_ref.astype(np.float64)).max()
        assert lerr <= (1e-3 if dtype == "bf16" else 1e-4), f"lse max-abs error {lerr:.3e}"
    return err
