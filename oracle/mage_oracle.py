"""ctypes front end of ``mage_oracle.c`` (test infrastructure, not product code).

Argument marshalling only: every number comes out of the C file, which follows
Alg. 1, Eq. 2 and Eq. 5 of arxiv 2602.14209 in fp64.  Inputs are float32 numpy
arrays (bf16 workloads pass bf16-representable float32 values).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mage_oracle.c")
_LIB = os.path.join(_HERE, "libmage_oracle.so")
_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.mage_oracle_threads.restype = ctypes.c_int
        lib.mage_oracle_block_probs.restype = ctypes.c_int
        lib.mage_oracle_block_probs.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
            _f32p, _f32p, _f64p, _f64p]
        lib.mage_oracle_topk.restype = ctypes.c_int
        lib.mage_oracle_topk.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int, _i32p]
        lib.mage_oracle_select.restype = ctypes.c_int
        lib.mage_oracle_select.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
            _f32p, _f32p, _i32p, _f32p, _f64p, _f64p]
        lib.mage_oracle_attn.restype = ctypes.c_int
        lib.mage_oracle_attn.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
            _f32p, _f32p, _f32p, _i32p, ctypes.c_int, _f32p, _f32p, ctypes.c_int, _f32p, _f32p]
        lib.mage_oracle_compact.restype = ctypes.c_int
        lib.mage_oracle_compact.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int, _f32p, _i32p, _f32p]
        lib.mage_oracle_page_summary.restype = ctypes.c_int
        lib.mage_oracle_page_summary.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int, _f32p, _f32p, _f32p]
        lib.mage_oracle_quest_probs.restype = ctypes.c_int
        lib.mage_oracle_quest_probs.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
                                                ctypes.c_int, _f32p, _f32p, _f32p, _f64p]
        lib.mage_oracle_quest_select.restype = ctypes.c_int
        lib.mage_oracle_quest_select.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
                                                 ctypes.c_int, ctypes.c_int, _f32p, _f32p, _i32p, _f32p]
        lib.mage_oracle_overlap.restype = ctypes.c_double
        lib.mage_oracle_overlap.argtypes = [ctypes.c_int, _i32p, _i32p]
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().mage_oracle_threads())


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a, typ):
    return None if a is None else a.ctypes.data_as(typ)


def _dims(q, kc):
    B, Hq, d = q.shape
    L, Hkv, d2 = kc.shape
    if d2 != d:
        raise ValueError("head dim mismatch")
    return B, Hq, Hkv, d, L


def block_probs(q1, k_cache):
    """(pbar[Hq,L], alpha[Hkv,L]) in fp64 -- Eq. 2 / Eq. 5 averaged probabilities."""
    q1, k_cache = _f32(q1), _f32(k_cache)
    B, Hq, Hkv, d, L = _dims(q1, k_cache)
    pbar = np.empty((Hq, L), np.float64)
    alpha = np.empty((Hkv, L), np.float64)
    rc = _load().mage_oracle_block_probs(B, Hq, Hkv, d, L, _ptr(q1, _f32p), _ptr(k_cache, _f32p),
                                         _ptr(pbar, _f64p), _ptr(alpha, _f64p))
    if rc:
        raise RuntimeError("mage_oracle_block_probs failed")
    return pbar, alpha


def topk(score, k):
    """Indices (ascending) of the k largest fp32 scores, ties to the smaller index."""
    score = _f32(score)
    if score.ndim != 1:
        raise ValueError("score must be 1-D")
    out = np.empty((k,), np.int32)
    rc = _load().mage_oracle_topk(_ptr(score, _f32p), score.shape[0], k, _ptr(out, _i32p))
    if rc:
        raise RuntimeError("mage_oracle_topk failed")
    return out


def select(q1, k_cache, k):
    """Step-1 selection.  Returns dict(idx[Hkv,k] int32, alpha32[Hkv,L], alpha[Hkv,L] f64, pbar[Hq,L] f64)."""
    q1, k_cache = _f32(q1), _f32(k_cache)
    B, Hq, Hkv, d, L = _dims(q1, k_cache)
    idx = np.empty((Hkv, k), np.int32)
    a32 = np.empty((Hkv, L), np.float32)
    alpha = np.empty((Hkv, L), np.float64)
    pbar = np.empty((Hq, L), np.float64)
    rc = _load().mage_oracle_select(B, Hq, Hkv, d, L, k, _ptr(q1, _f32p), _ptr(k_cache, _f32p),
                                    _ptr(idx, _i32p), _ptr(a32, _f32p), _ptr(alpha, _f64p), _ptr(pbar, _f64p))
    if rc:
        raise RuntimeError("mage_oracle_select failed")
    return {"idx": idx, "alpha32": a32, "alpha": alpha, "pbar": pbar}


def _attn(q, k_cache, v_cache, idx, k_blk, v_blk):
    q, k_cache, v_cache = _f32(q), _f32(k_cache), _f32(v_cache)
    B, Hq, Hkv, d, L = _dims(q, k_cache)
    if v_cache.shape != k_cache.shape:
        raise ValueError("K/V cache shape mismatch")
    k = 0
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        if idx.ndim != 2 or idx.shape[0] != Hkv:
            raise ValueError("idx must be [Hkv,k]")
        k = idx.shape[1]
    nb = 0
    if k_blk is not None:
        k_blk, v_blk = _f32(k_blk), _f32(v_blk)
        nb = k_blk.shape[0]
        if k_blk.shape != (nb, Hkv, d) or v_blk.shape != k_blk.shape:
            raise ValueError("k_blk / v_blk must be [nb,Hkv,d]")
    out = np.empty((B, Hq, d), np.float32)
    lse = np.empty((B, Hq), np.float32)
    rc = _load().mage_oracle_attn(B, Hq, Hkv, d, L, _ptr(q, _f32p), _ptr(k_cache, _f32p), _ptr(v_cache, _f32p),
                                  _ptr(idx, _i32p), k, _ptr(k_blk, _f32p), _ptr(v_blk, _f32p), nb,
                                  _ptr(out, _f32p), _ptr(lse, _f32p))
    if rc:
        raise RuntimeError("mage_oracle_attn failed")
    return out, lse


def exact_attn(q, k_cache, v_cache, k_blk=None, v_blk=None):
    """Exact attention over all L cache keys plus the in-block keys -> (out[B,Hq,d], lse[B,Hq])."""
    return _attn(q, k_cache, v_cache, None, k_blk, v_blk)


def sparse_attn(q, k_cache, v_cache, idx, k_blk=None, v_blk=None):
    """Sparse attention over cache[idx[kv(g)]] plus the in-block keys -> (out, lse)."""
    return _attn(q, k_cache, v_cache, idx, k_blk, v_blk)


def compact(cache, idx):
    """Rows selected by idx[Hkv,k] copied into a cache of length k: out[p,h,:] = cache[idx[h,p],h,:]."""
    cache = _f32(cache)
    L, Hkv, d = cache.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim != 2 or idx.shape[0] != Hkv:
        raise ValueError("idx must be [Hkv,k]")
    k = idx.shape[1]
    out = np.empty((k, Hkv, d), np.float32)
    rc = _load().mage_oracle_compact(Hkv, d, L, k, _ptr(cache, _f32p), _ptr(idx, _i32p), _ptr(out, _f32p))
    if rc:
        raise RuntimeError("mage_oracle_compact failed")
    return out


def page_summary(k_cache, p):
    """Quest page summaries (Sec. 2): per-channel (max, min) of every run of p cache rows -> two [ceil(L/p),Hkv,d] arrays."""
    k_cache = _f32(k_cache)
    L, Hkv, d = k_cache.shape
    n_pages = (L + p - 1) // p
    kmax = np.empty((n_pages, Hkv, d), np.float32)
    kmin = np.empty((n_pages, Hkv, d), np.float32)
    rc = _load().mage_oracle_page_summary(Hkv, d, L, p, _ptr(k_cache, _f32p), _ptr(kmax, _f32p), _ptr(kmin, _f32p))
    if rc:
        raise RuntimeError("mage_oracle_page_summary failed")
    return kmax, kmin


def quest_probs(q, kmax, kmin, L, p):
    """Per-block averaged estimated scores est[Hkv,L] (fp64): Eq. 2 with every logit replaced by its page's bound."""
    q, kmax, kmin = _f32(q), _f32(kmax), _f32(kmin)
    B, Hq, d = q.shape
    n_pages, Hkv, d2 = kmax.shape
    if d2 != d or kmin.shape != kmax.shape or n_pages != (L + p - 1) // p:
        raise ValueError("page summary shape mismatch")
    est = np.empty((Hkv, L), np.float64)
    rc = _load().mage_oracle_quest_probs(B, Hq, Hkv, d, L, p, _ptr(q, _f32p), _ptr(kmax, _f32p), _ptr(kmin, _f32p),
                                         _ptr(est, _f64p))
    if rc:
        raise RuntimeError("mage_oracle_quest_probs failed")
    return est


def quest_select(q, k_cache, p, k):
    """Estimated per-block KV subset.  Returns dict(idx[Hkv,k] int32 ascending, est32[Hkv,L])."""
    q, k_cache = _f32(q), _f32(k_cache)
    B, Hq, Hkv, d, L = _dims(q, k_cache)
    idx = np.empty((Hkv, k), np.int32)
    e32 = np.empty((Hkv, L), np.float32)
    rc = _load().mage_oracle_quest_select(B, Hq, Hkv, d, L, p, k, _ptr(q, _f32p), _ptr(k_cache, _f32p),
                                          _ptr(idx, _i32p), _ptr(e32, _f32p))
    if rc:
        raise RuntimeError("mage_oracle_quest_select failed")
    return {"idx": idx, "est32": e32}


def overlap(a, b):
    """|A intersect B| / k for two index sets of equal size k (Eq. 1, Eq. 3)."""
    a = np.ascontiguousarray(a, dtype=np.int32).ravel()
    b = np.ascontiguousarray(b, dtype=np.int32).ravel()
    if a.shape != b.shape:
        raise ValueError("sets must have the same size")
    r = _load().mage_oracle_overlap(a.shape[0], _ptr(a, _i32p), _ptr(b, _i32p))
    if r < 0:
        raise RuntimeError("mage_oracle_overlap failed")
    return float(r)

