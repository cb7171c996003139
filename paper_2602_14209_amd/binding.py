"""Thin ctypes binding of libmage.so (argument marshalling only).

Every step of the MAGE hot path runs inside the HIP library; PyTorch is used for
device memory and streams.  The functions carry the names of the C entry points
declared in ``include/mage.h`` and take torch CUDA(HIP) tensors in place of raw
device pointers.  There is no CPU fallback: if the library is missing, importing
or calling this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # noqa: F401  (must be imported first: libmage.so binds to the HIP runtime torch loaded)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmage.so")

MAGE_F32 = 0
MAGE_BF16 = 1
MAGE_OK = 0

EXPORTS = ("mage_version", "mage_status_string", "mage_workspace_bytes",
           "mage_select", "mage_block_probs", "mage_exact_attn", "mage_sparse_attn", "mage_step1",
           "mage_compact", "mage_sparse_attn_compact", "mage_sparse_attn_batched",
           "mage_page_summary", "mage_quest_workspace_bytes", "mage_quest_select", "mage_set_overlap",
           "mage_static_scratch_bytes", "mage_select_static",
           "mage_diag_empty", "mage_diag_stamp", "mage_diag_stamp_hz", "mage_diag_chase", "mage_diag_read", "mage_diag_copy", "mage_diag_merge", "mage_diag_gather")


class mage_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("Hq", ctypes.c_int), ("Hkv", ctypes.c_int), ("d", ctypes.c_int),
                ("L", ctypes.c_int64), ("k", ctypes.c_int), ("dtype", ctypes.c_int)]


class MageError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libmage.so (built in-tree by ``paper_2602_14209_amd.build``); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2602_14209_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        shp = ctypes.POINTER(mage_shape)
        L.mage_version.restype = ctypes.c_int
        L.mage_status_string.restype = ctypes.c_char_p
        L.mage_status_string.argtypes = [ctypes.c_int]
        L.mage_workspace_bytes.restype = sz
        L.mage_workspace_bytes.argtypes = [shp]
        L.mage_select.restype = ctypes.c_int
        L.mage_select.argtypes = [shp, vp, vp, vp, vp, vp, sz, vp]
        L.mage_block_probs.restype = ctypes.c_int
        L.mage_block_probs.argtypes = [shp, vp, vp, vp, vp, sz, vp]
        L.mage_exact_attn.restype = ctypes.c_int
        L.mage_exact_attn.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.mage_sparse_attn.restype = ctypes.c_int
        L.mage_sparse_attn.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.mage_compact.restype = ctypes.c_int
        L.mage_compact.argtypes = [shp, vp, vp, vp, vp, vp, vp]
        L.mage_sparse_attn_compact.restype = ctypes.c_int
        L.mage_sparse_attn_compact.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.mage_sparse_attn_batched.restype = ctypes.c_int
        L.mage_sparse_attn_batched.argtypes = [shp, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.mage_step1.restype = ctypes.c_int
        L.mage_step1.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.mage_page_summary.restype = ctypes.c_int
        L.mage_page_summary.argtypes = [shp, ctypes.c_int, vp, vp, vp]
        L.mage_quest_workspace_bytes.restype = sz
        L.mage_quest_workspace_bytes.argtypes = [shp, ctypes.c_int]
        L.mage_quest_select.restype = ctypes.c_int
        L.mage_quest_select.argtypes = [shp, ctypes.c_int, vp, vp, vp, vp, vp, sz, vp]
        L.mage_set_overlap.restype = ctypes.c_int
        L.mage_set_overlap.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
        L.mage_static_scratch_bytes.restype = sz
        L.mage_static_scratch_bytes.argtypes = []
        L.mage_select_static.restype = ctypes.c_int
        L.mage_select_static.argtypes = [shp, vp, vp, vp, vp, vp]
        L.mage_diag_empty.restype = ctypes.c_int
        L.mage_diag_empty.argtypes = [vp]
        L.mage_diag_stamp.restype = ctypes.c_int
        L.mage_diag_stamp.argtypes = [vp, vp]
        L.mage_diag_stamp_hz.restype = ctypes.c_int64
        L.mage_diag_stamp_hz.argtypes = []
        L.mage_diag_chase.restype = ctypes.c_int
        L.mage_diag_chase.argtypes = [vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, vp, vp]
        L.mage_diag_read.restype = ctypes.c_int
        L.mage_diag_read.argtypes = [vp, sz, vp, vp]
        L.mage_diag_copy.restype = ctypes.c_int
        L.mage_diag_copy.argtypes = [vp, vp, sz, vp]
        L.mage_diag_merge.restype = ctypes.c_int
        L.mage_diag_merge.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp, vp, vp, vp]
        L.mage_diag_gather.restype = ctypes.c_int
        L.mage_diag_gather.argtypes = [shp, ctypes.c_int, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().mage_status_string(int(status)).decode()


def make_shape(B: int, Hq: int, Hkv: int, d: int, L: int, k: int, dtype) -> mage_shape:
    if isinstance(dtype, str):
        dt = {"f32": MAGE_F32, "bf16": MAGE_BF16}[dtype]
    elif isinstance(dtype, torch.dtype):
        dt = {torch.float32: MAGE_F32, torch.bfloat16: MAGE_BF16}[dtype]
    else:
        dt = int(dtype)
    return mage_shape(B, Hq, Hkv, d, L, k, dt)


def mage_workspace_bytes(shape: mage_shape) -> int:
    return int(lib().mage_workspace_bytes(ctypes.byref(shape)))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _wsize(ws: Optional[torch.Tensor]) -> int:
    return 0 if ws is None else ws.numel() * ws.element_size()


def mage_select(shape: mage_shape, q1, k_cache, idx_out, alpha_out, workspace, stream=None) -> int:
    """Step-1 selection; see include/mage.h.  Returns the status code (0 = ok)."""
    return lib().mage_select(ctypes.byref(shape), _ptr(q1), _ptr(k_cache), _ptr(idx_out), _ptr(alpha_out),
                             _ptr(workspace), _wsize(workspace), _stream(stream))


def mage_block_probs(shape: mage_shape, q1, k_cache, pbar_out, workspace, stream=None) -> int:
    """Block-averaged probabilities per query head, pbar_out [Hq,L]; see include/mage.h."""
    return lib().mage_block_probs(ctypes.byref(shape), _ptr(q1), _ptr(k_cache), _ptr(pbar_out),
                                  _ptr(workspace), _wsize(workspace), _stream(stream))


def mage_exact_attn(shape: mage_shape, q, k_cache, v_cache, k_blk, v_blk, out, lse_out, workspace, stream=None) -> int:
    """Exact attention over cache + block; see include/mage.h."""
    return lib().mage_exact_attn(ctypes.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_blk), _ptr(v_blk),
                                 _ptr(out), _ptr(lse_out), _ptr(workspace), _wsize(workspace), _stream(stream))


def mage_sparse_attn(shape: mage_shape, q, k_cache, v_cache, idx, k_blk, v_blk, out, lse_out, workspace,
                     stream=None) -> int:
    """Sparse attention of one denoising step; see include/mage.h."""
    return lib().mage_sparse_attn(ctypes.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(idx), _ptr(k_blk),
                                  _ptr(v_blk), _ptr(out), _ptr(lse_out), _ptr(workspace), _wsize(workspace),
                                  _stream(stream))


def mage_step1(shape: mage_shape, q1, k_cache, v_cache, k_blk, v_blk, out, lse_out, idx_out, alpha_out, workspace,
               stream=None) -> int:
    """Step-1 attention and selection in one call (shared statistics pass); see include/mage.h."""
    return lib().mage_step1(ctypes.byref(shape), _ptr(q1), _ptr(k_cache), _ptr(v_cache), _ptr(k_blk), _ptr(v_blk),
                            _ptr(out), _ptr(lse_out), _ptr(idx_out), _ptr(alpha_out), _ptr(workspace),
                            _wsize(workspace), _stream(stream))


def mage_compact(shape: mage_shape, k_cache, v_cache, idx, k_sel, v_sel, stream=None) -> int:
    """Copy the selected rows into a cache of length k; see include/mage.h."""
    return lib().mage_compact(ctypes.byref(shape), _ptr(k_cache), _ptr(v_cache), _ptr(idx), _ptr(k_sel), _ptr(v_sel),
                              _stream(stream))


def mage_sparse_attn_compact(shape: mage_shape, q, k_sel, v_sel, k_blk, v_blk, out, lse_out, workspace,
                             stream=None) -> int:
    """Sparse step on compacted rows; see include/mage.h."""
    return lib().mage_sparse_attn_compact(ctypes.byref(shape), _ptr(q), _ptr(k_sel), _ptr(v_sel), _ptr(k_blk),
                                          _ptr(v_blk), _ptr(out), _ptr(lse_out), _ptr(workspace), _wsize(workspace),
                                          _stream(stream))


def mage_sparse_attn_batched(shape: mage_shape, n_seq: int, q, k_cache, v_cache, idx, k_blk, v_blk, out, lse_out,
                             stream=None) -> int:
    """Sparse step of n_seq independent sequences in one launch; see include/mage.h."""
    return lib().mage_sparse_attn_batched(ctypes.byref(shape), int(n_seq), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                          _ptr(idx), _ptr(k_blk), _ptr(v_blk), _ptr(out), _ptr(lse_out),
                                          _stream(stream))


def mage_page_summary(shape: mage_shape, p: int, k_cache, summary, stream=None) -> int:
    """Per-page (max, min) key rows; see include/mage.h."""
    return lib().mage_page_summary(ctypes.byref(shape), int(p), _ptr(k_cache), _ptr(summary), _stream(stream))


def mage_quest_workspace_bytes(shape: mage_shape, p: int) -> int:
    return int(lib().mage_quest_workspace_bytes(ctypes.byref(shape), int(p)))


def mage_quest_select(shape: mage_shape, p: int, q, summary, idx_out, est_out, workspace, stream=None) -> int:
    """Estimated per-block KV subset from page summaries; see include/mage.h."""
    return lib().mage_quest_select(ctypes.byref(shape), int(p), _ptr(q), _ptr(summary), _ptr(idx_out), _ptr(est_out),
                                   _ptr(workspace), _wsize(workspace), _stream(stream))


def mage_set_overlap(a, b, n_rows: int, k: int, a_rows: int, out, stream=None) -> int:
    """out[i] = |A_(i mod a_rows) & B_i| / k (Eq. 1, Eq. 3); see include/mage.h."""
    return lib().mage_set_overlap(_ptr(a), _ptr(b), int(n_rows), int(k), int(a_rows), _ptr(out), _stream(stream))


def mage_static_scratch_bytes() -> int:
    return int(lib().mage_static_scratch_bytes())


def mage_select_static(shape: mage_shape, q1, k_cache, idx_out, alpha_out, stream=None) -> int:
    """mage_select on the library's static scratch array (no workspace, no allocation); see include/mage.h."""
    return lib().mage_select_static(ctypes.byref(shape), _ptr(q1), _ptr(k_cache), _ptr(idx_out), _ptr(alpha_out),
                                    _stream(stream))


def mage_diag_empty(stream=None) -> int:
    return lib().mage_diag_empty(_stream(stream))


def mage_diag_stamp(out, stream=None) -> int:
    """out: one int64 element of a device tensor (a view such as stamps[i:i+1])."""
    return lib().mage_diag_stamp(_ptr(out), _stream(stream))


def mage_diag_stamp_hz() -> int:
    return int(lib().mage_diag_stamp_hz())


def mage_diag_chase(chain, start: int, n_hops: int, out, stream=None) -> int:
    return lib().mage_diag_chase(_ptr(chain), chain.numel(), int(start), int(n_hops), _ptr(out), _stream(stream))


def mage_diag_read(src, sink, stream=None) -> int:
    return lib().mage_diag_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream))


def mage_diag_copy(dst, src, stream=None) -> int:
    return lib().mage_diag_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream))


def mage_diag_merge(mode: int, n_groups: int, part, counters, out, src, stream=None) -> int:
    return lib().mage_diag_merge(int(mode), int(n_groups), _ptr(part), _ptr(counters), _ptr(out), _ptr(src), _stream(stream))


def mage_diag_gather(shape: mage_shape, n_seq: int, k_cache, v_cache, idx, sink, stream=None) -> int:
    return lib().mage_diag_gather(ctypes.byref(shape), int(n_seq), _ptr(k_cache), _ptr(v_cache), _ptr(idx), _ptr(sink),
                                  _stream(stream))


def check(status: int, where: str = "mage") -> None:
    if status != MAGE_OK:
        raise MageError(status, where)


def alloc_workspace(shape: mage_shape, device="cuda") -> torch.Tensor:
    n = mage_workspace_bytes(shape)
    if n == 0:
        raise ValueError("invalid shape")
    return torch.empty(n, dtype=torch.uint8, device=device)
