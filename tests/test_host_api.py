"""Host-side checks that need no GPU: the C-ABI library loads, exports every declared symbol,
validates its arguments before launching anything, and sizes its workspace consistently."""
import ctypes
import os
import re

import pytest

from paper_2602_14209_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mage_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = mb.lib()
    names = _declared_symbols()
    assert set(names) == set(mb.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.mage_version() >= 100


def test_status_strings():
    for code in range(0, -8, -1):
        s = mb.status_string(code)
        assert s and s != "unknown status"
    assert mb.status_string(-99) == "unknown status"


def test_workspace_bytes():
    s = mb.make_shape(32, 32, 8, 128, 131072, 512, "bf16")
    n = mb.mage_workspace_bytes(s)
    assert n >= 8 * 131072 * 4          # holds alpha[Hkv,L]
    assert n < 1 << 30
    assert mb.mage_workspace_bytes(mb.make_shape(32, 32, 8, 128, 131072, 0, "bf16")) == 0
    assert mb.mage_workspace_bytes(mb.make_shape(32, 30, 8, 128, 131072, 512, "bf16")) == 0
    assert mb.mage_workspace_bytes(mb.make_shape(4, 4, 1, 64, 2048, 64, "f32")) > 0


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), -2), (dict(Hq=0), -2), (dict(Hkv=0), -2), (dict(L=0), -2), (dict(k=0), -2),
    (dict(Hq=30), -2),              # Hq % Hkv != 0
    (dict(k=5000, L=4096), -2),     # k > L
    (dict(d=96), -3), (dict(dtype=7), -3), (dict(L=(1 << 30) + 1), -3),
    (dict(B=1 << 18, Hq=64), -3),                       # B*G > 2^20
    (dict(B=70000, Hq=8), -3),                          # B*G fits, B*B*G >= 2^32
    (dict(Hq=1 << 23, Hkv=1 << 23, d=64), -3),          # Hkv*d >= 2^29
])
def test_argument_validation_happens_before_any_launch(kw, code):
    base = dict(B=32, Hq=32, Hkv=8, d=128, L=4096, k=512, dtype=1)
    base.update(kw)
    s = mb.make_shape(**base)
    fake = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    L = mb.lib()
    assert L.mage_select(ctypes.byref(s), fake, fake, fake, None, fake, 1 << 40, None) == code
    assert L.mage_sparse_attn(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == code
    assert L.mage_step1(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, fake, None, fake, 1 << 40, None) == code
    assert L.mage_compact(ctypes.byref(s), fake, fake, fake, fake, fake, None) == code
    assert L.mage_sparse_attn_compact(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == code
    assert L.mage_sparse_attn_batched(ctypes.byref(s), 2, fake, fake, fake, fake, fake, fake, fake, None, None) == code
    if "k" not in kw:
        assert L.mage_exact_attn(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == code


def test_null_alignment_and_workspace_errors():
    s = mb.make_shape(32, 32, 8, 128, 4096, 512, "bf16")
    L = mb.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    big = 1 << 40
    assert L.mage_select(None, fake, fake, fake, None, fake, big, None) == -1
    assert L.mage_select(ctypes.byref(s), None, fake, fake, None, fake, big, None) == -1
    assert L.mage_select(ctypes.byref(s), fake, fake, None, None, fake, big, None) == -1
    assert L.mage_select(ctypes.byref(s), odd, fake, fake, None, fake, big, None) == -6
    assert L.mage_select(ctypes.byref(s), fake, fake, fake, None, fake, 16, None) == -4
    assert L.mage_select(ctypes.byref(s), fake, fake, fake, None, None, 0, None) == -4
    assert L.mage_exact_attn(ctypes.byref(s), fake, fake, fake, fake, None, fake, None, fake, big, None) == -1
    assert L.mage_exact_attn(ctypes.byref(s), fake, fake, odd, fake, fake, fake, None, fake, big, None) == -6
    assert L.mage_exact_attn(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, fake, 16, None) == -4
    assert L.mage_sparse_attn(ctypes.byref(s), fake, fake, fake, None, fake, fake, fake, None, fake, big, None) == -1
    assert L.mage_compact(ctypes.byref(s), fake, fake, None, fake, fake, None) == -1
    assert L.mage_compact(ctypes.byref(s), fake, odd, fake, fake, fake, None) == -6
    assert L.mage_sparse_attn_compact(ctypes.byref(s), None, fake, fake, fake, fake, fake, None, None, 0, None) == -1
    assert L.mage_sparse_attn_batched(ctypes.byref(s), 0, fake, fake, fake, fake, fake, fake, fake, None, None) == -2
    assert L.mage_sparse_attn_batched(ctypes.byref(s), 2, fake, fake, fake, None, fake, fake, fake, None, None) == -1
    sf32 = mb.make_shape(32, 32, 8, 128, 4096, 512, "f32")
    assert L.mage_sparse_attn_batched(ctypes.byref(sf32), 2, fake, fake, fake, fake, fake, fake, fake, None, None) == -3
    many_heads = mb.make_shape(32, 512, 512, 128, 4096, 512, "bf16")      # (n_seq*Hkv + 8)*Hkv >= 2^32
    assert L.mage_sparse_attn_batched(ctypes.byref(many_heads), 60000, fake, fake, fake, fake, fake, fake, fake, None, None) == -3
    assert L.mage_sparse_attn_batched(ctypes.byref(s), 65536, fake, fake, fake, fake, fake, fake, fake, None, None) == -2
    assert L.mage_step1(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, None, None, fake, big, None) == -1
    assert L.mage_step1(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, fake, None, fake, 16, None) == -4
    # the bf16 sparse step keeps its partials on chip and needs no workspace; the fp32 one does
    sf = mb.make_shape(32, 32, 8, 128, 4096, 512, "f32")
    assert L.mage_sparse_attn(ctypes.byref(sf), fake, fake, fake, fake, fake, fake, fake, None, fake, 16, None) == -4
    assert L.mage_sparse_attn(ctypes.byref(s), fake, fake, odd, fake, fake, fake, fake, None, None, 0, None) == -6


def test_second_workload_argument_validation():
    """Page estimator and overlap ratio: every argument error is reported before anything is launched."""
    L = mb.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    big = 1 << 40
    s = mb.make_shape(32, 32, 8, 128, 4096, 512, "bf16")
    assert L.mage_page_summary(ctypes.byref(s), 0, fake, fake, None) == -2
    assert L.mage_page_summary(ctypes.byref(s), 16, None, fake, None) == -1
    assert L.mage_page_summary(ctypes.byref(s), 16, fake, odd, None) == -6
    assert L.mage_page_summary(None, 16, fake, fake, None) == -1
    assert mb.mage_quest_workspace_bytes(s, 16) > 0
    assert mb.mage_quest_workspace_bytes(s, 0) == 0
    assert mb.mage_quest_workspace_bytes(s, 24) == 0                       # L % p != 0
    assert mb.mage_quest_workspace_bytes(mb.make_shape(32, 32, 8, 128, 4096, 500, "bf16"), 16) == 0   # k % p != 0
    assert mb.mage_quest_workspace_bytes(mb.make_shape(32, 32, 8, 128, 4096, 512, "f32"), 16) == 0
    assert L.mage_quest_select(ctypes.byref(s), 16, None, fake, fake, None, fake, big, None) == -1
    assert L.mage_quest_select(ctypes.byref(s), 16, fake, fake, None, None, fake, big, None) == -1
    assert L.mage_quest_select(ctypes.byref(s), 16, odd, fake, fake, None, fake, big, None) == -6
    assert L.mage_quest_select(ctypes.byref(s), 16, fake, fake, fake, None, fake, 16, None) == -4
    assert L.mage_quest_select(ctypes.byref(s), 24, fake, fake, fake, None, fake, big, None) == -3
    assert L.mage_quest_select(ctypes.byref(s), -1, fake, fake, fake, None, fake, big, None) == -2
    assert L.mage_set_overlap(None, fake, 4, 8, 4, fake, None) == -1
    assert L.mage_set_overlap(fake, fake, 0, 8, 1, fake, None) == -2
    assert L.mage_set_overlap(fake, fake, 4, 0, 4, fake, None) == -2
    assert L.mage_set_overlap(fake, fake, 4, 8, 5, fake, None) == -2          # more `a` rows than rows


def test_block_probs_argument_validation():
    """mage_block_probs: argument errors are reported before anything is launched."""
    L = mb.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    big = 1 << 40
    s = mb.make_shape(32, 32, 8, 128, 4096, 512, "bf16")
    assert L.mage_block_probs(None, fake, fake, fake, fake, big, None) == -1
    assert L.mage_block_probs(ctypes.byref(s), fake, fake, None, fake, big, None) == -1
    assert L.mage_block_probs(ctypes.byref(s), None, fake, fake, fake, big, None) == -1
    assert L.mage_block_probs(ctypes.byref(s), fake, fake, odd, fake, big, None) == -6
    assert L.mage_block_probs(ctypes.byref(s), fake, fake, fake, fake, 16, None) == -4
    bad = mb.make_shape(32, 32, 8, 96, 4096, 512, "bf16")
    assert L.mage_block_probs(ctypes.byref(bad), fake, fake, fake, fake, big, None) == -3
    wide = mb.make_shape(128, 32, 8, 128, 4096, 512, "bf16")       # B*G = 512 rows per KV head
    assert L.mage_block_probs(ctypes.byref(wide), fake, fake, fake, fake, big, None) == -3


def test_combined_calls_validate_everything_before_their_first_launch():
    """mage_step1 (fp32: attention, then selection) and mage_quest_select (query split, then selection over
    pages) must report what their LATER stage would reject before the earlier stage launches anything:
    with no GPU in this process a launch would come back as MAGE_ERR_HIP (-5) instead."""
    L = mb.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    big = 1 << 40
    sf = mb.make_shape(32, 32, 8, 128, 4096, 512, "f32")
    # attention arguments are fine; alpha_out (selection's) is misaligned / the workspace is too small for selection
    assert L.mage_step1(ctypes.byref(sf), fake, fake, fake, fake, fake, fake, None, fake, odd, fake, big, None) == -6
    assert L.mage_step1(ctypes.byref(sf), fake, fake, fake, None, None, fake, None, fake, None, fake, 16, None) == -4
    wide = mb.make_shape(128, 32, 8, 128, 4096, 512, "bf16")      # B*G = 512 rows per KV head: selection unsupported
    assert mb.mage_quest_workspace_bytes(wide, 16) > 0
    assert L.mage_quest_select(ctypes.byref(wide), 16, fake, fake, fake, None, fake, big, None) == -3
    assert L.mage_step1(ctypes.byref(wide), fake, fake, fake, fake, fake, fake, None, fake, None, fake, big, None) == -3
    assert L.mage_select(ctypes.byref(wide), fake, fake, fake, None, fake, big, None) == -3
    # ... while the attention calls accept that geometry, which is why mage_workspace_bytes() is not 0 for it
    assert mb.mage_workspace_bytes(wide) > 0


def test_static_scratch_entry_point_rejects_before_touching_the_device():
    """mage_select_static: shape and size errors come back without any device call (none is possible here)."""
    L = mb.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    assert mb.mage_static_scratch_bytes() == 8 << 20
    ok = mb.make_shape(32, 32, 8, 128, 131072, 512, "bf16")          # the headline shape fits
    huge = mb.make_shape(32, 32, 8, 128, 1 << 20, 512, "bf16")
    assert L.mage_select_static(ctypes.byref(huge), fake, fake, fake, None, None) == -7
    assert L.mage_select_static(ctypes.byref(ok), None, fake, fake, None, None) == -1
    assert L.mage_select_static(ctypes.byref(ok), fake, fake, None, None, None) == -1
    assert L.mage_select_static(ctypes.byref(ok), odd, fake, fake, None, None) == -6
    assert L.mage_select_static(ctypes.byref(mb.make_shape(32, 30, 8, 128, 4096, 512, "bf16")), fake, fake, fake, None, None) == -2
    assert L.mage_select_static(None, fake, fake, fake, None, None) == -1


def test_measurement_aids_validate_their_arguments():
    L = mb.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    s = mb.make_shape(32, 32, 8, 128, 4096, 512, "bf16")
    assert L.mage_diag_stamp(None, None) == -1
    assert L.mage_diag_stamp(odd, None) == -6
    assert L.mage_diag_chase(None, 16, 0, 4, fake, None) == -1
    assert L.mage_diag_chase(fake, 16, 16, 4, fake, None) == -2
    assert L.mage_diag_chase(fake, 16, 0, 0, fake, None) == -2
    assert L.mage_diag_read(None, 1024, fake, None) == -1
    assert L.mage_diag_read(odd, 1024, fake, None) == -6
    assert L.mage_diag_read(fake, 8, fake, None) == -2
    assert L.mage_diag_copy(fake, None, 1024, None) == -1
    assert L.mage_diag_copy(odd, fake, 1024, None) == -6
    assert L.mage_diag_merge(3, 4, fake, fake, fake, fake, None) == -2
    assert L.mage_diag_merge(1, 0, fake, fake, fake, fake, None) == -2
    assert L.mage_diag_merge(1, 4, fake, None, fake, fake, None) == -1
    assert L.mage_diag_merge(1, 4, odd, fake, fake, fake, None) == -6
    assert L.mage_diag_gather(ctypes.byref(s), 0, fake, fake, fake, fake, None) == -2
    assert L.mage_diag_gather(ctypes.byref(s), 2, fake, None, fake, fake, None) == -1
    sf = mb.make_shape(32, 32, 8, 128, 4096, 512, "f32")                # 512-byte rows
    assert L.mage_diag_gather(ctypes.byref(sf), 2, fake, fake, fake, fake, None) == -3


def test_binding_argument_counts_match_the_header():
    """Every prototype of include/mage.h has as many parameters as the binding marshals."""
    text = open(os.path.join(ROOT, "include", "mage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    protos = re.findall(r"\b(mage_[a-z0-9_]+)\s*\(([^;{]*?)\)\s*;", text, flags=re.S)
    assert len(protos) == len(mb.EXPORTS)
    lib = mb.lib()
    for name, params in protos:
        params = params.strip()
        n = 0 if params in ("", "void") else params.count(",") + 1
        argtypes = getattr(lib, name).argtypes
        assert argtypes is not None or n == 0, name
        assert len(argtypes or []) == n, (name, n, len(argtypes or []))


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU only" in r.stderr and r.stdout.strip() == ""
