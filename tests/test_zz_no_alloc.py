"""mage_select_static (selection on the library's static scratch array: no workspace argument, no
allocation) against mage_select on the same inputs, through the C ABI: two calls in a row, the second
on a smaller problem, so that what the first call left in the shared scratch array must not matter."""
import numpy as np
import pytest
import torch

from paper_2602_14209_amd import binding as mb
from paper_2602_14209_amd.workloads import Workload, make_layer

pytestmark = pytest.mark.gpu


def _both(w, seed, k):
    from gpu_util import to_device
    x = make_layer(w, seed, steps=1)
    shape = mb.make_shape(w.B, w.Hq, w.Hkv, w.d, w.L, k, w.dtype)
    q1, kc = to_device(x["q"][0], w.dtype), to_device(x["k_cache"], w.dtype)
    ws = mb.alloc_workspace(shape)
    idx_a = torch.full((w.Hkv, k), -1, dtype=torch.int32, device="cuda")
    idx_b = torch.full((w.Hkv, k), -2, dtype=torch.int32, device="cuda")
    al_a = torch.full((w.Hkv, w.L), float("nan"), dtype=torch.float32, device="cuda")
    al_b = torch.full((w.Hkv, w.L), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    print(f"[no-alloc] {w.name} dtype={w.dtype} L={w.L} Hq={w.Hq} Hkv={w.Hkv} d={w.d} B={w.B} k={k} seed={seed}", flush=True)
    mb.check(mb.mage_select_static(shape, q1, kc, idx_b, al_b), "mage_select_static")
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before      # torch's allocator was not asked either
    mb.check(mb.mage_select(shape, q1, kc, idx_a, al_a, ws), "mage_select")
    torch.cuda.synchronize()
    # same kernels, same launch plan: the index sets are identical, bit for bit, and so is alpha
    assert torch.equal(idx_a, idx_b), f"{w.name}: index sets differ"
    assert torch.equal(al_a.view(torch.int32), al_b.view(torch.int32)), f"{w.name}: alpha differs"
    # and without the alpha output (alpha then lives in the scratch array)
    idx_c = torch.full((w.Hkv, k), -3, dtype=torch.int32, device="cuda")
    mb.check(mb.mage_select_static(shape, q1, kc, idx_c, None), "mage_select_static")
    torch.cuda.synchronize()
    assert torch.equal(idx_a, idx_c)
    return x, idx_b.cpu().numpy(), al_b.cpu().numpy()


def test_two_calls_in_a_row_second_smaller(oracle_mod):
    from gpu_util import check_alpha, check_index_sets
    big = Workload("na_big", "bf16", Hq=32, Hkv=8, d=128, L=40000, B=32, ks=(512,), T=1, heavy_frac=0.01, heavy_scale=4.0)
    small = Workload("na_small", "bf16", Hq=14, Hkv=2, d=64, L=777, B=5, ks=(65,), T=1, heavy_frac=0.02, heavy_scale=3.0)
    tiny32 = Workload("na_f32", "f32", Hq=6, Hkv=2, d=64, L=300, B=7, ks=(33,), T=1)
    for w, seed in ((big, 8101), (small, 8102), (tiny32, 8103)):
        x, idx, alpha = _both(w, seed, w.k)
        ref = oracle_mod.select(x["q"][0], x["k_cache"], w.k)
        check_alpha(alpha, ref["alpha32"])
        check_index_sets(idx, ref["idx"], ref["alpha32"], w.L)


def test_too_large_for_the_static_array_is_rejected():
    cap = mb.mage_static_scratch_bytes()
    assert cap == 8 << 20
    shape = mb.make_shape(32, 32, 8, 128, 1 << 20, 512, "bf16")       # alpha alone is 32 MiB
    assert mb.mage_workspace_bytes(shape) > cap
    fake = torch.zeros(64, dtype=torch.int32, device="cuda")
    rc = mb.mage_select_static(shape, fake, fake, fake, None)
    assert rc == -7 and "static" in mb.status_string(rc)
