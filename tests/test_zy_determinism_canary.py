"""Run-to-run determinism and guard zones of every entry point, on the GPU:

* determinism: every entry point called twice on the same inputs gives bitwise identical outputs (no
  result depends on the order in which workgroups or atomics happen to run);
* guard zones: outputs and workspace are carved out of larger buffers filled with a pattern; after the
  calls nothing outside the carved region has changed (no kernel writes past what the header says it
  owns), for shapes with ragged tails.
"""
import numpy as np
import pytest
import torch

from paper_2602_14209_amd import binding as mb
from paper_2602_14209_amd.workloads import Workload, make_layer

pytestmark = pytest.mark.gpu
GUARD = 4096          # elements on each side


def _guarded(shape, dtype, fill):
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * GUARD,), fill, dtype=dtype, device="cuda")
    return buf, buf[GUARD:GUARD + n].view(*shape)


def _intact(buf, n, fill):
    head, tail = buf[:GUARD], buf[GUARD + n:]
    if buf.dtype.is_floating_point and np.isnan(fill):
        return bool(torch.isnan(head).all()) and bool(torch.isnan(tail).all())
    return bool((head == fill).all()) and bool((tail == fill).all())


CASES = [
    # name, dtype, Hq, Hkv, d, L, B, k
    ("g1", "bf16", 8, 2, 128, 1000, 32, 100),
    ("g2", "bf16", 14, 2, 64, 777, 5, 65),
    ("g3", "bf16", 4, 4, 128, 4097, 32, 512),
    ("g4", "f32", 6, 2, 64, 700, 7, 33),
]


@pytest.mark.parametrize("case", CASES)
def test_twice_bitwise_equal_and_guards_intact(case):
    from gpu_util import to_device
    name, dtype, Hq, Hkv, d, L, B, k = case
    w = Workload(name, dtype, Hq=Hq, Hkv=Hkv, d=d, L=L, B=B, ks=(k,), T=2, heavy_frac=0.02, heavy_scale=3.0)
    x = make_layer(w, 7100 + L, steps=2)
    shape = mb.make_shape(B, Hq, Hkv, d, L, k, dtype)
    q1, q2 = to_device(x["q"][0], dtype), to_device(x["q"][1], dtype)
    kc, vc = to_device(x["k_cache"], dtype), to_device(x["v_cache"], dtype)
    kb, vb = to_device(x["k_blk"][1], dtype), to_device(x["v_blk"][1], dtype)
    nan = float("nan")
    ws_bytes = mb.mage_workspace_bytes(shape)
    results = []
    for rep in range(2):
        ws_buf = torch.full((ws_bytes + 2 * GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
        ws = ws_buf[GUARD:GUARD + ws_bytes]
        out_b, out = _guarded((B, Hq, d), torch.float32, nan)
        lse_b, lse = _guarded((B, Hq), torch.float32, nan)
        idx_b, idx = _guarded((Hkv, k), torch.int32, -7)
        al_b, alpha = _guarded((Hkv, L), torch.float32, nan)
        pb_b, pbar = _guarded((Hq, L), torch.float32, nan)
        got = {}
        mb.check(mb.mage_select(shape, q1, kc, idx, alpha, ws), "mage_select")
        got["select_idx"], got["select_alpha"] = idx.clone(), alpha.clone()
        mb.check(mb.mage_block_probs(shape, q1, kc, pbar, ws), "mage_block_probs")
        got["pbar"] = pbar.clone()
        mb.check(mb.mage_exact_attn(shape, q1, kc, vc, kb, vb, out, lse, ws), "mage_exact_attn")
        got["exact_out"], got["exact_lse"] = out.clone(), lse.clone()
        mb.check(mb.mage_step1(shape, q1, kc, vc, kb, vb, out, lse, idx, alpha, ws), "mage_step1")
        got["step1_out"], got["step1_idx"], got["step1_alpha"] = out.clone(), idx.clone(), alpha.clone()
        mb.check(mb.mage_sparse_attn(shape, q2, kc, vc, idx, kb, vb, out, lse, ws), "mage_sparse_attn")
        got["sparse_out"], got["sparse_lse"] = out.clone(), lse.clone()
        torch.cuda.synchronize()
        assert (ws_buf[:GUARD] == 0x5A).all() and (ws_buf[GUARD + ws_bytes:] == 0x5A).all(), "workspace guard"
        assert _intact(out_b, out.numel(), nan), "out guard"
        assert _intact(lse_b, lse.numel(), nan), "lse guard"
        assert _intact(idx_b, idx.numel(), -7), "idx guard"
        assert _intact(al_b, alpha.numel(), nan), "alpha guard"
        assert _intact(pb_b, pbar.numel(), nan), "pbar guard"
        results.append({n: t.cpu() for n, t in got.items()})
    for n in results[0]:
        a, b = results[0][n], results[1][n]
        assert torch.equal(a.view(torch.int32), b.view(torch.int32)), f"{n} differs between two runs"
