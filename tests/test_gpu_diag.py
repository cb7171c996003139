"""The measurement aids (mage_diag_*) do what include/mage.h says, through the C ABI: bench.py's floors and
ceilings, and the profiler's byte calibration, rest on them."""
import numpy as np
import pytest
import torch

from paper_2602_14209_amd import binding as mb

pytestmark = pytest.mark.gpu


def test_copy_is_exact_and_leaves_a_short_tail_alone():
    n = (1 << 20) + 16 + 5                      # whole 16-byte units are copied, a tail shorter than 16 bytes is not
    g = torch.Generator(device="cuda").manual_seed(3)
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda", generator=g)
    dst = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    mb.check(mb.mage_diag_copy(dst, src), "mage_diag_copy")
    torch.cuda.synchronize()
    whole = n // 16 * 16
    assert torch.equal(dst[:whole], src[:whole])
    assert bool((dst[whole:] == 7).all())


def test_read_and_empty_and_gather_run():
    src = torch.ones(1 << 22, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    mb.check(mb.mage_diag_read(src, sink), "mage_diag_read")
    mb.check(mb.mage_diag_empty(), "mage_diag_empty")
    Hkv, d, L, k, n_seq = 2, 128, 3000, 100, 3
    shape = mb.make_shape(32, 8, Hkv, d, L, k, "bf16")
    kc = torch.zeros((n_seq, L, Hkv, d), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    rng = np.random.default_rng(5)
    idx = np.stack([np.sort(rng.choice(L, k, replace=False)) for _ in range(n_seq * Hkv)]).reshape(n_seq, Hkv, k).astype(np.int32)
    mb.check(mb.mage_diag_gather(shape, n_seq, kc, vc, torch.from_numpy(idx).cuda(), sink), "mage_diag_gather")
    torch.cuda.synchronize()
    assert int(sink.abs().sum()) == 0           # the sinks are "practically never written": all-ones / all-zero data never hits the magic value


def test_chase_follows_the_chain():
    n, hops, start = 1 << 16, 1000, 17
    rng = np.random.default_rng(11)
    chain = rng.integers(0, n, size=n, dtype=np.int64).astype(np.int32)
    want = start
    for _ in range(hops):
        want = int(chain[want])
    out = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    mb.check(mb.mage_diag_chase(torch.from_numpy(chain).cuda(), start, hops, out), "mage_diag_chase")
    torch.cuda.synchronize()
    assert int(out[0]) == want


@pytest.mark.parametrize("mode", [1, 2])
def test_merge_adds_the_four_partials_on_every_launch(mode):
    n_groups = 16
    g = torch.Generator(device="cuda").manual_seed(mode)
    src = torch.rand(4 * n_groups * 2048, dtype=torch.float32, device="cuda", generator=g)
    part = torch.zeros_like(src)
    out = torch.zeros(n_groups * 2048, dtype=torch.float32, device="cuda")
    cnt = torch.zeros(n_groups, dtype=torch.int32, device="cuda")
    p = src.clone().view(-1, 4)
    p[:, 0] += 1.0                               # what every workgroup writes: src with 1 added to the first of every four floats
    p = p.view(n_groups, 4, 2048)
    want = ((p[:, 0] + p[:, 1]) + p[:, 2]) + p[:, 3]
    for launch in range(3):                      # the counters keep counting: the last arriver of every launch merges
        out.zero_()
        mb.check(mb.mage_diag_merge(mode, n_groups, part, cnt, out, src), "mage_diag_merge")
        torch.cuda.synchronize()
        assert torch.equal(part.view(n_groups, 4, 2048), p)
        assert torch.equal(out.view(n_groups, 2048), want), f"launch {launch}"
        assert bool((cnt == 4 * (launch + 1)).all())


def test_stamps_increase_along_a_stream():
    hz = mb.mage_diag_stamp_hz()
    assert hz > 0
    st = torch.zeros(3, dtype=torch.int64, device="cuda")
    src = torch.ones(1 << 26, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    mb.check(mb.mage_diag_stamp(st[0:1]), "mage_diag_stamp")
    mb.check(mb.mage_diag_read(src, sink), "mage_diag_read")
    mb.check(mb.mage_diag_stamp(st[1:2]), "mage_diag_stamp")
    mb.check(mb.mage_diag_stamp(st[2:3]), "mage_diag_stamp")
    torch.cuda.synchronize()
    t = st.cpu().numpy()
    assert t[0] < t[1] <= t[2]
    read_us = (t[1] - t[0]) / hz * 1e6
    assert 1.0 < read_us < 5000.0, read_us       # 64 MiB at a few TB/s, plus two launches
