"""GPU parity of the second workload (Sec. 2 Quest page estimator under per-block selection, Eq. 2;
overlap ratios of Eq. 1 / Eq. 3): HIP library through the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2602_14209_amd.workloads import bf16_to_f32, round_to_bf16

pytestmark = pytest.mark.gpu


def _bf16(a):
    return bf16_to_f32(round_to_bf16(a.astype(np.float32)))


def _inputs(seed, B, Hq, Hkv, d, L, heavy=0.02):
    rng = np.random.default_rng(seed)
    qm = rng.standard_normal((Hq, d))
    q = _bf16(qm[None] + 0.1 * rng.standard_normal((B, Hq, d)))
    K = rng.standard_normal((L, Hkv, d))
    hot = rng.random((L, Hkv)) < heavy
    K[hot] *= 3.0
    return q, _bf16(K)


@pytest.mark.parametrize("case", [
    # dtype, Hkv, d, L, p
    ("bf16", 2, 128, 1000, 16),      # ragged last page
    ("bf16", 3, 64, 257, 2),
    ("bf16", 1, 128, 64, 1),
    ("f32", 2, 64, 100, 8),
    ("f32", 2, 128, 33, 5),
])
def test_page_summary_bit_exact(oracle_mod, case):
    import paper_2602_14209_amd.binding as mb
    from gpu_util import to_device
    dtype, Hkv, d, L, p = case
    rng = np.random.default_rng(7)
    K = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    if dtype == "bf16":
        K = _bf16(K)
    kmax, kmin = oracle_mod.page_summary(K, p)
    n_pages = kmax.shape[0]
    shape = mb.make_shape(1, Hkv, Hkv, d, L, 1, dtype)
    kd = to_device(K, dtype)
    out = torch.zeros((n_pages, Hkv, 2, d), dtype=kd.dtype, device="cuda")
    mb.check(mb.mage_page_summary(shape, p, kd, out), "mage_page_summary")
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.array_equal(got[:, :, 0, :], kmax) and np.array_equal(got[:, :, 1, :], kmin)


def _quest_case(oracle_mod, seed, B, Hq, Hkv, d, L, p, k):
    import paper_2602_14209_amd.binding as mb
    from gpu_util import check_alpha, check_index_sets, to_device
    q, K = _inputs(seed, B, Hq, Hkv, d, L)
    ref = oracle_mod.quest_select(q, K, p, k)
    shape = mb.make_shape(B, Hq, Hkv, d, L, k, "bf16")
    n_pages = L // p
    kd, qd = to_device(K, "bf16"), to_device(q, "bf16")
    summ = torch.zeros((n_pages, Hkv, 2, d), dtype=torch.bfloat16, device="cuda")
    mb.check(mb.mage_page_summary(shape, p, kd, summ), "mage_page_summary")
    nbytes = mb.mage_quest_workspace_bytes(shape, p)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    idx = torch.full((Hkv, k), -1, dtype=torch.int32, device="cuda")
    est = torch.full((Hkv, n_pages), float("nan"), dtype=torch.float32, device="cuda")
    mb.check(mb.mage_quest_select(shape, p, qd, summ, idx, est, ws), "mage_quest_select")
    torch.cuda.synchronize()
    idx, est = idx.cpu().numpy(), est.cpu().numpy()
    # one estimated score per page; the oracle's per-position scores are constant on a page
    ref_page = ref["est32"].reshape(Hkv, n_pages, p)
    assert np.all(ref_page == ref_page[:, :, :1])
    assert np.all(np.isfinite(est)) and np.all(est >= 0)
    np.testing.assert_allclose((est.astype(np.float64) * p).sum(axis=1), 1.0, atol=1e-4)
    floor = ref_page[:, :, 0].max(axis=1, keepdims=True) * 1e-6
    err = np.abs(est - ref_page[:, :, 0]) / (ref_page[:, :, 0] + floor)
    assert err.max() <= 2e-4, f"estimated score relative error {err.max():.3e}"
    check_index_sets(idx, ref["idx"], ref["est32"], L)
    # a second call without the score output gives the same set
    idx2 = torch.full((Hkv, k), -1, dtype=torch.int32, device="cuda")
    mb.check(mb.mage_quest_select(shape, p, qd, summ, idx2, None, ws), "mage_quest_select")
    torch.cuda.synchronize()
    assert np.array_equal(idx2.cpu().numpy(), idx)
    return idx, ref


@pytest.mark.parametrize("case", [
    # B, Hq, Hkv, d, L, p, k
    (8, 4, 2, 64, 960, 16, 64),
    (32, 8, 2, 128, 2048, 8, 128),       # rows of length 2d = 256
    (32, 16, 2, 128, 4096, 16, 512),     # G*B = 256: eight wavefronts in the column sums
    (5, 6, 3, 64, 300, 4, 20),           # ragged rows, few pages
    (16, 4, 4, 128, 640, 2, 2),          # one page selected
    (4, 2, 2, 64, 70, 1, 9),             # one position per page
])
def test_quest_select_small(oracle_mod, case):
    B, Hq, Hkv, d, L, p, k = case
    _quest_case(oracle_mod, 100 + p + k, B, Hq, Hkv, d, L, p, k)


def test_quest_page_size_one_is_mage_select(oracle_mod):
    """p = 1: the bound is q.k, so the estimator must return what mage_select returns."""
    import paper_2602_14209_amd.binding as mb
    from gpu_util import Problem
    B, Hq, Hkv, d, L, k = 16, 8, 2, 128, 1024, 64
    q, K = _inputs(5, B, Hq, Hkv, d, L)
    idx_q, ref = _quest_case(oracle_mod, 5, B, Hq, Hkv, d, L, 1, k)
    prob = Problem(q, K, K, None, None, k, "bf16")
    idx_s, _ = prob.select()
    assert np.array_equal(idx_s, ref["idx"]) or np.array_equal(idx_s, idx_q)
    assert np.array_equal(oracle_mod.select(q, K, k)["idx"], ref["idx"])


def test_quest_select_headline_shape(oracle_mod):
    """c4 geometry (L = 131072, d = 128, G*B = 128), p = 16, k = 512."""
    _quest_case(oracle_mod, 1004, 32, 32, 8, 128, 131072, 16, 512)


def test_quest_rejects_unsupported(oracle_mod):
    import paper_2602_14209_amd.binding as mb
    fake = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    idx = torch.zeros((2, 32), dtype=torch.int32, device="cuda")
    s = mb.make_shape(8, 4, 2, 64, 1000, 32, "bf16")
    assert mb.mage_quest_workspace_bytes(s, 16) == 0          # L % p != 0
    assert mb.mage_quest_select(s, 16, fake, fake, idx, None, fake) == -3
    s = mb.make_shape(8, 4, 2, 64, 1024, 30, "bf16")
    assert mb.mage_quest_select(s, 16, fake, fake, idx, None, fake) == -3    # k % p != 0
    s = mb.make_shape(8, 4, 2, 64, 1024, 32, "f32")
    assert mb.mage_quest_select(s, 16, fake, fake, idx, None, fake) == -3    # fp32
    s = mb.make_shape(8, 4, 2, 64, 1024, 32, "bf16")
    assert mb.mage_quest_select(s, 0, fake, fake, idx, None, fake) == -2
    assert mb.mage_quest_select(s, 16, fake, fake, idx, None, fake) == -4    # workspace too small


def test_set_overlap_matches_oracle(oracle_mod):
    import paper_2602_14209_amd.binding as mb
    rng = np.random.default_rng(9)
    Hkv, B, k, L = 3, 7, 200, 5000
    block = np.stack([np.sort(rng.choice(L, k, replace=False)) for _ in range(Hkv)]).astype(np.int32)
    # per-token sets: partly shared with the block set, in arbitrary order
    token = np.empty((B, Hkv, k), np.int32)
    for qi in range(B):
        for h in range(Hkv):
            keep = rng.choice(block[h], rng.integers(0, k + 1), replace=False)
            rest = rng.choice(np.setdiff1d(np.arange(L), block[h]), k - keep.size, replace=False)
            token[qi, h] = rng.permutation(np.concatenate([keep, rest]))
    a, b = torch.from_numpy(block).cuda(), torch.from_numpy(token).cuda()
    out = torch.full((B * Hkv,), float("nan"), dtype=torch.float32, device="cuda")
    mb.check(mb.mage_set_overlap(a, b, B * Hkv, k, Hkv, out), "mage_set_overlap")      # Eq. 1 layout
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(B, Hkv)
    for qi in range(B):
        for h in range(Hkv):
            assert got[qi, h] == np.float32(oracle_mod.overlap(block[h], token[qi, h]))
    out2 = torch.full((Hkv,), float("nan"), dtype=torch.float32, device="cuda")
    mb.check(mb.mage_set_overlap(a, a, Hkv, k, Hkv, out2), "mage_set_overlap")          # Eq. 3 layout, identical sets
    torch.cuda.synchronize()
    assert np.all(out2.cpu().numpy() == 1.0)
    assert mb.mage_set_overlap(a, b, 0, k, Hkv, out) == -2
    assert mb.mage_set_overlap(a, None, 3, k, 3, out) == -1
