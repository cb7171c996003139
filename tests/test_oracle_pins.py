"""Pins of the CPU oracle against things other than itself.

The paper (arxiv 2602.14209) prints no worked numeric example for any kernel, so
the oracle is pinned to library routines on special cases (scipy softmax, numpy
stable argsort, torch scaled_dot_product_attention), closed forms, and invariants
that the definitions in Alg. 1 / Eq. 2 / Eq. 5 imply.
"""
import numpy as np
import pytest
import torch
from scipy.special import softmax as sp_softmax

pytestmark = pytest.mark.filterwarnings("ignore")


def _rng(seed):
    return np.random.default_rng(seed)


def _brute_topk(score, k):
    order = np.argsort(-score.astype(np.float64), kind="stable")   # ties keep the smaller index first
    return np.sort(order[:k]).astype(np.int32)


# --------------------------------------------------------------------------- top-k
def test_topk_bruteforce_all_k(oracle_mod):
    rng = _rng(0)
    for L in (1, 2, 7, 33, 64):
        a = rng.random(L).astype(np.float32)
        for k in range(1, L + 1):
            assert np.array_equal(oracle_mod.topk(a, k), _brute_topk(a, k)), (L, k)


def test_topk_ties_lowest_index(oracle_mod):
    rng = _rng(1)
    for L in (16, 50, 64):
        a = (rng.integers(0, 4, L) / 4.0).astype(np.float32)      # many exact ties
        for k in range(1, L + 1):
            assert np.array_equal(oracle_mod.topk(a, k), _brute_topk(a, k)), (L, k)
    a = np.full(40, 0.025, np.float32)
    for k in (1, 5, 40):
        assert np.array_equal(oracle_mod.topk(a, k), np.arange(k, dtype=np.int32))


def test_topk_rejects_bad_k(oracle_mod):
    a = np.ones(8, np.float32)
    with pytest.raises(RuntimeError):
        oracle_mod.topk(a, 9)
    with pytest.raises(RuntimeError):
        oracle_mod.topk(a, 0)


# ----------------------------------------------------------------------- selection
def test_select_single_row_is_textbook_softmax(oracle_mod):
    # G = B = 1: Eq. 5 collapses to one softmax row; compare with scipy + stable argsort.
    rng = _rng(2)
    for d, L in ((64, 97), (128, 300)):
        q = rng.standard_normal((1, 1, d)).astype(np.float32)
        K = rng.standard_normal((L, 1, d)).astype(np.float32)
        logits = (K[:, 0, :].astype(np.float64) @ q[0, 0].astype(np.float64)) / np.sqrt(d)
        want = sp_softmax(logits)
        r = oracle_mod.select(q, K, 11)
        np.testing.assert_allclose(r["alpha"][0], want, rtol=1e-12, atol=0)
        np.testing.assert_allclose(r["pbar"][0], want, rtol=1e-12, atol=0)
        assert np.array_equal(r["idx"][0], _brute_topk(want.astype(np.float32), 11))


def test_select_block_and_group_average(oracle_mod):
    # Eq. 2 / Eq. 5: mean over the B tokens, then over the G heads of the group,
    # each row a scipy softmax.  Hq=6, Hkv=2 exercises the contiguous group map.
    rng = _rng(3)
    B, Hq, Hkv, d, L = 3, 6, 2, 64, 130
    G = Hq // Hkv
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    K = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    r = oracle_mod.select(q, K, 20)
    for g in range(Hq):
        h = g // G
        rows = [sp_softmax(K[:, h, :].astype(np.float64) @ q[b, g].astype(np.float64) / np.sqrt(d)) for b in range(B)]
        np.testing.assert_allclose(r["pbar"][g], np.mean(rows, axis=0), rtol=1e-12)
    for h in range(Hkv):
        np.testing.assert_allclose(r["alpha"][h], r["pbar"][h * G:(h + 1) * G].mean(axis=0), rtol=1e-12)
        assert np.array_equal(r["idx"][h], _brute_topk(r["alpha"][h].astype(np.float32), 20))
    assert r["alpha32"].dtype == np.float32
    assert np.array_equal(r["alpha32"], r["alpha"].astype(np.float32))


def test_select_sums_to_one(oracle_mod):
    rng = _rng(4)
    q = rng.standard_normal((4, 8, 64)).astype(np.float32) * 2
    K = rng.standard_normal((513, 2, 64)).astype(np.float32) * 2
    r = oracle_mod.select(q, K, 7)
    assert np.max(np.abs(r["pbar"].sum(axis=1) - 1)) < 1e-12
    assert np.max(np.abs(r["alpha"].sum(axis=1) - 1)) < 1e-12
    assert (r["alpha"] >= 0).all()


def test_select_uniform_cases(oracle_mod):
    # all keys equal, or Q1 = 0  =>  alpha == 1/L exactly-ish and S = {0..k-1} (tie-break)
    rng = _rng(5)
    B, Hq, Hkv, d, L, k = 2, 4, 2, 64, 77, 9
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    K = np.broadcast_to(rng.standard_normal((1, Hkv, d)).astype(np.float32), (L, Hkv, d)).copy()
    r = oracle_mod.select(q, K, k)
    np.testing.assert_allclose(r["alpha"], 1.0 / L, rtol=1e-13)
    assert np.array_equal(r["idx"], np.tile(np.arange(k, dtype=np.int32), (Hkv, 1)))
    K2 = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    r = oracle_mod.select(np.zeros_like(q), K2, k)
    np.testing.assert_allclose(r["alpha"], 1.0 / L, rtol=1e-13)
    assert np.array_equal(r["idx"], np.tile(np.arange(k, dtype=np.int32), (Hkv, 1)))


def test_select_duplicate_rows_tie_goes_to_lower_index(oracle_mod):
    rng = _rng(6)
    B, Hq, Hkv, d, L = 1, 1, 1, 64, 60       # one softmax row: monotone in the logits
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    K = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    base = oracle_mod.select(q, K, 1)["alpha"][0]
    order = np.argsort(-base, kind="stable")
    k = 5
    j_lo, j_hi = sorted((int(order[k - 1]), int(order[k + 6])))
    row = K[order[k - 1]].copy()
    K[j_lo] = row
    K[j_hi] = row                            # two identical rows tied for rank k; the k-1 rows ranked
                                             # above them stay above (only the normaliser changed)
    r = oracle_mod.select(q, K, k)
    assert r["alpha32"][0, j_lo] == r["alpha32"][0, j_hi]
    assert j_lo in r["idx"][0] and j_hi not in r["idx"][0]
    r2 = oracle_mod.select(q, K, k + 1)
    assert j_lo in r2["idx"][0] and j_hi in r2["idx"][0]


def test_select_planted_spike_and_group_map(oracle_mod):
    # heads (0,1) query along a, heads (2,3) along b, a orthogonal to b; all keys zero except one
    # spike per KV head.  KV head 0 carries a spike along b, KV head 1 a spike along a.  Under the
    # contiguous map group(0)={0,1} sees logit 0 everywhere => alpha uniform; an interleaved map would not.
    d, L, B = 64, 40, 2
    a = np.zeros(d, np.float32); a[0] = 8.0
    b = np.zeros(d, np.float32); b[1] = 8.0
    q = np.stack([a, a, b, b])[None].repeat(B, axis=0)           # [B,4,d]
    K = np.zeros((L, 2, d), np.float32)
    K[7, 0] = b
    K[23, 1] = a
    r = oracle_mod.select(q, K, 1)
    np.testing.assert_allclose(r["alpha"][0], 1.0 / L, rtol=1e-13)
    assert r["idx"][0, 0] == 0
    np.testing.assert_allclose(r["alpha"][1], 1.0 / L, rtol=1e-13)
    # now aligned spikes: closed form p_spike = e^{s}/(e^{s}+L-1), s = 64/sqrt(64) = 8
    K[7, 0] = a
    K[23, 1] = b
    r = oracle_mod.select(q, K, 1)
    p = np.exp(8.0) / (np.exp(8.0) + L - 1)
    np.testing.assert_allclose(r["alpha"][0, 7], p, rtol=1e-12)
    np.testing.assert_allclose(r["alpha"][1, 23], p, rtol=1e-12)
    np.testing.assert_allclose(r["alpha"][0, 0], (1 - p) / (L - 1), rtol=1e-12)
    assert r["idx"][0, 0] == 7 and r["idx"][1, 0] == 23


def test_select_permutation_equivariance(oracle_mod):
    rng = _rng(7)
    B, Hq, Hkv, d, L, k = 3, 4, 2, 64, 200, 17
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    K = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    r = oracle_mod.select(q, K, k)
    perm = rng.permutation(L)
    rp = oracle_mod.select(q, K[perm], k)                        # new row i holds old row perm[i]
    for h in range(Hkv):
        assert set(perm[rp["idx"][h]].tolist()) == set(r["idx"][h].tolist())


def test_select_mass_monotone_in_k(oracle_mod):
    rng = _rng(8)
    q = rng.standard_normal((2, 2, 64)).astype(np.float32)
    K = rng.standard_normal((64, 1, 64)).astype(np.float32) * 3
    prev = 0.0
    for k in range(1, 65):
        r = oracle_mod.select(q, K, k)
        mass = r["alpha"][0, r["idx"][0]].sum()
        assert mass >= prev
        prev = mass
    assert abs(prev - 1) < 1e-12


# ----------------------------------------------------------------------- attention
def _sdpa_reference(q, kc, vc, k_blk, v_blk, idx=None):
    """torch's scaled_dot_product_attention (CPU, fp64) over cache (optionally gathered) + block keys."""
    B, Hq, d = q.shape
    Hkv = kc.shape[1]
    G = Hq // Hkv
    outs, lses = [], []
    for h in range(Hkv):
        kk = kc[:, h] if idx is None else kc[idx[h], h]
        vv = vc[:, h] if idx is None else vc[idx[h], h]
        if k_blk is not None:
            kk = np.concatenate([kk, k_blk[:, h]], 0)
            vv = np.concatenate([vv, v_blk[:, h]], 0)
        qq = torch.from_numpy(q[:, h * G:(h + 1) * G].astype(np.float64)).permute(1, 0, 2)    # [G,B,d]
        kt = torch.from_numpy(kk.astype(np.float64))[None].expand(G, -1, -1)
        vt = torch.from_numpy(vv.astype(np.float64))[None].expand(G, -1, -1)
        o = torch.nn.functional.scaled_dot_product_attention(qq, kt, vt)                     # [G,B,d]
        outs.append(o.permute(1, 0, 2).numpy())
        lses.append(torch.logsumexp(qq @ kt.transpose(1, 2) / np.sqrt(d), dim=-1).T.numpy())
    return np.concatenate(outs, 1), np.concatenate(lses, 1)


@pytest.mark.parametrize("d", [64, 128])
def test_exact_attn_matches_torch_sdpa(oracle_mod, d):
    rng = _rng(10 + d)
    B, Hq, Hkv, L = 5, 6, 3, 211
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    kc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    vc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    kb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    vb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    out, lse = oracle_mod.exact_attn(q, kc, vc, kb, vb)
    want, want_lse = _sdpa_reference(q, kc, vc, kb, vb)
    np.testing.assert_allclose(out, want, rtol=0, atol=2e-7)
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-6)
    out2, _ = oracle_mod.exact_attn(q, kc, vc)                   # prefix only
    want2, _ = _sdpa_reference(q, kc, vc, None, None)
    np.testing.assert_allclose(out2, want2, rtol=0, atol=2e-7)


def test_sparse_attn_matches_torch_sdpa_on_gathered_rows(oracle_mod):
    rng = _rng(20)
    B, Hq, Hkv, d, L, k = 4, 4, 2, 64, 150, 13
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    kc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    vc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    kb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    vb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    idx = np.stack([np.sort(rng.choice(L, k, replace=False)) for _ in range(Hkv)]).astype(np.int32)
    out, lse = oracle_mod.sparse_attn(q, kc, vc, idx, kb, vb)
    want, want_lse = _sdpa_reference(q, kc, vc, kb, vb, idx)
    np.testing.assert_allclose(out, want, rtol=0, atol=2e-7)
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-6)


def test_attn_zero_query_gives_mean_of_values(oracle_mod):
    rng = _rng(21)
    B, Hq, Hkv, d, L, k = 3, 4, 2, 64, 90, 10
    q = np.zeros((B, Hq, d), np.float32)
    kc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    vc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    kb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    vb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    out, lse = oracle_mod.exact_attn(q, kc, vc, kb, vb)
    G = Hq // Hkv
    for g in range(Hq):
        want = np.concatenate([vc[:, g // G], vb[:, g // G]]).astype(np.float64).mean(axis=0)
        np.testing.assert_allclose(out[:, g], np.broadcast_to(want, (B, d)), atol=1e-7)
    np.testing.assert_allclose(lse, np.log(L + B), atol=1e-6)
    idx = np.stack([np.sort(rng.choice(L, k, replace=False)) for _ in range(Hkv)]).astype(np.int32)
    out, lse = oracle_mod.sparse_attn(q, kc, vc, idx, kb, vb)
    for g in range(Hq):
        h = g // G
        want = np.concatenate([vc[idx[h], h], vb[:, h]]).astype(np.float64).mean(axis=0)
        np.testing.assert_allclose(out[:, g], np.broadcast_to(want, (B, d)), atol=1e-7)
    np.testing.assert_allclose(lse, np.log(k + B), atol=1e-6)


def test_attn_one_hot_values_read_off_probabilities(oracle_mod):
    rng = _rng(22)
    B, Hq, Hkv, d, L = 2, 2, 1, 64, 60        # L + B <= d so every key gets its own value axis
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    kc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    kb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    vall = np.eye(d, dtype=np.float32)[: L + B]
    vc, vb = vall[:L, None, :].copy(), vall[L:, None, :].copy()
    out, _ = oracle_mod.exact_attn(q, kc, vc, kb, vb)
    keys = np.concatenate([kc[:, 0], kb[:, 0]]).astype(np.float64)
    for b in range(B):
        for g in range(Hq):
            p = sp_softmax(keys @ q[b, g].astype(np.float64) / np.sqrt(d))
            np.testing.assert_allclose(out[b, g, : L + B], p, atol=1e-7)
            assert np.all(out[b, g, L + B:] == 0)


def test_attn_shift_invariance(oracle_mod):
    # adding one vector c to every key (cache and block) shifts all logits of a row equally
    rng = _rng(23)
    B, Hq, Hkv, d, L = 3, 2, 1, 64, 80
    q = (rng.integers(-8, 9, (B, Hq, d)) / 8).astype(np.float32)
    kc = (rng.integers(-8, 9, (L, Hkv, d)) / 8).astype(np.float32)
    vc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    kb = (rng.integers(-8, 9, (B, Hkv, d)) / 8).astype(np.float32)
    vb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    c = (rng.integers(-4, 5, d) / 4).astype(np.float32)          # exactly representable sums
    o1, l1 = oracle_mod.exact_attn(q, kc, vc, kb, vb)
    o2, l2 = oracle_mod.exact_attn(q, kc + c, vc, kb + c, vb)
    np.testing.assert_allclose(o1, o2, atol=1e-6)
    shift = (q.astype(np.float64) @ c.astype(np.float64)) / np.sqrt(d)
    np.testing.assert_allclose(l2 - l1, shift, atol=1e-5)
    s1 = oracle_mod.select(q, kc, 9)
    s2 = oracle_mod.select(q, kc + c, 9)
    np.testing.assert_allclose(s1["alpha"], s2["alpha"], rtol=1e-10)
    assert np.array_equal(s1["idx"], s2["idx"])


def test_sparse_with_k_equal_L_is_exact_and_order_free(oracle_mod):
    rng = _rng(24)
    B, Hq, Hkv, d, L = 4, 4, 2, 64, 70
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    kc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    vc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    kb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    vb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    full = np.tile(np.arange(L, dtype=np.int32), (Hkv, 1))
    oe, le = oracle_mod.exact_attn(q, kc, vc, kb, vb)
    os_, ls = oracle_mod.sparse_attn(q, kc, vc, full, kb, vb)
    assert np.array_equal(oe, os_) and np.array_equal(le, ls)
    shuf = np.stack([rng.permutation(L) for _ in range(Hkv)]).astype(np.int32)
    o3, _ = oracle_mod.sparse_attn(q, kc, vc, shuf, kb, vb)
    np.testing.assert_allclose(o3, oe, atol=1e-6)
    sel = oracle_mod.select(q, kc, L)["idx"]
    assert np.array_equal(sel, full)


def test_sparse_rejects_out_of_range_index(oracle_mod):
    q = np.zeros((1, 1, 64), np.float32)
    kc = np.zeros((8, 1, 64), np.float32)
    with pytest.raises(RuntimeError):
        oracle_mod.sparse_attn(q, kc, kc, np.array([[8]], np.int32))
    with pytest.raises(RuntimeError):
        oracle_mod.sparse_attn(q, kc, kc, np.array([[-1]], np.int32))


def test_compact_is_fancy_indexing_and_commutes_with_attention(oracle_mod):
    rng = _rng(30)
    B, Hq, Hkv, d, L, k = 3, 4, 2, 64, 120, 11
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    kc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    vc = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    kb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    vb = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    idx = np.stack([rng.permutation(L)[:k] for _ in range(Hkv)]).astype(np.int32)
    ks, vs = oracle_mod.compact(kc, idx), oracle_mod.compact(vc, idx)
    want = np.stack([kc[idx[h], h] for h in range(Hkv)], axis=1)        # numpy fancy indexing, [k,Hkv,d]
    assert np.array_equal(ks, want)
    # attending the compacted rows exactly is attending the selected rows sparsely
    o1, l1 = oracle_mod.sparse_attn(q, kc, vc, idx, kb, vb)
    o2, l2 = oracle_mod.exact_attn(q, ks, vs, kb, vb)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    with pytest.raises(RuntimeError):
        oracle_mod.compact(kc, np.full((Hkv, 2), L, np.int32))


# --------------------------------------------------------------------------- page estimator (Sec. 2, Quest) and overlap metrics (Eq. 1, Eq. 3)
def test_page_summary_is_blockwise_max_min(oracle_mod):
    rng = _rng(40)
    for L, p in ((48, 16), (50, 16), (7, 3), (5, 8), (33, 1)):
        K = rng.standard_normal((L, 3, 8)).astype(np.float32)
        kmax, kmin = oracle_mod.page_summary(K, p)
        n_pages = -(-L // p)
        assert kmax.shape == kmin.shape == (n_pages, 3, 8)
        for P in range(n_pages):
            rows = K[P * p:(P + 1) * p]
            assert np.array_equal(kmax[P], rows.max(axis=0)) and np.array_equal(kmin[P], rows.min(axis=0)), (L, p, P)


def test_quest_page_size_one_is_the_oracle_selection(oracle_mod):
    """With one position per page the bound is q.k itself, so the estimator must be the exact selection, bit for bit."""
    rng = _rng(41)
    q = rng.standard_normal((5, 6, 16)).astype(np.float32)
    K = rng.standard_normal((70, 2, 16)).astype(np.float32)
    est = oracle_mod.quest_select(q, K, 1, 9)
    ref = oracle_mod.select(q, K, 9)
    assert np.array_equal(est["idx"], ref["idx"])
    assert np.array_equal(est["est32"], ref["alpha32"])


def test_quest_bound_is_exact_on_pages_of_identical_rows(oracle_mod):
    """If all rows of a page are equal, max = min = the row and the bound equals q.k: the estimated
    scores must be the exact averaged probabilities of the expanded cache (Eq. 2)."""
    rng = _rng(42)
    p, n_pages, Hkv, d = 4, 9, 2, 8
    q = rng.standard_normal((3, 4, d)).astype(np.float32)
    reps = rng.standard_normal((n_pages, Hkv, d)).astype(np.float32)
    K = np.repeat(reps, p, axis=0)
    kmax, kmin = oracle_mod.page_summary(K, p)
    assert np.array_equal(kmax, reps) and np.array_equal(kmin, reps)
    est = oracle_mod.quest_probs(q, kmax, kmin, n_pages * p, p)
    _, alpha = oracle_mod.block_probs(q, K)
    np.testing.assert_allclose(est, alpha, rtol=1e-12, atol=0)


def test_quest_bound_is_sign_aware_closed_form(oracle_mod):
    """d = 2, q = (1, -2); page A holds keys (3,5) and (-1,7): max = (3,7), min = (-1,5), so the bound is
    max(3,-1) + max(-14,-10) = -7 (a bound from the maxima alone would give -11).  Page B holds (0,0) twice:
    bound 0.  One query, one head: est(A) / est(B) = exp((-7 - 0) / sqrt(2))."""
    q = np.array([[[1.0, -2.0]]], np.float32)
    K = np.array([[[3.0, 5.0]], [[-1.0, 7.0]], [[0.0, 0.0]], [[0.0, 0.0]]], np.float32)
    kmax, kmin = oracle_mod.page_summary(K, 2)
    est = oracle_mod.quest_probs(q, kmax, kmin, 4, 2)[0]
    assert est[0] == est[1] and est[2] == est[3]
    np.testing.assert_allclose(est[0] / est[2], np.exp(-7.0 / np.sqrt(2.0)), rtol=1e-12)
    np.testing.assert_allclose(est.sum(), 1.0, rtol=1e-12)


def test_quest_bound_dominates_every_key_of_its_page(oracle_mod):
    """The page score is an upper bound of q.k over the page: with one query and one head the estimated
    probability of a position is >= Z_exact / Z_est times its exact probability, i.e. est * Z_est >= exp(logit)."""
    rng = _rng(43)
    L, p, d = 60, 6, 8
    q = rng.standard_normal((1, 1, d)).astype(np.float32)
    K = rng.standard_normal((L, 1, d)).astype(np.float32)
    kmax, kmin = oracle_mod.page_summary(K, p)
    est = oracle_mod.quest_probs(q, kmax, kmin, L, p)[0]
    logits = (K[:, 0, :].astype(np.float64) @ q[0, 0].astype(np.float64)) / np.sqrt(d)
    bounds = np.log(est) - np.log(est).max()                 # bound / sqrt(d) up to one additive constant ...
    page_max = logits.reshape(-1, p).max(axis=1)
    # ... which the page holding the largest bound fixes: there bound >= its own maximum logit
    shift = np.maximum(q[0, 0] * kmax[:, 0, :], q[0, 0] * kmin[:, 0, :]).astype(np.float64).sum(axis=1).max() / np.sqrt(d)
    assert np.all(bounds.reshape(-1, p)[:, 0] + shift >= page_max - 1e-9)
    assert np.all(np.abs(est.reshape(-1, p) - est.reshape(-1, p)[:, :1]) == 0)      # one score per page


def test_quest_select_takes_whole_pages_and_sums_to_one(oracle_mod):
    rng = _rng(44)
    L, p, k = 96, 8, 24
    q = rng.standard_normal((4, 4, 16)).astype(np.float32)
    K = rng.standard_normal((L, 2, 16)).astype(np.float32)
    r = oracle_mod.quest_select(q, K, p, k)
    np.testing.assert_allclose(r["est32"].sum(axis=1, dtype=np.float64), 1.0, atol=1e-5)
    for h in range(2):
        pages = np.unique(r["idx"][h] // p)
        assert len(pages) == k // p
        assert np.array_equal(r["idx"][h], (pages[:, None] * p + np.arange(p)[None, :]).ravel())
        page_score = r["est32"][h].reshape(-1, p)[:, 0]
        assert set(pages) == set(_brute_topk(page_score, k // p))


def test_overlap_is_set_intersection_over_k(oracle_mod):
    rng = _rng(45)
    for k in (1, 5, 64):
        a = rng.choice(300, k, replace=False).astype(np.int32)
        b = rng.choice(300, k, replace=False).astype(np.int32)
        want = len(set(a.tolist()) & set(b.tolist())) / k
        assert oracle_mod.overlap(a, b) == want
        assert oracle_mod.overlap(b, a) == want
        assert oracle_mod.overlap(a, a[::-1].copy()) == 1.0
        assert oracle_mod.overlap(a, (a + 1000).astype(np.int32)) == 0.0


def test_worked_example_fixture(oracle_mod):
    """tests/golden/worked_example.json: the oracle reproduces its stored output exactly, and the stored
    alpha of position 0 equals the closed form.  The four rows' logits over the six keys are small
    integers (a logit is (q0*k0 + q1*k1)/8 with q in {(8,0),(0,8),(8,8),(-8,0)}):
      row (q0,g0): k0        = [1,0,1,-1,2,1]     row (q0,g1): k1  = [0,1,1,0,0,0]
      row (q1,g0): k0 + k1   = [1,1,2,-1,2,1]     row (q1,g1): -k0 = [-1,0,-1,1,-2,-1]
    alpha[0] = 1/4 (e/Z1 + 1/Z2 + e/Z3 + e^-1/Z4) (Eq. 5); positions 0 and 5 hold equal keys (a tie)."""
    import importlib.util
    import json
    import math
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_worked_example", os.path.join(here, "golden", "make_worked_example.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = json.load(open(os.path.join(here, "golden", "worked_example.json")))
    assert mod.compute() == stored
    e = math.e
    z1 = 3 * e + 1 + 1 / e + e * e
    z2 = 4 + 2 * e
    z3 = 3 * e + 2 * e * e + 1 / e
    z4 = 3 / e + 1 + e + 1 / (e * e)
    alpha = [float.fromhex(x) for x in stored["alpha_fp64"]]
    assert abs(alpha[0] - 0.25 * (e / z1 + 1 / z2 + e / z3 + (1 / e) / z4)) < 1e-15
    assert abs(alpha[4] - 0.25 * (e * e / z1 + 1 / z2 + e * e / z3 + (1 / (e * e)) / z4)) < 1e-15
    assert alpha[0] == alpha[5] and abs(sum(alpha) - 1.0) < 1e-15
    assert stored["idx"] == [[2, 4]]
