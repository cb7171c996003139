"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on seeded inputs.

Bar (the benchmark spec): index sets bit-exact under the lowest-index tie-break, except entries whose
oracle fp32 score lies within 1e-6 relative of the oracle's k-th score; attention outputs within
max-abs 2e-2 (bf16 inputs, fp32 accumulate) / 1e-4 (fp32 inputs).
"""
import zlib

import numpy as np
import pytest

from paper_2602_14209_amd.workloads import CONFIGS, Workload, make_layer

pytestmark = pytest.mark.gpu


def _run_workload(oracle_mod, w: Workload, seed: int, ks=None, steps=None, blk=True):
    from gpu_util import Problem, check_alpha, check_index_sets, check_out
    x = make_layer(w, seed, steps=steps)
    T = x["q"].shape[0]
    for k in (ks or w.ks):
        print(f"[parity] {w.name} dtype={w.dtype} Hq={w.Hq} Hkv={w.Hkv} d={w.d} L={w.L} B={w.B} k={k} seed={seed}", flush=True)
        p = Problem(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0] if blk else None,
                    x["v_blk"][0] if blk else None, k, w.dtype)
        ref = oracle_mod.select(x["q"][0], x["k_cache"], k)
        idx, alpha = p.select()
        check_alpha(alpha, ref["alpha32"])
        check_index_sets(idx, ref["idx"], ref["alpha32"], w.L)
        idx2, _ = p.select(with_alpha=False)          # alpha kept in the workspace: same set
        assert np.array_equal(idx, idx2)
        o_ref, l_ref = oracle_mod.exact_attn(x["q"][0], x["k_cache"], x["v_cache"],
                                             x["k_blk"][0] if blk else None, x["v_blk"][0] if blk else None)
        o, l = p.exact()
        check_out(o, o_ref, l, l_ref, w.dtype)
        if w.G * w.B <= 256 or w.dtype == "f32":
            p.out.fill_(float("nan")); p.idx.fill_(-1); p.alpha.fill_(float("nan"))
            o, l, idx3, alpha3 = p.step1()                # fused step 1: same definitions, shared pass
            check_out(o, o_ref, l, l_ref, w.dtype)
            check_alpha(alpha3, ref["alpha32"])
            check_index_sets(idx3, ref["idx"], ref["alpha32"], w.L)
        for t in range(1, T):
            p.set_q(x["q"][t])
            if blk:
                p.set_blk(x["k_blk"][t], x["v_blk"][t])
            o_ref, l_ref = oracle_mod.sparse_attn(x["q"][t], x["k_cache"], x["v_cache"], ref["idx"],
                                                  x["k_blk"][t] if blk else None, x["v_blk"][t] if blk else None)
            o, l = p.sparse(ref["idx"])
            check_out(o, o_ref, l, l_ref, w.dtype)


def test_c0_tiny_fp32(oracle_mod):
    _run_workload(oracle_mod, CONFIGS["c0"], seed=1000)


@pytest.mark.parametrize("case", [
    # name, dtype, Hq, Hkv, d, L, B, k  -- several tiles, ragged tails, ragged rows, both wave counts
    ("s1", "bf16", 8, 2, 128, 1000, 32, 100),
    ("s2", "bf16", 8, 2, 64, 777, 32, 65),
    ("s3", "bf16", 14, 2, 128, 1500, 32, 200),      # G=7: 224 rows, 8 wavefronts
    ("s4", "bf16", 4, 4, 128, 300, 5, 17),          # G=1, B=5: ragged rows inside one M tile
    ("s5", "bf16", 6, 2, 64, 50, 3, 50),            # L < one tile, k = L
    ("s6", "bf16", 4, 1, 128, 4097, 32, 1),         # k = 1, L one past a tile boundary
    ("s7", "f32", 6, 2, 128, 700, 7, 33),
    ("s8", "f32", 8, 1, 64, 129, 16, 129),          # 128 rows: two fp32 row groups, k = L
    ("s9", "f32", 2, 2, 64, 31, 1, 5),
    ("s10", "bf16", 16, 2, 128, 2048, 48, 512),     # G*B = 384 > 256: row groups (no select)
    ("s11", "bf16", 4, 2, 128, 1, 32, 1),           # one cached key
    ("s12", "bf16", 4, 2, 128, 64, 32, 64),         # exactly one tile
    ("s13", "bf16", 4, 2, 128, 65, 32, 7),          # second tile holds one key: its upper half is all padding
    ("s14", "bf16", 8, 2, 64, 97, 16, 33),          # second tile holds 33 keys: one key in the upper half
    ("s15", "bf16", 1, 1, 128, 300, 1, 10),         # a single query row
    ("s16", "bf16", 12, 2, 128, 5000, 32, 300),     # G*B = 192: two row groups in attention, 8 wavefronts in the column sums
    ("s17", "bf16", 8, 8, 64, 20000, 32, 1500),     # k + B > 640 key positions: several passes of the sparse kernel
])
def test_small_shapes(oracle_mod, case):
    name, dtype, Hq, Hkv, d, L, B, k = case
    w = Workload(name, dtype, Hq=Hq, Hkv=Hkv, d=d, L=L, B=B, ks=(k,), T=3, heavy_frac=0.02, heavy_scale=3.0)
    if name == "s10":
        _attention_only(oracle_mod, w, seed=77)
    else:
        _run_workload(oracle_mod, w, seed=zlib.crc32(name.encode()) % 1000 + 5)     # fixed per case, printed by the run


def _attention_only(oracle_mod, w, seed):
    from gpu_util import Problem, check_out
    import paper_2602_14209_amd.binding as mb
    x = make_layer(w, seed, steps=2)
    k = w.ks[0]
    p = Problem(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0], k, w.dtype)
    o_ref, l_ref = oracle_mod.exact_attn(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0])
    o, l = p.exact()
    check_out(o, o_ref, l, l_ref, w.dtype)
    rng = np.random.default_rng(seed)
    idx = np.stack([np.sort(rng.choice(w.L, k, replace=False)) for _ in range(w.Hkv)]).astype(np.int32)
    o_ref, l_ref = oracle_mod.sparse_attn(x["q"][1], x["k_cache"], x["v_cache"], idx, x["k_blk"][1], x["v_blk"][1])
    p.set_q(x["q"][1]); p.set_blk(x["k_blk"][1], x["v_blk"][1])
    o, l = p.sparse(idx)
    check_out(o, o_ref, l, l_ref, w.dtype)
    rc = mb.mage_select(p.shape, p.q, p.kc, p.idx, None, p.ws)
    assert rc == -3        # MAGE_ERR_UNSUPPORTED: B*G > 256 with bf16


@pytest.mark.parametrize("case", [
    # the sparse kernel deals a row tile's output channels to 4, 2 or 1 workgroups, by how many workgroups
    # (KV heads x row tiles) the call has: <= 64, <= 128, more.  name, Hq, Hkv, d, L, B, k
    ("w1", 40, 20, 128, 900, 56, 150),      # 20 heads x 7 row tiles = 140 workgroups: channels unsplit
    ("w2", 32, 16, 128, 900, 40, 150),      # 16 x 5 = 80: two workgroups per row tile
    ("w3", 40, 20, 64, 900, 56, 150),       # d = 64, unsplit
    ("w4", 8, 2, 128, 3000, 32, 1100),      # four per row tile and two passes over the key positions
    ("w5", 32, 16, 64, 700, 40, 700),       # d = 64, 80 workgroups: two per row tile, two passes, k = L
    ("w6", 8, 2, 128, 4000, 32, 1500),      # three passes: the second finds its index entries already requested, the third asks for its own
    ("w7", 4, 1, 128, 2000, 16, 660),       # 43 tiles: the second pass is almost as long as the first
])
def test_sparse_channel_split_variants(oracle_mod, case):
    import torch
    import paper_2602_14209_amd.binding as mb
    from gpu_util import Problem, check_out
    name, Hq, Hkv, d, L, B, k = case
    w = Workload(name, "bf16", Hq=Hq, Hkv=Hkv, d=d, L=L, B=B, ks=(k,), T=2, heavy_frac=0.02, heavy_scale=3.0)
    seed = zlib.crc32(name.encode()) % 1000 + 5
    x = make_layer(w, seed, steps=2)
    rng = np.random.default_rng(seed)
    idx = np.stack([np.sort(rng.choice(L, k, replace=False)) for _ in range(Hkv)]).astype(np.int32)
    p = Problem(x["q"][1], x["k_cache"], x["v_cache"], x["k_blk"][1], x["v_blk"][1], k, w.dtype)
    o_ref, l_ref = oracle_mod.sparse_attn(x["q"][1], x["k_cache"], x["v_cache"], idx, x["k_blk"][1], x["v_blk"][1])
    print(f"[parity] channel split {case}", flush=True)
    o, l = p.sparse(idx)
    check_out(o, o_ref, l, l_ref, w.dtype)
    k_sel = torch.zeros((k, Hkv, d), dtype=p.kc.dtype, device="cuda")
    v_sel = torch.zeros_like(k_sel)
    mb.check(mb.mage_compact(p.shape, p.kc, p.vc, torch.from_numpy(idx).cuda(), k_sel, v_sel), "mage_compact")
    p.out.fill_(float("nan"))
    p.lse.fill_(float("nan"))
    mb.check(mb.mage_sparse_attn_compact(p.shape, p.q, k_sel, v_sel, p.kb, p.vb, p.out, p.lse, p.ws), "compact attn")
    torch.cuda.synchronize()
    check_out(p.out.cpu().numpy(), o_ref, p.lse.cpu().numpy(), l_ref, w.dtype)


def test_no_block_keys(oracle_mod):
    w = Workload("nb", "bf16", Hq=8, Hkv=2, d=128, L=600, B=32, ks=(128,), T=2, heavy_frac=0.02, heavy_scale=3.0)
    _run_workload(oracle_mod, w, seed=11, blk=False)
    w = Workload("nbf", "f32", Hq=4, Hkv=2, d=64, L=200, B=4, ks=(20,), T=2)
    _run_workload(oracle_mod, w, seed=12, blk=False)


def test_c1_bf16(oracle_mod):
    _run_workload(oracle_mod, CONFIGS["c1"], seed=1001, steps=3)


def test_c2_bf16(oracle_mod):
    _run_workload(oracle_mod, CONFIGS["c2"], seed=1002, steps=2)


@pytest.mark.parametrize("layer", [0, 1])
def test_c3_full_shape_two_layers(oracle_mod, layer):
    """Config 3 at its real shape (G = 7: 224 rows per KV head, two row groups streaming the same tiles,
    L = 65536), two of its independently seeded layers: selection, exact attention, fused step 1 and the
    sparse steps, every output compared in full."""
    from paper_2602_14209_amd.workloads import layer_seed
    _run_workload(oracle_mod, CONFIGS["c3"], seed=layer_seed(1000, 3, layer), steps=2)


def test_side_stream_select_beside_exact_attention(oracle_mod):
    """Alg. 1's arrangement at config 2's shape: the select stream waits for the event that says Q1 is
    ready, runs mage_select with a workspace of its own while the main stream runs mage_exact_attn of the
    same layer, and the main stream joins once.  Both streams' results are compared with the oracle."""
    import torch
    import paper_2602_14209_amd.binding as mb
    from gpu_util import Problem, check_alpha, check_index_sets, check_out, to_device
    w = CONFIGS["c2"]
    x = make_layer(w, 1002, steps=1)
    k = w.k
    print(f"[parity] side stream, c2 shape L={w.L} k={k}", flush=True)
    p = Problem(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0], k, w.dtype)
    ws_side = mb.alloc_workspace(p.shape)
    main_s, side_s = torch.cuda.Stream(), torch.cuda.Stream()
    q_host = to_device(x["q"][0], w.dtype)
    torch.cuda.synchronize()
    for rep in range(3):                         # the arrangement is replayed: stale results cannot pass
        p.out.fill_(float("nan")); p.lse.fill_(float("nan")); p.idx.fill_(-1); p.alpha.fill_(float("nan"))
        p.q.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(main_s):
            p.q.copy_(q_host)                    # "QKVProj": Q1 becomes ready on the main stream
            q_ready = torch.cuda.Event()
            q_ready.record(main_s)
        side_s.wait_event(q_ready)               # select stream: wait Q1 (non-blocking for the host)
        mb.check(mb.mage_select(p.shape, p.q, p.kc, p.idx, p.alpha, ws_side, side_s), "mage_select")
        mb.check(mb.mage_exact_attn(p.shape, p.q, p.kc, p.vc, p.kb, p.vb, p.out, p.lse, p.ws, main_s), "mage_exact_attn")
        done = torch.cuda.Event()
        done.record(side_s)
        main_s.wait_event(done)                  # synchronize(main, select): the one join of Phase 1
        main_s.synchronize()
    ref = oracle_mod.select(x["q"][0], x["k_cache"], k)
    check_alpha(p.alpha.cpu().numpy(), ref["alpha32"])
    check_index_sets(p.idx.cpu().numpy(), ref["idx"], ref["alpha32"], w.L)
    o_ref, l_ref = oracle_mod.exact_attn(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0])
    check_out(p.out.cpu().numpy(), o_ref, p.lse.cpu().numpy(), l_ref, w.dtype)


def test_sparse_k_equal_L_matches_exact_on_gpu(oracle_mod):
    from gpu_util import ATOL, Problem
    w = Workload("kL", "bf16", Hq=8, Hkv=2, d=128, L=384, B=32, ks=(384,), T=1)
    x = make_layer(w, 5)
    p = Problem(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0], 384, "bf16")
    oe, le = p.exact()
    full = np.tile(np.arange(w.L, dtype=np.int32), (w.Hkv, 1))
    os_, ls = p.sparse(full)
    assert np.abs(oe - os_).max() <= ATOL["bf16"]
    rng = np.random.default_rng(0)
    shuf = np.stack([rng.permutation(w.L) for _ in range(w.Hkv)]).astype(np.int32)
    o3, _ = p.sparse(shuf)
    assert np.abs(oe - o3).max() <= ATOL["bf16"]
    idx, _ = p.select()
    assert np.array_equal(idx, full)


def test_select_ties_and_uniform_on_gpu(oracle_mod):
    from gpu_util import Problem
    rng = np.random.default_rng(3)
    B, Hq, Hkv, d, L, k = 32, 4, 2, 128, 500, 37
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    from paper_2602_14209_amd.workloads import bf16_to_f32, round_to_bf16
    q = bf16_to_f32(round_to_bf16(q))
    K = np.broadcast_to(bf16_to_f32(round_to_bf16(rng.standard_normal((1, Hkv, d)).astype(np.float32))), (L, Hkv, d)).copy()
    p = Problem(q, K, K, None, None, k, "bf16")
    idx, alpha = p.select()
    # all keys equal: every score of a head is the same number and the set is {0..k-1}
    assert np.array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (Hkv, 1)))
    assert np.all(alpha == alpha[:, :1])
    np.testing.assert_allclose(alpha, 1.0 / L, rtol=1e-5)
    # duplicated rows: exact tie in the ranked fp32 score, the smaller index must win
    K2 = bf16_to_f32(round_to_bf16(rng.standard_normal((L, Hkv, d)).astype(np.float32)))
    ref = oracle_mod.select(q, K2, k)
    for h in range(Hkv):
        order = np.argsort(-ref["alpha32"][h], kind="stable")
        K2[order[k + 3], h] = K2[order[k - 1], h]
    ref = oracle_mod.select(q, K2, k)
    p = Problem(q, K2, K2, None, None, k, "bf16")
    idx, alpha = p.select()
    from gpu_util import check_index_sets
    check_index_sets(idx, ref["idx"], ref["alpha32"], L)


def _plant_near_tie(oracle_mod, q, K, k, h, lo=1.5e-6, hi=3.5e-6):
    """Make the keys at ranks k and k+1 of KV head h nearly tie: the rank-(k+1) key (a different key,
    so the two fp32 scores carry unrelated rounding errors) is moved, one bf16 step of one channel at a
    time, until the two averaged probabilities differ by a relative lo..hi -- more than the band that
    excuses a mismatch, less than an fp32 pipeline resolves reliably.  The steps are chosen with a numpy
    model of the change (a search heuristic only); the result is accepted on the oracle's values.
    Returns (keys, gap) or None."""
    from paper_2602_14209_amd.workloads import bf16_to_f32, round_to_bf16
    B, Hq, d = q.shape
    G = Hq // K.shape[1]
    ref = oracle_mod.select(q, K, k)
    order = np.argsort(-ref["alpha"][h], kind="stable")
    a, b = int(order[k - 1]), int(order[k])
    Q = q[:, h * G:(h + 1) * G].reshape(B * G, d).astype(np.float64) / np.sqrt(d)
    K = K.copy()
    for _ in range(60):
        Kh = K[:, h].astype(np.float64)
        S = Q @ Kh.T
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        Z = E.sum(axis=1)
        gap = (E[:, a] / Z).mean() / (E[:, b] / Z).mean() - 1.0          # > 0: a ahead
        if lo <= abs(gap) <= hi:
            break
        # every single bf16 step of key b: new value per (channel, direction)
        bits = round_to_bf16(K[b, h]).astype(np.int32)
        best = None
        for sign in (+1, -1):
            newv = bf16_to_f32((bits + sign).astype(np.uint16)).astype(np.float64)
            dS = Q * (newv - Kh[b])[None, :]                                # [rows, channels]: change of the logit of key b
            Eb = E[:, b][:, None] * np.exp(dS)
            Zn = Z[:, None] - E[:, b][:, None] + Eb
            g = (E[:, a][:, None] / Zn).mean(axis=0) / (Eb / Zn).mean(axis=0) - 1.0
            score = np.where(np.abs(g) >= lo, np.abs(g), np.inf)           # closest to the window from outside, never inside the excuse band
            c = int(np.argmin(score))
            if np.isfinite(score[c]) and (best is None or score[c] < best[0]):
                best = (score[c], c, newv[c])
        if best is None or best[0] >= abs(gap):
            return None
        K[b, h, best[1]] = np.float32(best[2])
    else:
        return None
    r2 = oracle_mod.select(q, K, k)
    al = r2["alpha"][h]
    srt = np.argsort(-al, kind="stable")
    gap = abs(al[a] - al[b]) / al[a]
    if {int(srt[k - 1]), int(srt[k])} != {a, b} or not (lo <= gap <= hi) or r2["alpha32"][h, a] == r2["alpha32"][h, b]:
        return None
    return K, gap


@pytest.mark.parametrize("seed", [31, 32, 33, 34, 35, 36])
def test_near_tie_at_rank_k_follows_the_oracle(oracle_mod, seed):
    """Two keys whose exact averaged probabilities differ by a few 1e-6 (relative) sit at ranks k and k+1:
    the fp32 scores of the kernels cannot tell them apart reliably, the fp64 re-score of the candidates
    near the k-th value must -- in mage_select and in the fused mage_step1."""
    from gpu_util import Problem, check_index_sets
    from paper_2602_14209_amd.workloads import bf16_to_f32, round_to_bf16
    rng = np.random.default_rng(seed)
    B, Hq, Hkv, d, L, k = 32, 8, 2, 128, 700, 64 + seed
    qm = rng.standard_normal((1, Hq, d)).astype(np.float32)
    q = bf16_to_f32(round_to_bf16(qm + 0.1 * rng.standard_normal((B, Hq, d)).astype(np.float32)))
    K = bf16_to_f32(round_to_bf16(rng.standard_normal((L, Hkv, d)).astype(np.float32)))
    V = bf16_to_f32(round_to_bf16(rng.standard_normal((L, Hkv, d)).astype(np.float32)))
    planted = 0
    for h in range(Hkv):
        got = _plant_near_tie(oracle_mod, q, K, k, h)
        if got is None:
            continue
        K, gap = got
        planted += 1
        print(f"[near-tie] seed={seed} head={h} k={k}: relative gap {gap:.2e} planted at ranks k, k+1", flush=True)
    assert planted >= 1, "no near-tie could be planted (the construction, not the kernels, needs attention)"
    ref = oracle_mod.select(q, K, k)
    p = Problem(q, K, V, None, None, k, "bf16")
    idx, _ = p.select()
    check_index_sets(idx, ref["idx"], ref["alpha32"], L)
    _, _, idx1, _ = p.step1()
    check_index_sets(idx1, ref["idx"], ref["alpha32"], L)


def test_select_long_rows_and_group_overflow(oracle_mod):
    """Top-k filter fed with group maxima: more groups than the LDS copy holds (L > 131072), and a
    row where every group reaches the bound (uniform alpha), which must leave by the radix route."""
    from gpu_util import Problem, check_alpha, check_index_sets
    from paper_2602_14209_amd.workloads import bf16_to_f32, round_to_bf16
    rng = np.random.default_rng(17)
    B, Hq, Hkv, d, L, k = 8, 2, 1, 64, 140001, 96
    q = bf16_to_f32(round_to_bf16(rng.standard_normal((B, Hq, d)).astype(np.float32)))
    K = bf16_to_f32(round_to_bf16(rng.standard_normal((L, Hkv, d)).astype(np.float32)))
    ref = oracle_mod.select(q, K, k)
    p = Problem(q, K, K, None, None, k, "bf16")
    idx, alpha = p.select()
    check_alpha(alpha, ref["alpha"])
    check_index_sets(idx, ref["idx"], ref["alpha32"], L)
    # all keys equal: 80000 / 16 = 5000 groups at the bound, more than the candidate list holds
    L2 = 80000
    K2 = np.broadcast_to(K[:1], (L2, Hkv, d)).copy()
    p = Problem(q, K2, K2, None, None, k, "bf16")
    idx, alpha = p.select()
    assert np.array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (Hkv, 1)))
    np.testing.assert_allclose(alpha, 1.0 / L2, rtol=1e-5)



def test_c4_full_size_headline_shape(oracle_mod):
    """The benchmark's shape and launch configuration (L=131072, Hq=32, Hkv=8, k=512): selection,
    exact attention (all block positions) and one sparse step per budget, all checked in full."""
    from gpu_util import Problem, check_alpha, check_index_sets, check_out
    w = CONFIGS["c4"]
    x = make_layer(w, 1004, steps=2)
    k = 512
    print(f"[parity] c4 full size L={w.L} k={k}", flush=True)
    p = Problem(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0], k, w.dtype)
    idx, alpha = p.select()
    o, l = p.exact()
    print("[parity] c4 GPU done, running the oracle", flush=True)
    ref = oracle_mod.select(x["q"][0], x["k_cache"], k)
    check_alpha(alpha, ref["alpha32"])
    check_index_sets(idx, ref["idx"], ref["alpha32"], w.L)
    o_ref, l_ref = oracle_mod.exact_attn(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0])
    check_out(o, o_ref, l, l_ref, w.dtype)
    o, l, idx3, alpha3 = p.step1()
    check_out(o, o_ref, l, l_ref, w.dtype)
    check_alpha(alpha3, ref["alpha32"])
    check_index_sets(idx3, ref["idx"], ref["alpha32"], w.L)
    for kk in w.ks:
        if kk == k:
            pk, ref_k = p, ref["idx"]
        else:
            pk = Problem(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][1], x["v_blk"][1], kk, w.dtype)
            ref_k = np.stack([oracle_mod.topk(ref["alpha32"][h], kk) for h in range(w.Hkv)])
            idx_k, _ = pk.select(with_alpha=False)
            check_index_sets(idx_k, ref_k, ref["alpha32"], w.L)
        pk.set_q(x["q"][1])
        pk.set_blk(x["k_blk"][1], x["v_blk"][1])
        o_ref, l_ref = oracle_mod.sparse_attn(x["q"][1], x["k_cache"], x["v_cache"], ref_k, x["k_blk"][1], x["v_blk"][1])
        o, l = pk.sparse(ref_k)
        check_out(o, o_ref, l, l_ref, w.dtype)


@pytest.mark.parametrize("case", [
    ("k1", "bf16", 8, 2, 128, 3000, 32, 200),
    ("k2", "bf16", 6, 2, 64, 500, 7, 37),
    ("k3", "f32", 4, 2, 64, 300, 5, 50),
    ("k4", "bf16", 32, 8, 128, 20000, 32, 1024),      # two passes of the sparse kernel
])
def test_compacted_rows(oracle_mod, case):
    """mage_compact is a copy (bit-exact); mage_sparse_attn_compact equals the sparse step."""
    import torch
    import paper_2602_14209_amd.binding as mb
    from gpu_util import Problem, check_out, to_device
    name, dtype, Hq, Hkv, d, L, B, k = case
    w = Workload(name, dtype, Hq=Hq, Hkv=Hkv, d=d, L=L, B=B, ks=(k,), T=2, heavy_frac=0.02, heavy_scale=3.0)
    x = make_layer(w, 321)
    print(f"[parity] compact {case}", flush=True)
    p = Problem(x["q"][1], x["k_cache"], x["v_cache"], x["k_blk"][1], x["v_blk"][1], k, dtype)
    rng = np.random.default_rng(9)
    idx = np.stack([rng.permutation(L)[:k] for _ in range(Hkv)]).astype(np.int32)     # unsorted on purpose
    idx_d = torch.from_numpy(idx).cuda()
    k_sel = torch.zeros((k, Hkv, d), dtype=p.kc.dtype, device="cuda")
    v_sel = torch.zeros_like(k_sel)
    mb.check(mb.mage_compact(p.shape, p.kc, p.vc, idx_d, k_sel, v_sel), "mage_compact")
    torch.cuda.synchronize()
    want_k = to_device(oracle_mod.compact(x["k_cache"], idx), dtype)
    want_v = to_device(oracle_mod.compact(x["v_cache"], idx), dtype)
    as_bits = (lambda t: t.view(torch.int16)) if dtype == "bf16" else (lambda t: t.view(torch.int32))
    assert torch.equal(as_bits(k_sel), as_bits(want_k)) and torch.equal(as_bits(v_sel), as_bits(want_v))
    o_ref, l_ref = oracle_mod.sparse_attn(x["q"][1], x["k_cache"], x["v_cache"], idx, x["k_blk"][1], x["v_blk"][1])
    p.out.fill_(float("nan"))
    mb.check(mb.mage_sparse_attn_compact(p.shape, p.q, k_sel, v_sel, p.kb, p.vb, p.out, p.lse, p.ws), "compact attn")
    torch.cuda.synchronize()
    check_out(p.out.cpu().numpy(), o_ref, p.lse.cpu().numpy(), l_ref, dtype)
    o, l = p.sparse(idx)
    check_out(o, o_ref, l, l_ref, dtype)


@pytest.mark.parametrize("case", [
    # name, n_seq, Hq, Hkv, d, L, B, k, in-block keys
    ("b1", 3, 8, 2, 128, 2500, 32, 300, True),       # 332 key positions: six tiles, the last one with 12 keys
    ("b2", 2, 14, 2, 128, 1500, 32, 200, True),      # G = 7: 224 rows, two row groups per unit, the second ragged
    ("b3", 5, 4, 4, 64, 777, 5, 65, True),           # d = 64, 5 rows, 20 units (a ragged block of workgroup ids)
    ("b4", 2, 8, 2, 128, 300, 32, 32, True),         # k + B = 64: exactly one tile
    ("b5", 2, 8, 2, 128, 300, 32, 7, True),          # one tile, 39 keys
    ("b6", 9, 4, 1, 128, 500, 32, 70, False),        # no in-block keys; second tile holds 6 keys (upper half skipped); 9 units
    ("b7", 1, 8, 2, 64, 4000, 16, 1000, True),       # a single sequence, many tiles
    ("b8", 40, 8, 8, 128, 600, 16, 100, True),       # 320 units: more workgroups than CUs (the two-per-CU ring)
    ("b9", 70, 8, 4, 64, 2500, 8, 2100, False),       # ... at d = 64, and more index entries than LDS holds at a time
    ("b10", 2, 4, 2, 128, 5000, 32, 4200, True),     # the deep ring with two refills of the index entries
    ("b11", 2, 4, 2, 128, 900, 64, 100, True),       # B = 64: the block's own rows fill the last two tiles
    ("b12", 3, 8, 2, 64, 700, 32, 20, True),         # d = 64, one ragged tile of selected rows that the block's rows complete
])
def test_batched_sparse_step(oracle_mod, case):
    """n_seq independent sequences in one launch equal the oracle's sparse step of every sequence."""
    import torch
    import paper_2602_14209_amd.binding as mb
    from gpu_util import check_out, to_device
    name, n_seq, Hq, Hkv, d, L, B, k, blk = case
    w = Workload(name, "bf16", Hq=Hq, Hkv=Hkv, d=d, L=L, B=B, ks=(k,), T=2, heavy_frac=0.02, heavy_scale=3.0)
    xs = [make_layer(w, 500 + s) for s in range(n_seq)]
    rng = np.random.default_rng(4)
    idx = np.stack([np.stack([np.sort(rng.choice(w.L, k, replace=False)) for _ in range(w.Hkv)]) for _ in range(n_seq)]).astype(np.int32)
    stack = lambda name, t=None: to_device(np.stack([x[name] if t is None else x[name][t] for x in xs]), "bf16")
    q, kc, vc = stack("q", 1), stack("k_cache"), stack("v_cache")
    kb, vb = (stack("k_blk", 1), stack("v_blk", 1)) if blk else (None, None)
    out = torch.full((n_seq, w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((n_seq, w.B, w.Hq), float("nan"), dtype=torch.float32, device="cuda")
    shape = mb.make_shape(w.B, w.Hq, w.Hkv, w.d, w.L, k, "bf16")
    print(f"[parity] batched sparse step {case}", flush=True)
    mb.check(mb.mage_sparse_attn_batched(shape, n_seq, q, kc, vc, torch.from_numpy(idx).cuda(), kb, vb, out, lse), "batched")
    torch.cuda.synchronize()
    for s in range(n_seq):
        o_ref, l_ref = oracle_mod.sparse_attn(xs[s]["q"][1], xs[s]["k_cache"], xs[s]["v_cache"], idx[s],
                                              xs[s]["k_blk"][1] if blk else None, xs[s]["v_blk"][1] if blk else None)
        check_out(out[s].cpu().numpy(), o_ref, lse[s].cpu().numpy(), l_ref, "bf16")
    # without the lse output
    out2 = torch.full_like(out, float("nan"))
    mb.check(mb.mage_sparse_attn_batched(shape, n_seq, q, kc, vc, torch.from_numpy(idx).cuda(), kb, vb, out2, None), "batched")
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))


def test_batched_sparse_step_with_more_units_than_one_grid_plane(oracle_mod):
    """264000 (sequence, head) units: the blocks of eight units spill from the grid's y dimension into z.
    Every output is written, and sequences on both sides of the boundary equal the oracle."""
    import torch
    import paper_2602_14209_amd.binding as mb
    from gpu_util import check_out, to_device
    from paper_2602_14209_amd.workloads import bf16_to_f32, round_to_bf16
    n_seq, Hq, Hkv, d, L, B, k = 33000, 8, 8, 64, 8, 1, 3
    rng = np.random.default_rng(77)
    bf16_values = lambda shape: bf16_to_f32(round_to_bf16(rng.standard_normal(shape, dtype=np.float32)))
    q, kc, vc = bf16_values((n_seq, B, Hq, d)), bf16_values((n_seq, L, Hkv, d)), bf16_values((n_seq, L, Hkv, d))
    kb, vb = bf16_values((n_seq, B, Hkv, d)), bf16_values((n_seq, B, Hkv, d))
    idx = np.sort(rng.permuted(np.tile(np.arange(L, dtype=np.int32), (n_seq, Hkv, 1)), axis=2)[:, :, :k], axis=2)
    out = torch.full((n_seq, B, Hq, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((n_seq, B, Hq), float("nan"), dtype=torch.float32, device="cuda")
    shape = mb.make_shape(B, Hq, Hkv, d, L, k, "bf16")
    print(f"[parity] batched sparse step, {n_seq * Hkv} units", flush=True)
    mb.check(mb.mage_sparse_attn_batched(shape, n_seq, to_device(q, "bf16"), to_device(kc, "bf16"), to_device(vc, "bf16"),
                                         torch.from_numpy(idx).cuda(), to_device(kb, "bf16"), to_device(vb, "bf16"), out, lse), "batched")
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
    for s in (0, 12345, 32767, 32768, 32769, n_seq - 1):
        o_ref, l_ref = oracle_mod.sparse_attn(q[s], kc[s], vc[s], idx[s], kb[s], vb[s])
        check_out(out[s].cpu().numpy(), o_ref, lse[s].cpu().numpy(), l_ref, "bf16")


@pytest.mark.parametrize("seed", list(range(12)))
def test_seeded_random_geometries(oracle_mod, seed):
    """Whole path (select, exact, fused step 1, sparse steps) on seeded random geometries inside the
    supported ranges: odd lengths, every group size, both head dimensions, both element types."""
    rng = np.random.default_rng(9000 + seed)
    dtype = "bf16" if seed % 4 else "f32"
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 3, 4, 7, 8]))
    B = int(rng.choice([1, 4, 16, 32]))
    while G * B > 256:
        G = max(1, G // 2)
    L = int(rng.integers(1, 1200 if dtype == "f32" else 6000))
    k = int(rng.integers(1, min(L, 700) + 1))
    w = Workload(f"rnd{seed}", dtype, Hq=Hkv * G, Hkv=Hkv, d=d, L=L, B=B, ks=(k,), T=2, heavy_frac=0.02, heavy_scale=3.0)
    _run_workload(oracle_mod, w, seed=9000 + seed)


@pytest.mark.parametrize("case", [
    # long single-row-group loops (the scores-one-tile-ahead order of the attention kernel) with a
    # ragged last tile, for both head dimensions
    ("a1", "bf16", 8, 8, 64, 49152 + 37, 32, 128),
    ("a2", "bf16", 16, 8, 128, 65536 + 1, 32, 256),
])
def test_long_single_row_group_loops(oracle_mod, case):
    from gpu_util import Problem, check_alpha, check_index_sets, check_out
    name, dtype, Hq, Hkv, d, L, B, k = case
    w = Workload(name, dtype, Hq=Hq, Hkv=Hkv, d=d, L=L, B=B, ks=(k,), T=2, heavy_frac=0.01, heavy_scale=4.0)
    x = make_layer(w, 4100 + len(name) + d, steps=2)
    print(f"[parity] {name} L={L} d={d}", flush=True)
    p = Problem(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0], k, dtype)
    o, l = p.exact()
    o1, l1, idx, alpha = p.step1()
    o_ref, l_ref = oracle_mod.exact_attn(x["q"][0], x["k_cache"], x["v_cache"], x["k_blk"][0], x["v_blk"][0])
    check_out(o, o_ref, l, l_ref, dtype)
    check_out(o1, o_ref, l1, l_ref, dtype)
    ref = oracle_mod.select(x["q"][0], x["k_cache"], k)
    check_alpha(alpha, ref["alpha32"])
    check_index_sets(idx, ref["idx"], ref["alpha32"], L)


@pytest.mark.parametrize("case", [
    # name, dtype, Hq, Hkv, d, L, B  -- per-query-head block averages (Eq. 2 per head)
    ("p1", "bf16", 8, 2, 128, 1000, 32),       # B = 32: one wavefront per head
    ("p2", "bf16", 14, 2, 64, 777, 5),          # G = 7, B = 5: a head's rows sit inside one M tile
    ("p3", "bf16", 4, 4, 128, 300, 48),         # B = 48: two M tiles, the second ragged
    ("p4", "bf16", 1, 1, 128, 4097, 130),       # B > 128: the eight-wavefront column sums
    ("p5", "f32", 6, 2, 64, 700, 7),
    ("p6", "f32", 4, 1, 128, 129, 70),          # B > 64: two fp32 row groups per head
])
def test_block_probs_per_query_head(oracle_mod, case):
    from gpu_util import Problem, check_alpha
    name, dtype, Hq, Hkv, d, L, B = case
    w = Workload(name, dtype, Hq=Hq, Hkv=Hkv, d=d, L=L, B=B, ks=(1,), T=2, heavy_frac=0.02, heavy_scale=3.0)
    x = make_layer(w, 5200 + L, steps=1)
    p = Problem(x["q"][0], x["k_cache"], x["v_cache"], None, None, 1, dtype)
    pbar = p.block_probs()
    pbar_ref, alpha_ref = oracle_mod.block_probs(x["q"][0], x["k_cache"])
    assert pbar.shape == (Hq, L)
    check_alpha(pbar, pbar_ref.astype(np.float32))            # rows sum to 1, relative error per entry
    # the mean over a KV head's group is the alpha that mage_select ranks
    _, alpha = p.select()
    G = Hq // Hkv
    np.testing.assert_allclose(pbar.reshape(Hkv, G, L).mean(axis=1), alpha, rtol=2e-5, atol=1e-9)
