"""Writes tests/golden/worked_example.json: a tiny hand-written problem and what the CPU oracle computes
for it.  Calls nothing but `oracle/` (never the HIP library).  Run from the repository root:

    python tests/golden/make_worked_example.py

The paper (arxiv 2602.14209) prints no numeric input/output pair for any step of Alg. 1, so there is
nothing of the paper's to store; this fixture pins the oracle against accidental change and gives a
reader a case small enough to follow by hand: d = 64 with only channels 0 and 1 non-zero, so a logit is
(q0*k0 + q1*k1) / 8 (Alg. 1: softmax(Q K^T / sqrt(d)), Eq. 5 averaging, Top-k with ties to the
smaller index).  Floats are stored as C99 hex strings, exactly."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

B, Hq, Hkv, d, L, k = 2, 2, 1, 64, 6, 2


def inputs():
    q = np.zeros((B, Hq, d), np.float32)
    q[0, 0, :2] = (8, 0)
    q[0, 1, :2] = (0, 8)
    q[1, 0, :2] = (8, 8)
    q[1, 1, :2] = (-8, 0)
    kc = np.zeros((L, Hkv, d), np.float32)
    for j, (a, b) in enumerate([(1, 0), (0, 1), (1, 1), (-1, 0), (2, 0), (1, 0)]):   # rows 0 and 5 are equal: a tie
        kc[j, 0, :2] = (a, b)
    vc = np.zeros((L, Hkv, d), np.float32)
    vc[:, 0, 0] = np.arange(L, dtype=np.float32)           # channel 0 reads off the expected position
    vc[:, 0, 1] = 1.0
    kb = np.zeros((B, Hkv, d), np.float32)
    kb[0, 0, :2] = (0, 2)
    kb[1, 0, :2] = (0, 0)
    vb = np.zeros((B, Hkv, d), np.float32)
    vb[:, 0, 0] = (10.0, 20.0)
    vb[:, 0, 1] = 1.0
    return q, kc, vc, kb, vb


def compute():
    q, kc, vc, kb, vb = inputs()
    oracle.build()
    sel = oracle.select(q, kc, k)
    pbar, alpha = oracle.block_probs(q, kc)
    o_exact, lse_exact = oracle.exact_attn(q, kc, vc, kb, vb)
    o_sparse, lse_sparse = oracle.sparse_attn(q, kc, vc, sel["idx"], kb, vb)
    hexs = lambda a: [float(x).hex() for x in np.asarray(a, np.float64).ravel()]
    return {
        "citation": "Alg. 1 (select stream, Phase 2), Eq. 2, Eq. 5 of arxiv 2602.14209; values computed by oracle/, not printed in the paper",
        "shape": {"B": B, "Hq": Hq, "Hkv": Hkv, "d": d, "L": L, "k": k},
        "nonzero_channels": {"q": q[:, :, :2].tolist(), "k_cache": kc[:, 0, :2].tolist(), "v_cache": vc[:, 0, :2].tolist(),
                             "k_blk": kb[:, 0, :2].tolist(), "v_blk": vb[:, 0, :2].tolist()},
        "idx": np.asarray(sel["idx"]).tolist(),
        "alpha_fp64": hexs(alpha),
        "pbar_fp64": hexs(pbar),
        "exact_out_channels01": hexs(o_exact[:, :, :2]),
        "exact_lse": hexs(lse_exact),
        "sparse_out_channels01": hexs(o_sparse[:, :, :2]),
        "sparse_lse": hexs(lse_sparse),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "worked_example.json")
    json.dump(compute(), open(out, "w"), indent=1)
    print("wrote", out)
