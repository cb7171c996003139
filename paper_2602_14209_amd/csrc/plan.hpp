// Host-side launch plans and workspace layout for the MAGE kernels (gfx950).
//
// A plan is a pure function of the problem geometry, so mage_workspace_bytes() and the
// launchers always agree.  Partial results of split attention live in the caller's workspace:
//   part_o [Hkv][n_split][rpad][d] fp32  unnormalised weighted value sums
//   part_m [Hkv][n_split][rpad]    fp32  running maximum of the log2-scaled logits
//   part_l [Hkv][n_split][rpad]    fp32  sum of exp2(logit2 - part_m)
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/mage.h"

namespace mage {

constexpr int kBf16Tile = 64;   // keys per LDS tile, MFMA path
constexpr int kF32Tile = 32;    // keys per LDS tile, fp32 vector path
constexpr int kF32Rows = 64;    // query rows per workgroup, fp32 vector path
constexpr int kTargetWorkgroups = 512;   // fp32 vector path: 2 per CU on 256 CUs
constexpr int kBf16Workgroups = 256;     // MFMA path: one 8-wavefront workgroup per CU (its tile ring fills the LDS)
constexpr int kStatsWorkgroups = 512;    // MFMA selection passes (row statistics, column sums): two per CU
constexpr int kSelectWorkgroups = 2048;  // fp32 selection passes: 8 per CU

struct SplitPlan {
    int R;            // query rows sharing one KV head: G*B
    int rows_per_wg;  // rows one workgroup covers
    int row_groups;   // workgroups along the row axis
    int rpad;         // row_groups * rows_per_wg
    int waves;        // wavefronts per workgroup of the column-sum pass (one per 32 rows; MFMA path)
    int tile;         // keys per tile
    int kps;          // cache keys per split (multiple of tile)
    int n_split;      // splits along the key axis, including a block-only split if any
    int n_cyc;        // splits that own cache keys (the first n_cyc)
    int blk_split;    // split that also attends the in-block keys
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

inline void plan_rows(const mage_shape &s, SplitPlan &p)
{
    p.R = (s.Hq / s.Hkv) * s.B;
    if (s.dtype == MAGE_BF16) {
        p.rows_per_wg = 128;
        p.waves = p.R > 128 ? 8 : 4;
        p.tile = kBf16Tile;
    } else {
        p.waves = 4;
        p.rows_per_wg = kF32Rows;
        p.tile = kF32Tile;
    }
    p.row_groups = ceil_div(p.R, p.rows_per_wg);
    p.rpad = p.row_groups * p.rows_per_wg;
}

// Dense pass over all L cache keys.  Exact attention pays a [rows x d] partial per split, so it
// aims at two workgroups per CU; the two passes of selection leave only a (max, sum) pair per
// row and split, so they cut the keys much finer (more workgroups in flight, even tail).
inline SplitPlan plan_dense(const mage_shape &s, int target_workgroups = 0, bool rows_in_one_workgroup = false)
{
    SplitPlan p{};
    plan_rows(s, p);
    if (target_workgroups == 0) target_workgroups = s.dtype == MAGE_BF16 ? kBf16Workgroups : kTargetWorkgroups;
    const int64_t tiles = (s.L + p.tile - 1) / p.tile;
    const int64_t per_split = (int64_t)s.Hkv * (rows_in_one_workgroup ? 1 : p.row_groups);   // workgroups per key split
    const int64_t target = target_workgroups / per_split > 0 ? target_workgroups / per_split : 1;
    int64_t tps = (tiles + target - 1) / target;     // tiles per split
    const int64_t min_tps = s.dtype == MAGE_BF16 ? 4 : 8;
    if (tps < min_tps) tps = min_tps;
    p.n_split = (int)((tiles + tps - 1) / tps);
    p.kps = (int)(tps * p.tile);
    p.blk_split = p.n_split - 1;
    p.n_cyc = p.n_split;
    return p;
}

// Selection, first pass (row statistics).  The fp32 vector path uses one plan for both passes.
inline SplitPlan plan_stats(const mage_shape &s)
{
    return plan_dense(s, s.dtype == MAGE_BF16 ? kStatsWorkgroups : kSelectWorkgroups);
}

// Selection, second pass (column sums).  The MFMA kernel parks the sums of up to kColsumTiles tiles
// in LDS and writes them out together.  Like the statistics pass it wants long splits (every
// workgroup pays a pipeline fill) and a power-of-two number of them.
constexpr int kColsumTiles = 8;
constexpr int kGroupKeys = 16;           // keys per group maximum handed from the column sums to the top-k filter
// The MFMA kernel keeps all rows of a KV head in one workgroup (4 or 8 wavefronts); its registers
// and LDS let three 4-wavefront or two 8-wavefront workgroups share a CU.
constexpr int kColsumWorkgroups4 = 768, kColsumWorkgroups8 = 512;
inline SplitPlan plan_colsum(const mage_shape &s)
{
    if (s.dtype != MAGE_BF16) return plan_dense(s, kSelectWorkgroups);
    const int R = (s.Hq / s.Hkv) * s.B;
    return plan_dense(s, R > 128 ? kColsumWorkgroups8 : kColsumWorkgroups4, true);
}

// Sparse step: k gathered cache keys, in-block keys in a split of their own when k is large
// enough for the gather splits to be full tiles.
inline SplitPlan plan_sparse(const mage_shape &s)
{
    SplitPlan p{};
    plan_rows(s, p);
    const int64_t tiles = ((int64_t)s.k + p.tile - 1) / p.tile;
    const int64_t max_splits = 8;
    const int64_t tps = (tiles + max_splits - 1) / max_splits;
    const int n_cache = (int)((tiles + tps - 1) / tps);
    p.kps = (int)(tps * p.tile);
    p.n_cyc = n_cache;
    if (s.k >= p.tile) {
        p.n_split = n_cache + 1;
        p.blk_split = n_cache;
    } else {
        p.n_split = n_cache;
        p.blk_split = n_cache - 1;
    }
    return p;
}

inline size_t partial_bytes(const mage_shape &s, const SplitPlan &p)
{
    const size_t rows = (size_t)s.Hkv * p.n_split * p.rpad;
    return align_up(rows * s.d * sizeof(float), 256) + 2 * align_up(rows * sizeof(float), 256);
}

struct SelectLayout {
    size_t part_m, part_l, lse2, alpha, gmax, bytes;
};

inline SelectLayout select_layout(const mage_shape &s, const SplitPlan &p)
{
    SelectLayout l{};
    const size_t rows = (size_t)s.Hkv * p.n_split * p.rpad;
    size_t off = 0;
    l.part_m = off; off += align_up(rows * sizeof(float), 256);
    l.part_l = off; off += align_up(rows * sizeof(float), 256);
    l.lse2 = off;   off += align_up((size_t)s.Hkv * p.rpad * sizeof(float), 256);
    l.alpha = off;  off += align_up((size_t)s.Hkv * (size_t)s.L * sizeof(float), 256);
    l.gmax = off;   off += align_up((size_t)s.Hkv * (size_t)((s.L + kGroupKeys - 1) / kGroupKeys) * sizeof(float), 256);
    l.bytes = off;
    return l;
}

// Fused step 1 (exact attention that also feeds selection): the attention partials, then the
// prefix statistics per attention split, then selection's lse2 and alpha.
struct Step1Layout {
    size_t partials, stat_m, stat_l, lse2, alpha, gmax, bytes;
};

inline Step1Layout step1_layout(const mage_shape &s, const SplitPlan &attn)
{
    Step1Layout l{};
    const size_t rows = (size_t)s.Hkv * attn.n_split * attn.rpad;
    size_t off = 0;
    l.partials = off; off += partial_bytes(s, attn);
    l.stat_m = off;   off += align_up(rows * sizeof(float), 256);
    l.stat_l = off;   off += align_up(rows * sizeof(float), 256);
    l.lse2 = off;     off += align_up((size_t)s.Hkv * attn.rpad * sizeof(float), 256);
    l.alpha = off;    off += align_up((size_t)s.Hkv * (size_t)s.L * sizeof(float), 256);
    l.gmax = off;     off += align_up((size_t)s.Hkv * (size_t)((s.L + kGroupKeys - 1) / kGroupKeys) * sizeof(float), 256);
    l.bytes = off;
    return l;
}

// Arguments shared by the attention / statistics / column-sum kernels of both element types.
struct KernelArgs {
    const void *q, *kc, *vc, *kblk, *vblk;
    const int32_t *idx;      // gather indices [Hkv][nc] or nullptr
    float *out, *lse_out;    // final outputs (used directly when n_split == 1)
    float *part_o, *part_m, *part_l;
    float *stat_m, *stat_l;  // exact attention, optional: prefix-only (cache keys) statistics per split, as part_m/part_l
    const float *lse2;       // column-sum pass: per-row log2-domain log-sum-exp [Hkv][rpad]
    float *lse2_out;         // combine, optional: the same, merged from stat_m / stat_l
    float *alpha;            // column-sum pass: [Hkv][L] (or [Hq][L] with head_rows)
    int head_rows;           // column-sum pass: 0, or B = one grid row per QUERY head, summing that head's B rows only (Eq. 2 per head)
    float *gmax;             // column-sum pass, optional: [Hkv][ceil(L / kGroupKeys)] maxima of alpha over groups of consecutive keys
    int B, Hq, Hkv, G, R, rpad;
    long long L;             // rows in the cache
    long long nc;            // cache keys attended: L (dense) or k (gather)
    int kps, n_split, blk_split, n_blk;
    int n_cyc;               // MFMA path: split s < n_cyc owns the cache tiles s, s + n_cyc, s + 2*n_cyc, ...
    // batched launches (grid z = sequence): element strides between consecutive sequences, 0 when not batched
    long long seq_q, seq_kv, seq_idx, seq_blk, seq_out, seq_lse;
    float scale_log2;        // log2(e) / sqrt(d)
    float inv_rows;          // 1 / (G*B)
    // worked out on the host so that the bf16 kernels start without a division (fill_split_consts):
    int tiles_q, tiles_r;    // ceil(nc / 64) cache tiles = tiles_q * n_cyc + tiles_r
    unsigned inv_B;          // ceil(2^32 / B) for B >= 2: row / B == (row * inv_B) >> 32 while row * B < 2^32
};

// What the top-k kernel needs to re-score the few candidates whose fp32 alpha lies within `eps`
// (relative) of the k-th value in fp64 from the inputs (see topk.hip); q == nullptr switches it off.
struct RescoreArgs {
    const void *q, *kc;              // queries [B,Hq,d], keys [L,Hkv,d]
    const float *stat_m, *stat_l;    // row statistics per key split [Hkv][n_split][rpad], log2 domain
    int esz;                         // bytes per element of q / kc: 2 (bf16) or 4 (fp32)
    int d, Hq, Hkv, G, B, R, n_split, rpad;
    float scale_log2;                // the factor the statistics were taken with
    double inv_rows;                 // 1 / (R * key weight)
    float eps;
};

}  // namespace mage
