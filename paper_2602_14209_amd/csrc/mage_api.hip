// C ABI of the MAGE hot path (declared in include/mage.h): host-side validation, launch plans,
// workspace carving and kernel dispatch.  Nothing here allocates or synchronises.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "plan.hpp"

namespace mage {
hipError_t bf16_attn(const KernelArgs &a, int d, int row_groups, hipStream_t stream);
hipError_t bf16_sparse_batched(const KernelArgs &a, int d, int row_groups, int n_seq, hipStream_t stream);
hipError_t bf16_stats(const KernelArgs &a, int d, int row_groups, hipStream_t stream);
hipError_t bf16_colsum(const KernelArgs &a, int d, int waves, hipStream_t stream);
hipError_t bf16_sparse(const KernelArgs &a, int d, bool compact, hipStream_t stream);
hipError_t launch_compact(const void *k_src, const void *v_src, const int32_t *idx, void *k_dst, void *v_dst,
                          int Hkv, int d, int k, int esz, hipStream_t stream);
hipError_t f32_attn(const KernelArgs &a, int d, int row_groups, bool gather, hipStream_t stream);
hipError_t f32_stats(const KernelArgs &a, int d, int row_groups, hipStream_t stream);
hipError_t f32_colsum(const KernelArgs &a, int d, hipStream_t stream);
hipError_t launch_combine(const KernelArgs &a, int d, hipStream_t stream);
hipError_t launch_lse(const KernelArgs &a, float *lse2_out, hipStream_t stream);
hipError_t launch_page_summary(const void *kc, void *out, long long L, int Hkv, int d, int p, bool bf16, hipStream_t stream);
hipError_t launch_quest_query(const void *q, void *q2, long long rows, int d, hipStream_t stream);
hipError_t launch_expand_pages(const int32_t *pages, int32_t *idx, int Hkv, int k, int p, hipStream_t stream);
hipError_t launch_overlap(const int32_t *a, const int32_t *b, int n_rows, int k, int a_rows, float *out, hipStream_t stream);
hipError_t launch_topk(const float *alpha, const float *group_max, int Hkv, long long L, int k, int32_t *idx_out, const RescoreArgs &rs,
                       hipStream_t stream);
}  // namespace mage

using namespace mage;

namespace {

constexpr int64_t kMaxL = (int64_t)1 << 30;
// Candidates this close (relative) to the k-th averaged probability are re-scored in fp64.  The fp32
// alpha of the kernels is within 1e-6 (relative) of the exact value (measured at the 32K..128K shapes:
// median 7e-8, largest 7e-7), so two candidates further apart than this band are ranked correctly.
constexpr float kNearTieBand = 4e-6f;

// The inputs and row statistics the top-k kernel re-scores near-ties from.
RescoreArgs rescore_args(const mage_shape &s, const KernelArgs &a, const float *stat_m, const float *stat_l, int n_split, int rpad,
                         float scale_log2, int key_weight)
{
    RescoreArgs r{};
    r.q = a.q;
    r.kc = a.kc;
    r.stat_m = stat_m;
    r.stat_l = stat_l;
    r.esz = s.dtype == MAGE_BF16 ? 2 : 4;
    r.d = s.d;
    r.Hq = s.Hq;
    r.Hkv = s.Hkv;
    r.G = s.Hq / s.Hkv;
    r.B = s.B;
    r.R = r.G * s.B;
    r.n_split = n_split;
    r.rpad = rpad;
    r.scale_log2 = scale_log2;
    r.inv_rows = 1.0 / ((double)r.R * (double)key_weight);
    r.eps = kNearTieBand;
    return r;
}

int check_shape(const mage_shape *s, bool need_k)
{
    if (!s) return MAGE_ERR_NULL;
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->d <= 0 || s->L <= 0) return MAGE_ERR_SHAPE;
    if (s->Hq % s->Hkv != 0) return MAGE_ERR_SHAPE;
    if (need_k && (s->k <= 0 || (int64_t)s->k > s->L)) return MAGE_ERR_SHAPE;
    if (s->d != 64 && s->d != 128) return MAGE_ERR_UNSUPPORTED;
    if (s->dtype != MAGE_F32 && s->dtype != MAGE_BF16) return MAGE_ERR_UNSUPPORTED;
    if (s->L > kMaxL) return MAGE_ERR_UNSUPPORTED;
    const int64_t rows = (int64_t)(s->Hq / s->Hkv) * s->B;      // query rows that share a KV head
    if (rows > (1 << 20)) return MAGE_ERR_UNSUPPORTED;
    // what the kernels' 32-bit arithmetic assumes: row / B by a multiply-high, row strides in bytes
    if (rows * s->B >= ((int64_t)1 << 32) || (int64_t)s->Hkv * s->d * 4 >= ((int64_t)1 << 31)) return MAGE_ERR_UNSUPPORTED;
    return MAGE_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

KernelArgs base_args(const mage_shape &s, const SplitPlan &p)
{
    KernelArgs a{};
    a.B = s.B;
    a.Hq = s.Hq;
    a.Hkv = s.Hkv;
    a.G = s.Hq / s.Hkv;
    a.R = p.R;
    a.rpad = p.rpad;
    a.L = s.L;
    a.kps = p.kps;
    a.n_split = p.n_split;
    a.blk_split = p.blk_split;
    a.n_cyc = p.n_cyc;
    a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)s.d));
    a.inv_rows = (float)(1.0 / (double)p.R);
    return a;
}

void carve_partials(const mage_shape &s, const SplitPlan &p, void *workspace, KernelArgs &a)
{
    const size_t rows = (size_t)s.Hkv * p.n_split * p.rpad;
    char *w = static_cast<char *>(workspace);
    a.part_o = reinterpret_cast<float *>(w);
    w += align_up(rows * s.d * sizeof(float), 256);
    a.part_m = reinterpret_cast<float *>(w);
    w += align_up(rows * sizeof(float), 256);
    a.part_l = reinterpret_cast<float *>(w);
}

// Launch-free argument check of an attention call (exact, or sparse through the tiled kernels).
int attention_check(const mage_shape *shape, const SplitPlan &p, bool gather,
                    const void *q, const void *k_cache, const void *v_cache, const int32_t *idx,
                    const void *k_blk, const void *v_blk, const float *out,
                    const void *workspace, size_t workspace_bytes)
{
    if (!q || !k_cache || !v_cache || !out || (gather && !idx)) return MAGE_ERR_NULL;
    if (gather && shape->dtype == MAGE_BF16) return MAGE_ERR_UNSUPPORTED;     // bf16 gathers rows in the sparse kernels, not here
    if ((k_blk == nullptr) != (v_blk == nullptr)) return MAGE_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_blk) || !aligned16(v_blk) ||
        !aligned16(out) || !aligned16(workspace))
        return MAGE_ERR_ALIGN;
    if (p.n_split > 1 && (!workspace || workspace_bytes < partial_bytes(*shape, p))) return MAGE_ERR_WORKSPACE;
    return MAGE_OK;
}

int run_attention(const mage_shape *shape, const SplitPlan &p, bool gather,
                  const void *q, const void *k_cache, const void *v_cache, const int32_t *idx,
                  const void *k_blk, const void *v_blk, float *out, float *lse_out,
                  void *workspace, size_t workspace_bytes, void *hip_stream,
                  float *stat_m = nullptr, float *stat_l = nullptr, float *lse2_out = nullptr)
{
    const int rc = attention_check(shape, p, gather, q, k_cache, v_cache, idx, k_blk, v_blk, out, workspace, workspace_bytes);
    if (rc != MAGE_OK) return rc;

    KernelArgs a = base_args(*shape, p);
    a.q = q;
    a.kc = k_cache;
    a.vc = v_cache;
    // with no in-block keys the block pointers are never dereferenced; keep them valid anyway
    a.kblk = k_blk ? k_blk : k_cache;
    a.vblk = v_blk ? v_blk : v_cache;
    a.n_blk = k_blk ? shape->B : 0;
    a.idx = idx;
    a.nc = gather ? (long long)shape->k : (long long)shape->L;
    a.out = out;
    a.lse_out = lse_out;
    a.stat_m = stat_m;
    a.stat_l = stat_l;
    a.lse2_out = p.n_split > 1 ? lse2_out : nullptr;
    if (p.n_split > 1) carve_partials(*shape, p, workspace, a);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = shape->dtype == MAGE_BF16 ? bf16_attn(a, shape->d, p.row_groups, stream)
                                             : f32_attn(a, shape->d, p.row_groups, gather, stream);
    if (e != hipSuccess) return MAGE_ERR_HIP;
    if (p.n_split > 1) {
        e = launch_combine(a, shape->d, stream);
        if (e != hipSuccess) return MAGE_ERR_HIP;
    }
    return MAGE_OK;
}

// bf16 sparse step: one kernel, partials merged on chip, no workspace.  `compact`: the cache
// argument already holds the k selected rows; n_seq > 1: strided batch of independent sequences.
int run_sparse_bf16(const mage_shape *shape, bool compact, int n_seq, const void *q, const void *k_cache,
                    const void *v_cache, const int32_t *idx, const void *k_blk, const void *v_blk,
                    float *out, float *lse_out, void *hip_stream)
{
    if (!q || !k_cache || !v_cache || !out || (!compact && !idx)) return MAGE_ERR_NULL;
    if ((k_blk == nullptr) != (v_blk == nullptr)) return MAGE_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_blk) || !aligned16(v_blk) ||
        !aligned16(out))
        return MAGE_ERR_ALIGN;
    SplitPlan p{};
    plan_rows(*shape, p);
    p.n_split = 1;
    p.n_cyc = 1;
    KernelArgs a = base_args(*shape, p);
    a.q = q;
    a.kc = k_cache;
    a.vc = v_cache;
    a.kblk = k_blk ? k_blk : k_cache;
    a.vblk = v_blk ? v_blk : v_cache;
    a.n_blk = k_blk ? shape->B : 0;
    a.idx = idx;
    a.nc = shape->k;
    a.out = out;
    a.lse_out = lse_out;
    if (n_seq > 1) {
        a.seq_q = (long long)shape->B * shape->Hq * shape->d;
        a.seq_kv = (long long)shape->L * shape->Hkv * shape->d;
        a.seq_idx = (long long)shape->Hkv * shape->k;
        a.seq_blk = k_blk ? (long long)shape->B * shape->Hkv * shape->d : 0;
        a.seq_out = a.seq_q;
        a.seq_lse = (long long)shape->B * shape->Hq;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (n_seq > 1 && !compact) {
        // enough independent work to fill the chip: one workgroup per (sequence, head) reads every
        // selected row once (the latency-oriented kernel re-reads it per row tile)
        return bf16_sparse_batched(a, shape->d, p.row_groups, n_seq, stream) == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
    }
    if (n_seq != 1) return MAGE_ERR_UNSUPPORTED;            // compacted rows: one sequence per call
    if (bf16_sparse(a, shape->d, compact, stream) != hipSuccess) return MAGE_ERR_HIP;
    return MAGE_OK;
}

// The selection pipeline (row statistics, log-sum-exp, column sums, top-k) on a validated
// geometry.  `scale_log2` = log2(e) times the factor on the logit; `key_weight`: every key stands for
// that many positions of equal score (its probability is shared among them); shape->d may be 256
// here (page-summary rows).
// Launch-free argument check of the selection pipeline (everything select_impl can reject).
int select_check(const mage_shape *shape, const void *q1, const void *k_cache,
                 const int32_t *idx_out, const float *alpha_out, const float *pbar_out,
                 const void *workspace, size_t workspace_bytes)
{
    if (!q1 || !k_cache || (!idx_out && !pbar_out)) return MAGE_ERR_NULL;
    const SplitPlan p = plan_stats(*shape);
    if (shape->dtype == MAGE_BF16 && p.rpad > 256) return MAGE_ERR_UNSUPPORTED;   // the column-sum pass keeps all rows of a head in one workgroup
    if (!aligned16(q1) || !aligned16(k_cache) || !aligned16(workspace) || !aligned16(alpha_out) || !aligned16(pbar_out)) return MAGE_ERR_ALIGN;
    if (!workspace || workspace_bytes < select_layout(*shape, p).bytes) return MAGE_ERR_WORKSPACE;
    return MAGE_OK;
}

int select_impl(const mage_shape *shape, float scale_log2, int key_weight, const void *q1, const void *k_cache,
                int32_t *idx_out, float *alpha_out, float *pbar_out,
                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const int rc = select_check(shape, q1, k_cache, idx_out, alpha_out, pbar_out, workspace, workspace_bytes);
    if (rc != MAGE_OK) return rc;
    const SplitPlan p = plan_stats(*shape), pc = plan_colsum(*shape);
    const SelectLayout lay = select_layout(*shape, p);

    char *w = static_cast<char *>(workspace);
    KernelArgs a = base_args(*shape, p);
    a.scale_log2 = scale_log2;
    a.inv_rows /= (float)key_weight;
    a.q = q1;
    a.kc = k_cache;
    a.vc = k_cache;
    a.kblk = k_cache;
    a.vblk = k_cache;
    a.n_blk = 0;
    a.blk_split = -1;
    a.nc = shape->L;
    a.part_m = reinterpret_cast<float *>(w + lay.part_m);
    a.part_l = reinterpret_cast<float *>(w + lay.part_l);
    float *lse2 = reinterpret_cast<float *>(w + lay.lse2);
    a.lse2 = lse2;
    a.alpha = alpha_out ? alpha_out : reinterpret_cast<float *>(w + lay.alpha);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool bf = shape->dtype == MAGE_BF16;
    a.gmax = bf ? reinterpret_cast<float *>(w + lay.gmax) : nullptr;   // the MFMA column sums also leave group maxima for the top-k filter
    hipError_t e = bf ? bf16_stats(a, shape->d, p.row_groups, stream) : f32_stats(a, shape->d, p.row_groups, stream);
    if (e != hipSuccess) return MAGE_ERR_HIP;
    e = launch_lse(a, lse2, stream);
    if (e != hipSuccess) return MAGE_ERR_HIP;
    KernelArgs c = a;                                // the column sums have their own split of the keys
    c.kps = pc.kps;
    c.n_split = pc.n_split;
    c.n_cyc = pc.n_cyc;
    if (idx_out) {
        e = bf ? bf16_colsum(c, shape->d, pc.waves, stream) : f32_colsum(c, shape->d, stream);
        if (e != hipSuccess) return MAGE_ERR_HIP;
        e = launch_topk(a.alpha, a.gmax, shape->Hkv, shape->L, shape->k, idx_out,
                        rescore_args(*shape, a, a.part_m, a.part_l, p.n_split, p.rpad, scale_log2, key_weight), stream);
        if (e != hipSuccess) return MAGE_ERR_HIP;
    }
    if (pbar_out) {                                  // the same sums restricted to the B rows of one query head at a time
        c.head_rows = shape->B;
        c.alpha = pbar_out;
        c.gmax = nullptr;
        c.inv_rows = 1.f / ((float)shape->B * (float)key_weight);
        e = bf ? bf16_colsum(c, shape->d, shape->B > 128 ? 8 : 4, stream) : f32_colsum(c, shape->d, stream);
        if (e != hipSuccess) return MAGE_ERR_HIP;
    }
    return MAGE_OK;
}


}  // namespace

extern "C" {

int mage_version(void) { return 100; }

const char *mage_status_string(int status)
{
    switch (status) {
    case MAGE_OK: return "ok";
    case MAGE_ERR_NULL: return "a required pointer is NULL";
    case MAGE_ERR_SHAPE: return "invalid shape (non-positive size, Hq % Hkv != 0, or k > L)";
    case MAGE_ERR_UNSUPPORTED: return "unsupported configuration (d not in {64,128}, unknown dtype, L > 2^30, or B, G or Hkv beyond the kernels' 32-bit ranges)";
    case MAGE_ERR_WORKSPACE: return "workspace missing or smaller than mage_workspace_bytes()";
    case MAGE_ERR_HIP: return "HIP reported a launch error";
    case MAGE_ERR_ALIGN: return "a data pointer is not 16-byte aligned";
    case MAGE_ERR_SCRATCH: return "the problem needs more scratch memory than the library's static buffer holds";
    default: return "unknown status";
    }
}

size_t mage_workspace_bytes(const mage_shape *shape)
{
    if (check_shape(shape, true) != MAGE_OK) return 0;
    const SplitPlan dense = plan_dense(*shape), sparse = plan_sparse(*shape);
    size_t need = partial_bytes(*shape, dense);
    const size_t b = partial_bytes(*shape, sparse);
    if (b > need) need = b;
    const size_t c = select_layout(*shape, plan_stats(*shape)).bytes;
    if (c > need) need = c;
    const size_t e = step1_layout(*shape, dense).bytes;
    if (e > need) need = e;
    return need;
}

int mage_select(const mage_shape *shape, const void *q1, const void *k_cache,
                int32_t *idx_out, float *alpha_out,
                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    return select_impl(shape, (float)(1.4426950408889634 / sqrt((double)shape->d)), 1, q1, k_cache, idx_out, alpha_out, nullptr,
                       workspace, workspace_bytes, hip_stream);
}

}  // extern "C"

// ---- selection without a caller-provided workspace ----
// The selection kernels' scratch data (row statistics per key split, alpha when the caller does not
// ask for it, the group maxima) live in this file-scope device array instead: every GPU the library runs
// on holds its own copy at its own address for the life of the process.  Host code must not use the
// array's name as a device address (in host code it is only a handle); the address on each device
// is asked for once, with that device current, and kept.
namespace {

constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];        // device address of `scratch` on each device, nullptr = not asked yet
std::mutex g_scratch_mutex;

// Address of this device's copy of the scratch array (the current device's), or nullptr on error.
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

size_t mage_static_scratch_bytes(void) { return kStaticScratchBytes; }

int mage_select_static(const mage_shape *shape, const void *q1, const void *k_cache,
                       int32_t *idx_out, float *alpha_out, void *hip_stream)
{
    const int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    if (select_layout(*shape, plan_stats(*shape)).bytes > kStaticScratchBytes) return MAGE_ERR_SCRATCH;
    // everything but the workspace, so that argument errors are reported without touching the device
    const int ra = select_check(shape, q1, k_cache, idx_out, alpha_out, nullptr, reinterpret_cast<const void *>(256), kStaticScratchBytes);
    if (ra != MAGE_OK) return ra;
    void *ws = static_scratch();
    if (!ws) return MAGE_ERR_HIP;
    return select_impl(shape, (float)(1.4426950408889634 / sqrt((double)shape->d)), 1, q1, k_cache, idx_out, alpha_out, nullptr,
                       ws, kStaticScratchBytes, hip_stream);
}

int mage_block_probs(const mage_shape *shape, const void *q1, const void *k_cache, float *pbar_out,
                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    if (!pbar_out) return MAGE_ERR_NULL;
    return select_impl(shape, (float)(1.4426950408889634 / sqrt((double)shape->d)), 1, q1, k_cache, nullptr, nullptr, pbar_out,
                       workspace, workspace_bytes, hip_stream);
}

int mage_step1(const mage_shape *shape, const void *q1, const void *k_cache, const void *v_cache,
               const void *k_blk, const void *v_blk, float *out, float *lse_out, int32_t *idx_out, float *alpha_out,
               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    if (!idx_out) return MAGE_ERR_NULL;
    if (shape->dtype != MAGE_BF16) {
        // fp32: the two calls back to back (no shared pass in the vector path); both are validated
        // before the first one launches anything
        rc = select_check(shape, q1, k_cache, idx_out, alpha_out, nullptr, workspace, workspace_bytes);
        if (rc != MAGE_OK) return rc;
        rc = run_attention(shape, plan_dense(*shape), false, q1, k_cache, v_cache, nullptr, k_blk, v_blk, out, lse_out,
                           workspace, workspace_bytes, hip_stream);
        if (rc != MAGE_OK) return rc;
        return mage_select(shape, q1, k_cache, idx_out, alpha_out, workspace, workspace_bytes, hip_stream);
    }
    const SplitPlan pa = plan_dense(*shape);
    const SplitPlan ps = plan_colsum(*shape);
    if (ps.rpad > 256) return MAGE_ERR_UNSUPPORTED;
    if (!aligned16(alpha_out)) return MAGE_ERR_ALIGN;
    const Step1Layout lay = step1_layout(*shape, pa);
    if (!workspace || workspace_bytes < lay.bytes) return MAGE_ERR_WORKSPACE;
    char *w = static_cast<char *>(workspace);
    float *stat_m = reinterpret_cast<float *>(w + lay.stat_m), *stat_l = reinterpret_cast<float *>(w + lay.stat_l);
    float *lse2 = reinterpret_cast<float *>(w + lay.lse2);
    rc = run_attention(shape, pa, false, q1, k_cache, v_cache, nullptr, k_blk, v_blk, out, lse_out,
                       w + lay.partials, lay.stat_m - lay.partials, hip_stream, stat_m, stat_l, lse2);
    if (rc != MAGE_OK) return rc;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (pa.n_split == 1) {                           // unsplit keys: no combine pass ran, merge the one statistics set here
        KernelArgs r = base_args(*shape, pa);
        r.part_m = stat_m;
        r.part_l = stat_l;
        if (launch_lse(r, lse2, stream) != hipSuccess) return MAGE_ERR_HIP;
    }
    KernelArgs a = base_args(*shape, ps);            // column sums on selection's own, finer split
    a.q = q1;
    a.kc = k_cache;
    a.vc = k_cache;
    a.kblk = k_cache;
    a.vblk = k_cache;
    a.n_blk = 0;
    a.blk_split = -1;
    a.nc = shape->L;
    a.lse2 = lse2;
    a.alpha = alpha_out ? alpha_out : reinterpret_cast<float *>(w + lay.alpha);
    a.gmax = reinterpret_cast<float *>(w + lay.gmax);
    if (bf16_colsum(a, shape->d, ps.waves, stream) != hipSuccess) return MAGE_ERR_HIP;
    if (launch_topk(a.alpha, a.gmax, shape->Hkv, shape->L, shape->k, idx_out,
                    rescore_args(*shape, a, stat_m, stat_l, pa.n_split, pa.rpad, a.scale_log2, 1), stream) != hipSuccess)
        return MAGE_ERR_HIP;
    return MAGE_OK;
}

int mage_exact_attn(const mage_shape *shape, const void *q, const void *k_cache, const void *v_cache,
                    const void *k_blk, const void *v_blk, float *out, float *lse_out,
                    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const int rc = check_shape(shape, false);
    if (rc != MAGE_OK) return rc;
    return run_attention(shape, plan_dense(*shape), false, q, k_cache, v_cache, nullptr, k_blk, v_blk, out, lse_out,
                         workspace, workspace_bytes, hip_stream);
}

int mage_sparse_attn(const mage_shape *shape, const void *q, const void *k_cache, const void *v_cache,
                     const int32_t *idx, const void *k_blk, const void *v_blk, float *out, float *lse_out,
                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    if (shape->dtype != MAGE_BF16)
        return run_attention(shape, plan_sparse(*shape), true, q, k_cache, v_cache, idx, k_blk, v_blk, out, lse_out,
                             workspace, workspace_bytes, hip_stream);
    return run_sparse_bf16(shape, false, 1, q, k_cache, v_cache, idx, k_blk, v_blk, out, lse_out, hip_stream);
}

int mage_compact(const mage_shape *shape, const void *k_cache, const void *v_cache, const int32_t *idx,
                 void *k_sel, void *v_sel, void *hip_stream)
{
    const int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    if (!k_cache || !v_cache || !idx || !k_sel || !v_sel) return MAGE_ERR_NULL;
    if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_sel) || !aligned16(v_sel)) return MAGE_ERR_ALIGN;
    const int esz = shape->dtype == MAGE_BF16 ? 2 : 4;
    if (launch_compact(k_cache, v_cache, idx, k_sel, v_sel, shape->Hkv, shape->d, shape->k, esz,
                       static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return MAGE_ERR_HIP;
    return MAGE_OK;
}

int mage_sparse_attn_compact(const mage_shape *shape, const void *q, const void *k_sel, const void *v_sel,
                             const void *k_blk, const void *v_blk, float *out, float *lse_out,
                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    if (shape->dtype != MAGE_BF16) {
        // fp32: the compacted rows are a cache of length k; attend all of it
        mage_shape s = *shape;
        s.L = shape->k;
        return run_attention(&s, plan_dense(s), false, q, k_sel, v_sel, nullptr, k_blk, v_blk, out, lse_out,
                             workspace, workspace_bytes, hip_stream);
    }
    return run_sparse_bf16(shape, true, 1, q, k_sel, v_sel, nullptr, k_blk, v_blk, out, lse_out, hip_stream);
}

int mage_sparse_attn_batched(const mage_shape *shape, int n_seq, const void *q, const void *k_cache,
                             const void *v_cache, const int32_t *idx, const void *k_blk, const void *v_blk,
                             float *out, float *lse_out, void *hip_stream)
{
    const int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    if (n_seq <= 0 || n_seq > 65535) return MAGE_ERR_SHAPE;
    if (shape->dtype != MAGE_BF16) return MAGE_ERR_UNSUPPORTED;
    // (sequence, head) = unit / Hkv by a multiply-high in the kernel
    if (((int64_t)n_seq * shape->Hkv + 8) * shape->Hkv >= ((int64_t)1 << 32)) return MAGE_ERR_UNSUPPORTED;
    return run_sparse_bf16(shape, false, n_seq, q, k_cache, v_cache, idx, k_blk, v_blk, out, lse_out, hip_stream);
}

// ---- second workload: page estimator and overlap ratio ----
namespace {

// geometry of the scoring passes: pages as keys, [max | min] rows of length 2d, k/p pages to select
int quest_shape(const mage_shape *shape, int p, mage_shape &s2)
{
    const int rc = check_shape(shape, true);
    if (rc != MAGE_OK) return rc;
    if (p <= 0) return MAGE_ERR_SHAPE;
    if (shape->dtype != MAGE_BF16 || shape->L % p != 0 || shape->k % p != 0) return MAGE_ERR_UNSUPPORTED;
    s2 = *shape;
    s2.d = 2 * shape->d;
    s2.L = shape->L / p;
    s2.k = shape->k / p;
    return MAGE_OK;
}

struct QuestLayout {
    size_t q2, select, pages, bytes;
};

QuestLayout quest_layout(const mage_shape &shape, const mage_shape &s2)
{
    QuestLayout l{};
    size_t off = 0;
    l.q2 = off;     off += align_up((size_t)shape.B * shape.Hq * s2.d * 2, 256);
    l.select = off; off += align_up(select_layout(s2, plan_stats(s2)).bytes, 256);
    l.pages = off;  off += align_up((size_t)shape.Hkv * s2.k * sizeof(int32_t), 256);
    l.bytes = off;
    return l;
}

}  // namespace

int mage_page_summary(const mage_shape *shape, int p, const void *k_cache, void *summary, void *hip_stream)
{
    const int rc = check_shape(shape, false);
    if (rc != MAGE_OK) return rc;
    if (p <= 0) return MAGE_ERR_SHAPE;
    if (!k_cache || !summary) return MAGE_ERR_NULL;
    if (!aligned16(k_cache) || !aligned16(summary)) return MAGE_ERR_ALIGN;
    const hipError_t e = launch_page_summary(k_cache, summary, shape->L, shape->Hkv, shape->d, p, shape->dtype == MAGE_BF16,
                                             static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

size_t mage_quest_workspace_bytes(const mage_shape *shape, int p)
{
    mage_shape s2;
    if (quest_shape(shape, p, s2) != MAGE_OK) return 0;
    return quest_layout(*shape, s2).bytes;
}

int mage_quest_select(const mage_shape *shape, int p, const void *q, const void *summary,
                      int32_t *idx_out, float *est_out,
                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    mage_shape s2;
    const int rc = quest_shape(shape, p, s2);
    if (rc != MAGE_OK) return rc;
    if (!q || !summary || !idx_out) return MAGE_ERR_NULL;
    if (!aligned16(q) || !aligned16(summary) || !aligned16(workspace) || !aligned16(est_out)) return MAGE_ERR_ALIGN;
    const QuestLayout lay = quest_layout(*shape, s2);
    if (!workspace || workspace_bytes < lay.bytes) return MAGE_ERR_WORKSPACE;
    char *w = static_cast<char *>(workspace);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    void *q2 = w + lay.q2;
    int32_t *pages = reinterpret_cast<int32_t *>(w + lay.pages);
    const int rv = select_check(&s2, q2, summary, pages, est_out, nullptr, w + lay.select, lay.pages - lay.select);
    if (rv != MAGE_OK) return rv;                    // nothing has been launched yet
    if (launch_quest_query(q, q2, (long long)shape->B * shape->Hq, shape->d, stream) != hipSuccess) return MAGE_ERR_HIP;
    // the bound is scaled like a logit of the original head dimension
    const int rs = select_impl(&s2, (float)(1.4426950408889634 / sqrt((double)shape->d)), p, q2, summary, pages, est_out, nullptr,
                               w + lay.select, lay.pages - lay.select, hip_stream);
    if (rs != MAGE_OK) return rs;
    if (launch_expand_pages(pages, idx_out, shape->Hkv, shape->k, p, stream) != hipSuccess) return MAGE_ERR_HIP;
    return MAGE_OK;
}

int mage_set_overlap(const int32_t *a, const int32_t *b, int n_rows, int k, int a_rows, float *out, void *hip_stream)
{
    if (!a || !b || !out) return MAGE_ERR_NULL;
    if (n_rows <= 0 || k <= 0 || a_rows <= 0 || a_rows > n_rows || n_rows > (1 << 24)) return MAGE_ERR_SHAPE;
    const hipError_t e = launch_overlap(a, b, n_rows, k, a_rows, out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

}  // extern "C"
