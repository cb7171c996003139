/*
 * mage.h -- C ABI of the MI355X (gfx950) implementation of the MAGE hot path
 * ([MASK]-Guided Sparse Attention for block-diffusion LLM decoding, arxiv 2602.14209).
 *
 * Notation (the paper's): B block size, Hq query heads, Hkv KV heads, G = Hq/Hkv query
 * heads per KV group, d head dimension, L cached prefix length (the paper's N), k budget,
 * T denoising steps per block.  Query head g belongs to KV head g / G (contiguous groups).
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is a DEVICE pointer (HBM), row-major and contiguous, 16-byte
 *     aligned.  `shape` is a HOST pointer.  `hip_stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).
 *   - The caller owns every buffer, including the workspace; the library never allocates,
 *     never frees and never synchronises: it validates its arguments on the host, enqueues
 *     kernels on `hip_stream` and returns.  Results are complete when the stream reaches the
 *     point after the call.  Two calls that share a workspace must be ordered (same stream,
 *     or an event between them).
 *   - Return value: MAGE_OK or a negative mage_status.  Argument errors are detected before
 *     anything is launched; in that case no buffer is touched.
 *   - Element type of q / k_cache / v_cache / k_blk / v_blk is shape->dtype: MAGE_F32
 *     (float) or MAGE_BF16 (bfloat16 bit patterns, uint16).  Arithmetic accumulates in fp32;
 *     `out`, `lse_out`, `alpha_out` are fp32; indices are int32.
 *   - T is not an argument: the caller invokes mage_sparse_attn once per denoising step
 *     2..T with the index set that mage_select produced at step 1 (Alg. 1, Phase 2).
 *   - Supported: d in {64, 128}; Hq % Hkv == 0; 1 <= k <= L <= 2^30; B*G <= 2^20, B*B*G < 2^32 and
 *     Hkv*d < 2^29 (the kernels' 32-bit row arithmetic); B*G <= 256 for mage_select and mage_step1
 *     with MAGE_BF16; mage_sparse_attn_batched with MAGE_BF16 only.
 */
#ifndef MAGE_H
#define MAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MAGE_F32 = 0, MAGE_BF16 = 1 } mage_dtype;

typedef enum {
    MAGE_OK = 0,
    MAGE_ERR_NULL = -1,        /* a required pointer is NULL */
    MAGE_ERR_SHAPE = -2,       /* B, Hq, Hkv, d, L or k <= 0; Hq % Hkv != 0; k > L */
    MAGE_ERR_UNSUPPORTED = -3, /* d not in {64,128}; unknown dtype; L > 2^30; B, G or Hkv beyond the stated ranges */
    MAGE_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than mage_workspace_bytes() */
    MAGE_ERR_HIP = -5,         /* a kernel launch reported an error */
    MAGE_ERR_ALIGN = -6,       /* a data pointer is not 16-byte aligned */
    MAGE_ERR_SCRATCH = -7      /* mage_select_static: the problem needs more than mage_static_scratch_bytes() */
} mage_status;

/* Problem geometry of one layer and one block (Alg. 1 "Require: cache C, B, k, T"). */
typedef struct {
    int B;       /* block size: queries per block */
    int Hq;      /* query heads */
    int Hkv;     /* KV heads */
    int d;       /* head dimension */
    int64_t L;   /* cached prefix length */
    int k;       /* selection budget per KV head (ignored by mage_exact_attn, which only needs k >= 1) */
    int dtype;   /* mage_dtype of q / K / V */
} mage_shape;

/* Library version (major*10000 + minor*100 + patch).  Host only. */
int mage_version(void);

/* Static, never-freed description of a status code.  Host only. */
const char *mage_status_string(int status);

/* Bytes of device workspace that any of the calls below needs for `shape`
 * (the maximum over the calls that support the shape: a bf16 shape with B*G > 256 still gets the
 * size its attention calls need, although mage_select and mage_step1 reject it).  Host only, pure.
 * Returns 0 if `shape` is invalid. */
size_t mage_workspace_bytes(const mage_shape *shape);

/*
 * Step-1 selection (Alg. 1, select stream; Sec. 4 Phase 1, Eq. 5; Eq. 2 per-block form).
 *   A[g,q,j]   = softmax over the L prefix positions j of  q1[q,g,:].k_cache[j,g/G,:] / sqrt(d)
 *   alpha[h,j] = 1/(G*B) * sum_{g in group(h)} sum_q A[g,q,j]
 *   S[h]       = the k positions j with the largest alpha[h,j]; equal values: smaller j first
 * In:  q1 [B,Hq,d] (the All-[MASK] block's queries), k_cache [L,Hkv,d].
 * Out: idx_out [Hkv,k] int32, each row ascending in j;
 *      alpha_out [Hkv,L] fp32, nullable (the averaged probabilities that were ranked).
 * The ranking is taken on fp32 values of alpha: the ones the kernels computed, except that candidates
 * within 4e-6 (relative) of the k-th largest are first recomputed from the inputs in fp64 (exact dot
 * products, fp64 normalisers and exponentials) and rounded once to fp32, so that rounding error of the
 * fp32 pass cannot decide which of two nearly equal keys is kept.  alpha_out keeps the fp32 pass's values.
 */
int mage_select(const mage_shape *shape, const void *q1, const void *k_cache,
                int32_t *idx_out, float *alpha_out,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * mage_select for callers that can neither allocate nor pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs, kernels and
 * results as mage_select; the scratch data of the kernels lives in a static device array of
 * mage_static_scratch_bytes() bytes (8 MiB; every GPU the library runs on holds one until the process
 * ends), which covers e.g. Hkv = 8, L = 131072.  A shape that needs more returns MAGE_ERR_SCRATCH
 * and launches nothing.  The call allocates nothing and frees nothing.  The current device must be
 * the one `hip_stream` belongs to.  All calls on one GPU share that GPU's array: two calls that
 * overlap in time (different streams, no event between them) race.
 */
size_t mage_static_scratch_bytes(void);
int mage_select_static(const mage_shape *shape, const void *q1, const void *k_cache,
                       int32_t *idx_out, float *alpha_out, void *hip_stream);

/*
 * Block-averaged probabilities per QUERY head (Sec. 3, Eq. 2 written per head; the inner
 * average of Eq. 5):
 *   pbar[g,j] = 1/B * sum_q A[g,q,j],   A as in mage_select
 * so every row of pbar sums to 1 over j, and the mean of the G rows of a KV head's group is
 * mage_select's alpha.  A diagnostic output (which positions each head of the block looks at);
 * the index set is taken per KV head by mage_select.
 * In:  q1 [B,Hq,d], k_cache [L,Hkv,d]; shape as for mage_select (k is validated, not used).
 * Out: pbar_out [Hq,L] fp32.
 * Cost: the pass over K that mage_select makes, plus G further passes (one per head of a group).
 * Same limits as mage_select (B*G <= 256 with MAGE_BF16); workspace as mage_workspace_bytes().
 */
int mage_block_probs(const mage_shape *shape, const void *q1, const void *k_cache, float *pbar_out,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Exact attention of the block over the whole cache plus the block itself (Alg. 1 main
 * stream "Attn(Q,K,V,C)"; also the Exact baseline of Sec. 5):
 *   out[q,g,:] = softmax_j( [q.K_cache^T ; q.K_blk^T] / sqrt(d) ) . [V_cache ; V_blk]
 * one softmax over L + B keys of KV head g/G, in-block part bidirectional (no mask).
 * In:  q [B,Hq,d]; k_cache, v_cache [L,Hkv,d]; k_blk, v_blk [B,Hkv,d] (both NULL = no
 *      in-block keys).
 * Out: out [B,Hq,d] fp32; lse_out [B,Hq] fp32, nullable (natural-log sum-exp of the logits).
 */
int mage_exact_attn(const mage_shape *shape, const void *q, const void *k_cache, const void *v_cache,
                    const void *k_blk, const void *v_blk,
                    float *out, float *lse_out,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Sparse attention of one denoising step (Alg. 1 Phase 2 "SparseAttn(Q_h,K_h,V_h,C[S])";
 * Sec. 4 Phase 2): as mage_exact_attn, with the cache restricted, per KV head h, to the k
 * positions idx[h,:]; one softmax over k + B keys.
 * In:  idx [Hkv,k] int32, every entry in [0,L) (a precondition: not checked on the device;
 *      an out-of-range entry reads out of bounds).  Order within a row is free; duplicates
 *      are attended as many times as they appear.
 * Out: out [B,Hq,d] fp32; lse_out [B,Hq] fp32, nullable.
 */
int mage_sparse_attn(const mage_shape *shape, const void *q, const void *k_cache, const void *v_cache,
                     const int32_t *idx, const void *k_blk, const void *v_blk,
                     float *out, float *lse_out,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Step 1 in one call (Alg. 1 Phase 1, both streams' work on one stream): mage_exact_attn of the
 * All-[MASK] block AND mage_select of the same queries.  The attention pass already walks every
 * prefix key, so it also leaves the per-row prefix softmax statistics (max, sum-exp over the L
 * cache keys only) that selection needs; selection then reads K once instead of twice.  Results
 * are those of the two separate calls (same definitions; the row statistics come from a different
 * split of the keys, so alpha can differ in the last bits).
 * In/out: as mage_exact_attn (q1 is the block's step-1 queries) and mage_select.
 */
int mage_step1(const mage_shape *shape, const void *q1, const void *k_cache, const void *v_cache,
               const void *k_blk, const void *v_blk,
               float *out, float *lse_out, int32_t *idx_out, float *alpha_out,
               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Compacted selection.  The index set is fixed for steps 2..T (Sec. 4 Phase 2), so the selected
 * rows can be copied once per block into a cache of length k,
 *   k_sel[p,h,:] = k_cache[idx[h,p],h,:],  v_sel likewise,   p in [0,k),
 * and every later step attends it without an index indirection.
 * In:  k_cache, v_cache [L,Hkv,d]; idx [Hkv,k] (entries in [0,L)).
 * Out: k_sel, v_sel [k,Hkv,d], same element type.  No workspace.
 */
int mage_compact(const mage_shape *shape, const void *k_cache, const void *v_cache, const int32_t *idx,
                 void *k_sel, void *v_sel, void *hip_stream);

/*
 * mage_sparse_attn on rows compacted by mage_compact: softmax over the k rows of k_sel / v_sel
 * [k,Hkv,d] plus the B in-block keys.  Same result as mage_sparse_attn with the index set the
 * rows were compacted with (up to the order of fp32 additions).  shape->L is not used.
 */
int mage_sparse_attn_compact(const mage_shape *shape, const void *q, const void *k_sel, const void *v_sel,
                             const void *k_blk, const void *v_blk, float *out, float *lse_out,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * mage_sparse_attn for n_seq independent sequences in one launch (decoding a batch of blocks):
 * every array gains a leading sequence axis -- q, out [n_seq,B,Hq,d]; k_cache, v_cache
 * [n_seq,L,Hkv,d]; idx [n_seq,Hkv,k]; k_blk, v_blk [n_seq,B,Hkv,d]; lse_out [n_seq,B,Hq].
 * The launch then carries enough independent work to be bound by HBM bandwidth rather than by
 * the latency of one small gather.  1 <= n_seq <= 65535 (MAGE_ERR_SHAPE otherwise); MAGE_BF16 only and
 * (n_seq*Hkv + 8)*Hkv < 2^32 (MAGE_ERR_UNSUPPORTED otherwise).
 */
int mage_sparse_attn_batched(const mage_shape *shape, int n_seq, const void *q, const void *k_cache,
                             const void *v_cache, const int32_t *idx, const void *k_blk, const void *v_blk,
                             float *out, float *lse_out, void *hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Second workload: the lightweight estimator the paper compares against, under the same per-block
 * selection (Sec. 2 "Methods for AR LLMs": Quest; Sec. 3.1, Eq. 2 per-block form), and the overlap
 * ratio both of its accuracy measures are (Eq. 1, Eq. 3).
 * ------------------------------------------------------------------------------------------- */

/*
 * Page summaries (Sec. 2, Quest): the cache of every KV head is cut into pages of p consecutive
 * positions (the last one may be shorter) and each page is summarised by its per-channel maximum
 * and minimum key:  summary[P,h,0,:] = max_j k_cache[j,h,:],  summary[P,h,1,:] = min_j,  j in page P.
 * In:  k_cache [L,Hkv,d].  Out: summary [ceil(L/p),Hkv,2,d], same element type.  shape->k and
 * shape->B are not used.  p >= 1.  No workspace.
 */
int mage_page_summary(const mage_shape *shape, int p, const void *k_cache, void *summary, void *hip_stream);

/* Bytes of workspace mage_quest_select needs for `shape` and page size p (0 if invalid). */
size_t mage_quest_workspace_bytes(const mage_shape *shape, int p);

/*
 * Estimated per-block KV subset (Eq. 2, per-block form, with the estimator's scores in place of the
 * exact ones).  The page score of a query is the sign-aware upper bound on q.k over the page,
 *   bound[g,q,P] = sum_c max(q[q,g,c] * Kmax[P,g/G,c], q[q,g,c] * Kmin[P,g/G,c]);
 * the estimated score of position j is softmax over the L positions of bound[g,q,page(j)] / sqrt(d)
 * (the exact score with every logit replaced by its page's bound; the paper does not spell this
 * step out), averaged over the G heads of the group and the B tokens; the subset is its Top-k,
 * equal scores to the smaller position -- i.e. the k/p best pages, whole.
 * In:  q [B,Hq,d]; summary from mage_page_summary with the same p.
 * Out: idx_out [Hkv,k] int32 ascending; est_out [Hkv,L/p] fp32, nullable (the averaged estimated
 *      score of one position of each page).
 * Needs MAGE_BF16, L % p == 0, k % p == 0 and B*G <= 256 (MAGE_ERR_UNSUPPORTED otherwise).
 */
int mage_quest_select(const mage_shape *shape, int p, const void *q, const void *summary,
                      int32_t *idx_out, float *est_out,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Overlap of index sets: out[i] = |A_(i mod a_rows) intersect B_i| / k for i in [0, n_rows).
 * Eq. 1 (estimation accuracy of a subset against per-token oracle subsets: a = the evaluated
 * subset [Hkv,k], a_rows = Hkv, b = oracle subsets [B,Hkv,k], n_rows = B*Hkv) and Eq. 3 (recall of
 * the step-1 oracle subset at a later noise level: a_rows = n_rows = Hkv).
 * In:  a [a_rows,k] int32, every row ascending and duplicate-free (as mage_select emits them);
 *      b [n_rows,k] int32, rows duplicate-free, any order.  Out: out [n_rows] fp32.
 */
int mage_set_overlap(const int32_t *a, const int32_t *b, int n_rows, int k, int a_rows, float *out, void *hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Measurement aids (not part of the method): the floors and ceilings the benchmark prints beside the
 * attention figures, so that a latency-bound launch can be told from a bandwidth-bound one.
 * ------------------------------------------------------------------------------------------- */

/* One kernel that does nothing: the cost of a launch slot in a stream or a HIP graph. */
int mage_diag_empty(void *hip_stream);

/* One kernel that stores the device's constant-rate wall clock to *out (8-byte aligned device memory).
 * Two of them around a run of launches on one stream -- also inside a captured HIP graph, where no
 * host-side event can go -- give the time that run took: (later - earlier) / mage_diag_stamp_hz().
 * mage_diag_stamp_hz: ticks per second of that clock on the current device, 0 if it cannot be queried. */
int mage_diag_stamp(uint64_t *out, void *hip_stream);
int64_t mage_diag_stamp_hz(void);

/* One lane follows n_hops dependent loads: i = chain[i], from i = start; the last i goes to *out.
 * chain [n_entries] int32, every entry in [0, n_entries) (a precondition).  Time / n_hops is the
 * latency of one dependent memory round trip (the sparse step has two: index entry, then row). */
int mage_diag_chase(const int32_t *chain, int64_t n_entries, int start, int n_hops, int32_t *out, void *hip_stream);

/* Streaming read of `bytes` bytes (16-byte loads on every CU); sink [4096] uint32 is scratch that is
 * practically never written.  bytes / time is the read bandwidth this GPU reaches. */
int mage_diag_read(const void *src, size_t bytes, uint32_t *sink, void *hip_stream);

/* Streaming copy dst[0:bytes) = src[0:bytes) (whole 16-byte units; a tail shorter than 16 bytes is not
 * copied).  2 * bytes / time is the copy bandwidth; it also is the kernel of known traffic that the
 * profiler's byte counters are scaled with. */
int mage_diag_copy(void *dst, const void *src, size_t bytes, void *hip_stream);

/* What merging partial results ACROSS workgroups inside one launch costs.  4 * n_groups workgroups each write
 * an 8 KB partial (src [4*n_groups*2048] fp32 + 1 in the first of every four floats) to part [4*n_groups*2048];
 * the last workgroup of each group of four to arrive adds the four partials into out [n_groups*2048].
 * mode 0: partials only, nobody merges; mode 1: device-scope fences around a counter; mode 2: no fence
 * instruction (device-scope stores and loads, the writer waits for its stores before the counter).
 * counters [n_groups] uint32 must be zero before the first launch and keep counting afterwards. */
int mage_diag_merge(int mode, int n_groups, float *part, unsigned *counters, float *out, const float *src, void *hip_stream);

/* The memory accesses of mage_sparse_attn_batched and nothing else: reads idx [n_seq,Hkv,k] and, for
 * every entry, that row of k_cache and of v_cache [n_seq,L,Hkv,d].  The rate at which the gather
 * itself can run on this GPU (a ceiling for the sparse step).  d * element size <= 256 bytes.
 * sink [1] uint32 is practically never written. */
int mage_diag_gather(const mage_shape *shape, int n_seq, const void *k_cache, const void *v_cache, const int32_t *idx,
                     uint32_t *sink, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MAGE_H */
