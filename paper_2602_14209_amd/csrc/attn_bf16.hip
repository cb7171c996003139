// bf16 MFMA kernels of the MAGE hot path for gfx950 (CDNA4, 64-wide wavefronts).
//
//   attn_bf16_kernel<D,NW,MODE,GATHER>
//     MODE_ATTN : split-key flash-style attention of the G*B query rows of one KV head over a
//                 slice of keys (contiguous cache rows, or cache rows gathered through the
//                 selected index set, then optionally the in-block keys) -- Alg. 1 main stream
//                 "Attn(Q,K,V,C)" and Phase 2 "SparseAttn(Q_h,K_h,V_h,C[S])".
//     MODE_STATS: the same score pass without values: per-row running max and normaliser of
//                 softmax(Q1 K^T / sqrt(d)) over the prefix (Alg. 1 select stream, first half).
//   colsum_bf16_kernel<D,NW>
//                 second pass of selection: recomputes the scores, normalises each row with
//                 its final log-sum-exp and averages over the G*B rows (Eq. 5) -> alpha[h,j].
//
// Tiling: one workgroup = NW wavefronts; wavefront w owns 32 query rows (one 32x32 MFMA tile
// along M); all wavefronts share each 64-key K / V tile, staged once in LDS from coalesced
// 16-byte global loads and register-prefetched one tile ahead.
//
// Scores are produced transposed (S^T = K Q^T, v_mfma_f32_32x32x16_bf16 with the K tile as
// the A operand): a lane then holds 32 scores of ONE query row, so the online softmax is
// in-lane work, and the exponentiated scores are already laid out as the B operand of
// O^T = V^T P^T.  V is transposed on its way into LDS (pairs of keys per 32-bit write).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.hpp"

namespace mage {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned short u16;

enum { MODE_ATTN = 0, MODE_STATS = 1 };

constexpr int KPAD = 8;                      // bf16 elements of padding per K row in LDS
constexpr int VT_STRIDE = kBf16Tile + 8;     // bf16 elements per V^T row in LDS

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }

// position of key kappa inside a V^T row: bits 2 and 3 of the key index swapped, so that the 8
// keys one lane feeds to one P.V MFMA are contiguous (see the score register layout below)
__device__ __forceinline__ int vt_pos(int kappa) { return (kappa & ~0xC) | ((kappa >> 1) & 4) | ((kappa << 1) & 8); }

template <int D, int NT, bool WITH_V>
struct TileStager {
    static constexpr int CH = D / 8;                         // 16-byte chunks per row
    static constexpr int ITEMS = (kBf16Tile / 2) * CH;       // (key pair, chunk) work items per tile
    static constexpr int IPT = (ITEMS + NT - 1) / NT;        // items per thread
    uint4 kreg[IPT][2];
    uint4 vreg[WITH_V ? IPT : 1][2];

    // Issue the global loads of one tile.  `row_of(key)` returns the source row (already clamped
    // to a valid key) and `kbase`/`vbase` point at element (row 0, this KV head, 0).
    template <class RowOf>
    __device__ __forceinline__ void fetch(const u16 *kbase, const u16 *vbase, long long row_stride, RowOf row_of)
    {
#pragma unroll
        for (int i = 0; i < IPT; ++i) {
            const int id = threadIdx.x + i * NT;
            if (ITEMS % NT == 0 || id < ITEMS) {
                const int c = id % CH, p = id / CH;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const long long off = row_of(2 * p + e) * row_stride + c * 8;
                    kreg[i][e] = *reinterpret_cast<const uint4 *>(kbase + off);
                    if (WITH_V) vreg[i][e] = *reinterpret_cast<const uint4 *>(vbase + off);
                }
            }
        }
    }

    // registers -> LDS: K row-major [key][D+KPAD]; V transposed [physical d row][key position]
    // with physical row = (d % 8) * CH + d / 8 (16 consecutive lanes hit 16 consecutive rows on
    // both the write and the read side, which keeps the 144-byte row stride conflict-free).
    __device__ __forceinline__ void commit(u16 *ks, u16 *vt)
    {
#pragma unroll
        for (int i = 0; i < IPT; ++i) {
            const int id = threadIdx.x + i * NT;
            if (ITEMS % NT == 0 || id < ITEMS) {
                const int c = id % CH, p = id / CH;
                *reinterpret_cast<uint4 *>(ks + (2 * p) * (D + KPAD) + c * 8) = kreg[i][0];
                *reinterpret_cast<uint4 *>(ks + (2 * p + 1) * (D + KPAD) + c * 8) = kreg[i][1];
                if (WITH_V) {
                    const int pos = vt_pos(2 * p);
                    const uint32_t a[4] = {vreg[i][0].x, vreg[i][0].y, vreg[i][0].z, vreg[i][0].w};
                    const uint32_t b[4] = {vreg[i][1].x, vreg[i][1].y, vreg[i][1].z, vreg[i][1].w};
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const uint32_t even = (a[w] & 0xffffu) | (b[w] << 16);        // d = c*8 + 2w
                        const uint32_t odd = (a[w] >> 16) | (b[w] & 0xffff0000u);    // d = c*8 + 2w + 1
                        *reinterpret_cast<uint32_t *>(vt + ((2 * w) * CH + c) * VT_STRIDE + pos) = even;
                        *reinterpret_cast<uint32_t *>(vt + ((2 * w + 1) * CH + c) * VT_STRIDE + pos) = odd;
                    }
                }
            }
        }
    }
};

// Query fragment of this lane: row (l % 32) of the wavefront's M tile, 8 consecutive channels
// per MFMA k-step.  Row r of a KV head's row space is (g_local = r / B, q = r % B).
template <int D>
__device__ __forceinline__ void load_q_frag(const KernelArgs &a, int h, int row, bf16x8_t (&qf)[D / 16])
{
    const int lg = (threadIdx.x & 63) >> 5;
    if (row < a.R) {
        const int gl = row / a.B, qi = row - gl * a.B;
        const u16 *src = static_cast<const u16 *>(a.q) + ((long long)qi * a.Hq + (long long)h * a.G + gl) * D + 8 * lg;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qf[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(src + ks * 16));
    } else {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qf[ks] = as_bf16x8(make_uint4(0, 0, 0, 0));
    }
}

// Which keys does split `s` cover?  Cache keys [c0, c1) and, on the block split, n_blk block keys.
struct SplitRange {
    long long c0, c1;
    int cache_tiles, blk_tiles;
};

__device__ __forceinline__ SplitRange split_range(const KernelArgs &a, int s)
{
    SplitRange r;
    r.c0 = (long long)s * a.kps;
    r.c1 = r.c0 + a.kps;
    if (r.c1 > a.nc) r.c1 = a.nc;
    if (r.c0 > r.c1) r.c0 = r.c1;
    r.cache_tiles = (int)((r.c1 - r.c0 + kBf16Tile - 1) / kBf16Tile);
    r.blk_tiles = (s == a.blk_split) ? (a.n_blk + kBf16Tile - 1) / kBf16Tile : 0;
    return r;
}

template <int D, int NW, int MODE, bool GATHER>
__global__ __launch_bounds__(NW * 64) void attn_bf16_kernel(const KernelArgs a)
{
    constexpr int NT = NW * 64;
    constexpr bool WITH_V = (MODE == MODE_ATTN);
    constexpr int KS = D / 16;     // MFMA k-steps over the head dimension
    constexpr int DT = D / 32;     // 32-row tiles of O^T

    __shared__ __attribute__((aligned(16))) u16 ks_lds[kBf16Tile * (D + KPAD)];
    __shared__ __attribute__((aligned(16))) u16 vt_lds[WITH_V ? D * VT_STRIDE : 8];

    const int h = blockIdx.x, split = blockIdx.y, rg = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int row0 = (rg * NW + wave) * 32;           // first row of this wavefront's M tile
    const int row = row0 + l32;
    const bool wave_active = row0 < a.R;

    const SplitRange sr = split_range(a, split);
    const int ntiles = sr.cache_tiles + sr.blk_tiles;

    bf16x8_t qf[KS];
    load_q_frag<D>(a, h, row, qf);

    f32x16_t o[WITH_V ? DT : 1];
#pragma unroll
    for (int i = 0; i < (WITH_V ? DT : 1); ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    TileStager<D, NT, WITH_V> st;
    const long long cache_stride = (long long)a.Hkv * D;
    const u16 *kc = static_cast<const u16 *>(a.kc) + (long long)h * D;
    const u16 *vc = static_cast<const u16 *>(a.vc) + (long long)h * D;
    const u16 *kb = static_cast<const u16 *>(a.kblk) + (long long)h * D;
    const u16 *vb = static_cast<const u16 *>(a.vblk) + (long long)h * D;
    const int32_t *idx = GATHER ? a.idx + (long long)h * a.nc : nullptr;

    auto tile_valid = [&](int t) -> int {
        if (t < sr.cache_tiles) {
            const long long left = sr.c1 - (sr.c0 + (long long)t * kBf16Tile);
            return left < kBf16Tile ? (int)left : kBf16Tile;
        }
        const int left = a.n_blk - (t - sr.cache_tiles) * kBf16Tile;
        return left < kBf16Tile ? left : kBf16Tile;
    };
    auto fetch_tile = [&](int t) {
        const int valid = tile_valid(t);
        if (t < sr.cache_tiles) {
            const long long base = sr.c0 + (long long)t * kBf16Tile;
            st.fetch(kc, vc, cache_stride, [&](int key) -> long long {
                const long long pos = base + (key < valid ? key : valid - 1);
                return GATHER ? (long long)idx[pos] : pos;
            });
        } else {
            const int base = (t - sr.cache_tiles) * kBf16Tile;
            st.fetch(kb, vb, cache_stride, [&](int key) -> long long { return base + (key < valid ? key : valid - 1); });
        }
    };

    if (ntiles > 0) fetch_tile(0);
    for (int t = 0; t < ntiles; ++t) {
        st.commit(ks_lds, vt_lds);
        __syncthreads();
        if (t + 1 < ntiles) fetch_tile(t + 1);
        const int valid = tile_valid(t);

        if (wave_active) {
            // S^T tile: sc[kt][v] = score of query row l32 against key kt*32 + 8*(v/4) + 4*lg + v%4
            f32x16_t sc[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[kt][v] = 0.f;
                const u16 *krow = ks_lds + (kt * 32 + l32) * (D + KPAD) + 8 * lg;
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const bf16x8_t kf = as_bf16x8(*reinterpret_cast<const uint4 *>(krow + s * 16));
                    sc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sc[kt], 0, 0, 0);
                }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = kt * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
                    float s2 = sc[kt][v] * a.scale_log2;
                    if (valid < kBf16Tile && key >= valid) s2 = -INFINITY;
                    sc[kt][v] = s2;
                    mx = fmaxf(mx, s2);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            float psum = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(sc[kt][v] - m_new);
                    sc[kt][v] = p;
                    psum += p;
                }
            l_run = l_run * corr + psum;

            if (WITH_V) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[dt][v] *= corr;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int m2 = 0; m2 < 2; ++m2) {
                        bf16x8_t pf;
#pragma unroll
                        for (int e = 0; e < 8; ++e) pf[e] = (__bf16)sc[kt][8 * m2 + e];
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) {
                            const u16 *vrow = vt_lds + (dt * 32 + l32) * VT_STRIDE + kt * 32 + m2 * 16 + lg * 8;
                            const bf16x8_t vf = as_bf16x8(*reinterpret_cast<const uint4 *>(vrow));
                            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[dt], 0, 0, 0);
                        }
                    }
            }
        }
        __syncthreads();
    }

    if (!wave_active) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32);

    if (MODE == MODE_STATS) {
        if (row < a.R && lg == 0) {
            const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
            a.part_m[pi] = m_run;
            a.part_l[pi] = l_tot;
        }
        return;
    }

    if (row >= a.R) return;
    // O^T register (dt, v) holds channel d = 8*c + e of query row `row`, where the physical
    // V^T row is pr = dt*32 + 8*(v/4) + 4*lg + v%4, c = pr % CH, e = pr / CH.
    constexpr int CH = D / 8;
    if (a.n_split == 1) {
        const int gl = row / a.B, qi = row - gl * a.B;
        float *dst = a.out + ((long long)qi * a.Hq + (long long)h * a.G + gl) * D;
        const float inv = 1.f / l_tot;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int pr = dt * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
                dst[8 * (pr % CH) + pr / CH] = o[dt][v] * inv;
            }
        if (a.lse_out && lg == 0)
            a.lse_out[(long long)qi * a.Hq + (long long)h * a.G + gl] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    } else {
        const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
        float *dst = a.part_o + pi * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int pr = dt * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
                dst[8 * (pr % CH) + pr / CH] = o[dt][v];
            }
        if (lg == 0) {
            a.part_m[pi] = m_run;
            a.part_l[pi] = l_tot;
        }
    }
}

// Second pass of selection.  Scores are produced untransposed (S = Q K^T: the query fragment
// is the A operand), so a lane holds 16 query rows of ONE key and the sum over rows is in-lane.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void colsum_bf16_kernel(const KernelArgs a)
{
    constexpr int NT = NW * 64;
    constexpr int KS = D / 16;
    __shared__ __attribute__((aligned(16))) u16 ks_lds[kBf16Tile * (D + KPAD)];
    __shared__ float red[NW][kBf16Tile];

    const int h = blockIdx.x, split = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int row0 = wave * 32;
    const bool wave_active = row0 < a.R;

    const SplitRange sr = split_range(a, split);
    const int ntiles = sr.cache_tiles;

    bf16x8_t qf[KS];
    load_q_frag<D>(a, h, row0 + l32, qf);

    // per-register row statistics: register v is query row row0 + 8*(v/4) + 4*lg + v%4
    float lse2[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int r = row0 + 8 * (v >> 2) + 4 * lg + (v & 3);
        lse2[v] = r < a.R ? a.lse2[(long long)h * a.rpad + r] : INFINITY;   // exp2(-inf) = 0 for padding rows
    }

    TileStager<D, NT, false> st;
    const long long cache_stride = (long long)a.Hkv * D;
    const u16 *kc = static_cast<const u16 *>(a.kc) + (long long)h * D;

    auto tile_valid = [&](int t) -> int {
        const long long left = sr.c1 - (sr.c0 + (long long)t * kBf16Tile);
        return left < kBf16Tile ? (int)left : kBf16Tile;
    };
    auto fetch_tile = [&](int t) {
        const int valid = tile_valid(t);
        const long long base = sr.c0 + (long long)t * kBf16Tile;
        st.fetch(kc, kc, cache_stride, [&](int key) -> long long { return base + (key < valid ? key : valid - 1); });
    };

    if (ntiles > 0) fetch_tile(0);
    for (int t = 0; t < ntiles; ++t) {
        st.commit(ks_lds, nullptr);
        __syncthreads();
        if (t + 1 < ntiles) fetch_tile(t + 1);
        const int valid = tile_valid(t);

#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            float col = 0.f;
            if (wave_active) {
                f32x16_t sc;
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[v] = 0.f;
                const u16 *krow = ks_lds + (kt * 32 + l32) * (D + KPAD) + 8 * lg;
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const bf16x8_t kf = as_bf16x8(*reinterpret_cast<const uint4 *>(krow + s * 16));
                    sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[s], kf, sc, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) col += __builtin_amdgcn_exp2f(fmaf(sc[v], a.scale_log2, -lse2[v]));
                col += __shfl_xor(col, 32);
            }
            if (lg == 0) red[wave][kt * 32 + l32] = col;
        }
        __syncthreads();
        if (threadIdx.x < kBf16Tile && (int)threadIdx.x < valid) {
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) acc += red[w][threadIdx.x];
            a.alpha[(long long)h * a.L + sr.c0 + (long long)t * kBf16Tile + threadIdx.x] = acc * a.inv_rows;
        }
    }
}

// ------------------------------------------------------------------------------ launchers
template <int D, int NW, int MODE, bool GATHER>
static hipError_t launch_attn(const KernelArgs &a, int row_groups, hipStream_t stream)
{
    dim3 grid(a.Hkv, a.n_split, row_groups), block(NW * 64);
    hipLaunchKernelGGL((attn_bf16_kernel<D, NW, MODE, GATHER>), grid, block, 0, stream, a);
    return hipGetLastError();
}

template <int D, int NW>
static hipError_t launch_colsum(const KernelArgs &a, hipStream_t stream)
{
    dim3 grid(a.Hkv, a.n_split), block(NW * 64);
    hipLaunchKernelGGL((colsum_bf16_kernel<D, NW>), grid, block, 0, stream, a);
    return hipGetLastError();
}

hipError_t bf16_attn(const KernelArgs &a, int d, int waves, int row_groups, bool gather, hipStream_t stream)
{
    if (d == 128 && waves == 4) return gather ? launch_attn<128, 4, MODE_ATTN, true>(a, row_groups, stream) : launch_attn<128, 4, MODE_ATTN, false>(a, row_groups, stream);
    if (d == 128 && waves == 8) return gather ? launch_attn<128, 8, MODE_ATTN, true>(a, row_groups, stream) : launch_attn<128, 8, MODE_ATTN, false>(a, row_groups, stream);
    if (d == 64 && waves == 4) return gather ? launch_attn<64, 4, MODE_ATTN, true>(a, row_groups, stream) : launch_attn<64, 4, MODE_ATTN, false>(a, row_groups, stream);
    if (d == 64 && waves == 8) return gather ? launch_attn<64, 8, MODE_ATTN, true>(a, row_groups, stream) : launch_attn<64, 8, MODE_ATTN, false>(a, row_groups, stream);
    return hipErrorInvalidValue;
}

hipError_t bf16_stats(const KernelArgs &a, int d, int waves, int row_groups, hipStream_t stream)
{
    if (d == 128 && waves == 4) return launch_attn<128, 4, MODE_STATS, false>(a, row_groups, stream);
    if (d == 128 && waves == 8) return launch_attn<128, 8, MODE_STATS, false>(a, row_groups, stream);
    if (d == 64 && waves == 4) return launch_attn<64, 4, MODE_STATS, false>(a, row_groups, stream);
    if (d == 64 && waves == 8) return launch_attn<64, 8, MODE_STATS, false>(a, row_groups, stream);
    return hipErrorInvalidValue;
}

hipError_t bf16_colsum(const KernelArgs &a, int d, int waves, hipStream_t stream)
{
    if (d == 128 && waves == 4) return launch_colsum<128, 4>(a, stream);
    if (d == 128 && waves == 8) return launch_colsum<128, 8>(a, stream);
    if (d == 64 && waves == 4) return launch_colsum<64, 4>(a, stream);
    if (d == 64 && waves == 8) return launch_colsum<64, 8>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace mage
