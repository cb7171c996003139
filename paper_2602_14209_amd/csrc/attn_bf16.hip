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
// along M); all wavefronts share each 64-key K / V tile.
//
// Data movement: tiles go HBM -> LDS directly (global_load_lds, 16 bytes per lane, no VGPR
// staging), double-buffered, one workgroup barrier per tile.  Rows stay row-major in LDS with an
// XOR swizzle of their 16-byte chunks, so that
//   - the K fragment of a lane (one key row, 8 channels) is one conflict-free ds_read_b128;
//   - the V fragment (8 keys at one channel) is two transposing reads (ds_read_b64_tr_b16), which
//     deliver V^T straight from the row-major tile.
//
// Scores are produced transposed (S^T = K Q^T, v_mfma_f32_32x32x16_bf16 with the K tile as the A
// operand): a lane then holds 32 scores of ONE query row, so the online softmax is in-lane work,
// and the exponentiated scores are already laid out as the B operand of O^T = V^T P^T.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.hpp"
#include "probe.hpp"

namespace mage {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short u16;

enum { MODE_ATTN = 0, MODE_STATS = 1 };

#define MAGE_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define MAGE_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }

// XOR swizzle of the 16-byte chunk index of tile row r.  16 consecutive rows (one ds_read_b128
// phase of the K fragment) and 4 consecutive rows (one half of a transposing V read) both land on
// distinct LDS banks.
template <int D>
__device__ __forceinline__ int swz(int r)
{
    return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
}

template <int D>
struct TileGeom {
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int CH = D / 8;                               // 16-byte chunks per row
    static constexpr int MAT_BYTES = kBf16Tile * ROW_BYTES;        // one 64-key K (or V) tile
    static constexpr int RPI = 1024 / ROW_BYTES;                   // rows covered by one wavefront-wide load
    static constexpr int LOADS = kBf16Tile / RPI;                  // wavefront-wide loads per matrix per tile
};

// Issue this wavefront's share of the direct HBM->LDS loads of one tile.  `row_of(r)` gives the
// source row of tile row r (already clamped to a valid key); `kbase`/`vbase` point at element
// (row 0, this KV head, channel 0); `buf` is the LDS tile buffer (K matrix, then V matrix).
template <int D, int NW, bool WITH_V, class RowOf>
__device__ __forceinline__ void issue_tile(const u16 *kbase, const u16 *vbase, long long row_stride,
                                           unsigned char *buf, RowOf row_of)
{
    using G = TileGeom<D>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int n = 0; n < G::LOADS / NW; ++n) {
        const int unit = n * NW + wave;                            // which 1 KB of the matrix
        const int r = unit * G::RPI + lane / G::CH;
        const int chunk = (lane % G::CH) ^ swz<D>(r);
        const long long off = row_of(r) * row_stride + chunk * 8;
        __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(kbase + off), MAGE_LDS_PTR(buf + unit * 1024), 16, 0, 0);
        if (WITH_V)
            __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(vbase + off), MAGE_LDS_PTR(buf + G::MAT_BYTES + unit * 1024), 16, 0, 0);
    }
}

// The same for a full tile of contiguous cache rows: `kptr[n]` is this lane's source address for
// load n at the first tile of the split (computed once); tile t lies t * 64 rows further on.
template <int D, int NW, bool WITH_V>
__device__ __forceinline__ void issue_tile_stream(const u16 *const (&kptr)[TileGeom<D>::LOADS / NW], long long tile_elems,
                                                  long long v_minus_k, int t, unsigned char *buf)
{
    using G = TileGeom<D>;
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int n = 0; n < G::LOADS / NW; ++n) {
        const int unit = n * NW + wave;
        const u16 *src = kptr[n] + t * tile_elems;
        __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(src), MAGE_LDS_PTR(buf + unit * 1024), 16, 0, 0);
        if (WITH_V)
            __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(src + v_minus_k), MAGE_LDS_PTR(buf + G::MAT_BYTES + unit * 1024), 16, 0, 0);
    }
}

template <int D, int NW>
__device__ __forceinline__ void stream_pointers(const u16 *kc, long long c0, long long row_stride,
                                                const u16 *(&kptr)[TileGeom<D>::LOADS / NW])
{
    using G = TileGeom<D>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int n = 0; n < G::LOADS / NW; ++n) {
        const int r = (n * NW + wave) * G::RPI + lane / G::CH;
        kptr[n] = kc + (c0 + r) * row_stride + ((lane % G::CH) ^ swz<D>(r)) * 8;
    }
}

// Wait until at most PENDING of this wavefront's HBM->LDS loads are outstanding (loads complete in
// issue order, so the oldest tile has landed), then meet the rest of the workgroup.
template <int PENDING>
__device__ __forceinline__ void tile_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory");
    __syncthreads();
}

// K fragment: key row `rk` of the tile, channels [16*ks + 8*lg, +8)
template <int D>
__device__ __forceinline__ bf16x8_t read_k_frag(const unsigned char *kbuf, int rk, int ks, int lg)
{
    const int chunk = (2 * ks + lg) ^ swz<D>(rk);
    return as_bf16x8(*reinterpret_cast<const uint4 *>(kbuf + rk * TileGeom<D>::ROW_BYTES + chunk * 16));
}

// V^T fragment for O^T tile dt: lane holds channel dt*32 + (lane & 31) of the 8 keys
// key0 + {0,1,2,3, 8,9,10,11}.  Within each 16-lane block, lane i' addresses 4 channels
// (4*(i' & 3) ..) of key (i' >> 2); the transposing read hands lane i the 4 keys at channel i.
template <int D>
__device__ __forceinline__ bf16x8_t read_vt_frag(const unsigned char *vbuf, int key0, int dt, int lane)
{
    const int blk = lane >> 4, ip = lane & 15;
    const int j = ip >> 2, q = ip & 3;
    const int d = dt * 32 + 16 * (blk & 1) + 4 * q;
    const int key_a = key0 + j, key_b = key0 + 8 + j;
    const unsigned char *pa = vbuf + key_a * TileGeom<D>::ROW_BYTES + (((d >> 3) ^ swz<D>(key_a)) * 16) + 8 * (q & 1);
    const unsigned char *pb = vbuf + key_b * TileGeom<D>::ROW_BYTES + (((d >> 3) ^ swz<D>(key_b)) * 16) + 8 * (q & 1);
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t *)(pa));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t *)(pb));
    const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, both);
}

// Query fragment of this lane: row (l % 32) of the wavefront's M tile, 8 consecutive channels
// per MFMA k-step.  Row r of a KV head's row space is (g_local = r / B, q = r % B).
template <int D>
__device__ __forceinline__ void load_q_frag(const KernelArgs &a, const u16 *q, int h, int row, bf16x8_t (&qf)[D / 16])
{
    const int lg = (threadIdx.x & 63) >> 5;
    if (row < a.R) {
        const int gl = row / a.B, qi = row - gl * a.B;
        const u16 *src = q + ((long long)qi * a.Hq + (long long)h * a.G + gl) * D + 8 * lg;
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
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2))) void attn_bf16_kernel(const KernelArgs a)
{
    using G = TileGeom<D>;
    constexpr bool WITH_V = (MODE == MODE_ATTN);
    constexpr int NBUF = WITH_V ? 2 : 3;                            // LDS tile buffers = prefetch distance + 1
    constexpr int LPT = (G::LOADS / NW) * (WITH_V ? 2 : 1);         // loads one wavefront issues per tile
    constexpr int KS = D / 16;     // MFMA k-steps over the head dimension
    constexpr int DT = D / 32;     // 32-row tiles of O^T
    constexpr int BUF_BYTES = G::MAT_BYTES * (WITH_V ? 2 : 1);
    constexpr int OST = D + 4;     // floats per staged output row
    constexpr int STAGE_BYTES = WITH_V ? 2 * 32 * OST * 4 : 0;
    static_assert(NBUF * BUF_BYTES >= STAGE_BYTES, "output staging must fit in the tile buffers");

    // tile buffers; after the key loop the same memory stages the output transposition
    __shared__ __attribute__((aligned(1024))) unsigned char smem[NBUF * BUF_BYTES];

    // key splits vary fastest over the grid: consecutive workgroups (dealt round-robin to the XCDs)
    // stream different key ranges of the same head, so every XCD touches every HBM channel
    // A batched launch (independent sequences, unsplit keys) uses the x axis for the sequence.
    const bool batched = a.seq_kv != 0;
    const long long z = batched ? blockIdx.x : 0;
    const int split = batched ? 0 : blockIdx.x, h = blockIdx.y, rg = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int row0 = (rg * NW + wave) * 32;           // first row of this wavefront's M tile
    const int row = row0 + l32;
    const bool wave_active = row0 < a.R;

    MAGE_PROBE_DECL;
    MAGE_PROBE_AT(0);
    const SplitRange sr = split_range(a, split);
    const int ntiles = sr.cache_tiles + sr.blk_tiles;

    const long long cache_stride = (long long)a.Hkv * D;
    const u16 *kc = static_cast<const u16 *>(a.kc) + z * a.seq_kv + (long long)h * D;
    const u16 *vc = static_cast<const u16 *>(a.vc) + z * a.seq_kv + (long long)h * D;
    const u16 *kb = static_cast<const u16 *>(a.kblk) + z * a.seq_blk + (long long)h * D;
    const u16 *vb = static_cast<const u16 *>(a.vblk) + z * a.seq_blk + (long long)h * D;
    const int32_t *idx = GATHER ? a.idx + z * a.seq_idx + (long long)h * a.nc : nullptr;

    auto tile_valid = [&](int t) -> int {
        if (t < sr.cache_tiles) {
            const long long left = sr.c1 - (sr.c0 + (long long)t * kBf16Tile);
            return left < kBf16Tile ? (int)left : kBf16Tile;
        }
        const int left = a.n_blk - (t - sr.cache_tiles) * kBf16Tile;
        return left < kBf16Tile ? left : kBf16Tile;
    };
    const u16 *kptr[G::LOADS / NW];
    if (!GATHER) stream_pointers<D, NW>(kc, sr.c0, cache_stride, kptr);
    const long long tile_elems = (long long)kBf16Tile * cache_stride;
    const long long v_minus_k = vc - kc;
    auto issue = [&](int t) {
        const int valid = tile_valid(t);
        unsigned char *buf = smem + (t % NBUF) * BUF_BYTES;
        if (!GATHER && t < sr.cache_tiles && valid == kBf16Tile) {
            issue_tile_stream<D, NW, WITH_V>(kptr, tile_elems, v_minus_k, t, buf);
        } else if (t < sr.cache_tiles) {
            const long long base = sr.c0 + (long long)t * kBf16Tile;
            issue_tile<D, NW, WITH_V>(kc, vc, cache_stride, buf, [&](int r) -> long long {
                const long long pos = base + (r < valid ? r : valid - 1);
                return GATHER ? (long long)idx[pos] : pos;
            });
        } else {
            const int base = (t - sr.cache_tiles) * kBf16Tile;
            issue_tile<D, NW, WITH_V>(kb, vb, cache_stride, buf, [&](int r) -> long long { return base + (r < valid ? r : valid - 1); });
        }
    };

#pragma unroll
    for (int t = 0; t < NBUF - 1; ++t)
        if (t < ntiles) issue(t);      // first: the longest dependent chain (index -> row)

    bf16x8_t qf[KS];
    load_q_frag<D>(a, static_cast<const u16 *>(a.q) + z * a.seq_q, h, row, qf);

    f32x16_t o[WITH_V ? DT : 1];
#pragma unroll
    for (int i = 0; i < (WITH_V ? DT : 1); ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;     // running max (log2 domain) and this lane's share of the normaliser
    float m_pre = -INFINITY, l_pre = 0.f;     // the same after the last cache tile (prefix-only statistics)

    for (int t = 0; t < ntiles; ++t) {
        // tile t landed (NBUF-2 younger tiles may still be in flight); everyone is done with tile t-1
        if (t + NBUF - 2 < ntiles) tile_barrier<(NBUF - 2) * LPT>();
        else tile_barrier<0>();
        if (t == 0) MAGE_PROBE_AT(1);
        if (t + NBUF - 1 < ntiles) issue(t + NBUF - 1);
        const int valid = tile_valid(t);
        const unsigned char *kbuf = smem + (t % NBUF) * BUF_BYTES;
        const unsigned char *vbuf = kbuf + G::MAT_BYTES;
        if (WITH_V && t == sr.cache_tiles) {   // first in-block tile: freeze the prefix statistics
            m_pre = m_run;
            l_pre = l_run;
        }

#ifdef MAGE_PROBE_NO_COMPUTE
        if (false) {
#else
        if (wave_active) {
#endif
            // S^T tile: sc[kt][v] = score of query row l32 against key kt*32 + 8*(v/4) + 4*lg + v%4
            f32x16_t sc[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[kt][v] = 0.f;
                bf16x8_t kf[KS];
#pragma unroll
                for (int s = 0; s < KS; ++s) kf[s] = read_k_frag<D>(kbuf, kt * 32 + l32, s, lg);
#pragma unroll
                for (int s = 0; s < KS; ++s) sc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], sc[kt], 0, 0, 0);
            }
            if (valid < kBf16Tile) {           // uniform: only the last tile of a slice has padding keys
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (kt * 32 + 8 * (v >> 2) + 4 * lg + (v & 3) >= valid) sc[kt][v] = -INFINITY;
            }
            float mx = fmaxf(sc[0][0], sc[1][0]);
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, fmaxf(sc[0][v], sc[1][v]));
            mx = fmaxf(mx, __shfl_xor(mx, 32)) * a.scale_log2;
            const float m_new = fmaxf(m_run, mx);
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            const bool grew = m_new > m_run;
            m_run = m_new;
            float psum = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sc[kt][v], a.scale_log2, -m_new));
                    sc[kt][v] = p;
                    psum += p;
                }
            l_run = l_run * corr + psum;

            if (WITH_V) {
                if (__any(grew)) {             // rescale only when some row's maximum moved
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int v = 0; v < 16; ++v) o[dt][v] *= corr;
                }
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int m2 = 0; m2 < 2; ++m2) {
                        bf16x8_t pf;
#pragma unroll
                        for (int e = 0; e < 8; ++e) pf[e] = (__bf16)sc[kt][8 * m2 + e];
                        bf16x8_t vf[DT];
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) vf[dt] = read_vt_frag<D>(vbuf, kt * 32 + m2 * 16 + 4 * lg, dt, lane);
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt], pf, o[dt], 0, 0, 0);
                    }
            }
        }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    MAGE_PROBE_AT(2);
    if (WITH_V && a.stat_m != nullptr) {
        if (sr.blk_tiles == 0) {
            m_pre = m_run;
            l_pre = l_run;
        }
        const float lp = l_pre + __shfl_xor(l_pre, 32);
        if (wave_active && row < a.R && lg == 0) {
            const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
            a.stat_m[pi] = m_pre;
            a.stat_l[pi] = lp;
        }
    }

    if (MODE == MODE_STATS) {
        if (wave_active && row < a.R && lg == 0) {
            const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
            a.part_m[pi] = m_run;
            a.part_l[pi] = l_tot;
        }
        return;
    }

    // Epilogue.  O^T register (dt, v) holds channel d = dt*32 + 8*(v/4) + 4*lg + v%4 of query row
    // `row`.  Two wavefronts at a time transpose their 32 x D block through LDS and write whole
    // rows (16 bytes per lane, consecutive lanes on consecutive addresses).
    constexpr int LPR = D / 4;          // lanes per output row
    constexpr int RPS = 64 / LPR;       // rows per store instruction
    const bool direct = a.n_split == 1;
    const float inv = direct ? 1.f / l_tot : 1.f;
    float *stage = reinterpret_cast<float *>(smem) + (wave & 1) * 32 * OST;
    __syncthreads();                    // every wavefront is done reading the last tile
    for (int round = 0; round < NW / 2; ++round) {
        if ((wave >> 1) == round && wave_active) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    f32x4_t val = {o[dt][4 * v4] * inv, o[dt][4 * v4 + 1] * inv, o[dt][4 * v4 + 2] * inv, o[dt][4 * v4 + 3] * inv};
                    *reinterpret_cast<f32x4_t *>(stage + l32 * OST + dt * 32 + 8 * v4 + 4 * lg) = val;
                }
#pragma unroll
            for (int it = 0; it < 32 / RPS; ++it) {
                const int rr = it * RPS + lane / LPR, col = (lane % LPR) * 4;
                const f32x4_t val = *reinterpret_cast<const f32x4_t *>(stage + rr * OST + col);
                const int orow = row0 + rr;
                if (orow < a.R) {
                    float *dst;
                    if (direct) {
                        const int gl = orow / a.B, qi = orow - gl * a.B;
                        dst = a.out + z * a.seq_out + ((long long)qi * a.Hq + (long long)h * a.G + gl) * D;
                    } else {
                        dst = a.part_o + (((long long)h * a.n_split + split) * a.rpad + orow) * D;
                    }
                    *reinterpret_cast<f32x4_t *>(dst + col) = val;
                }
            }
        }
        __syncthreads();
    }
    MAGE_PROBE_AT(3);
    MAGE_PROBE_FLUSH();
    if (!wave_active || row >= a.R || lg != 0) return;
    if (direct) {
        if (a.lse_out) {
            const int gl = row / a.B, qi = row - gl * a.B;
            a.lse_out[z * a.seq_lse + (long long)qi * a.Hq + (long long)h * a.G + gl] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
        }
    } else {
        const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
        a.part_m[pi] = m_run;
        a.part_l[pi] = l_tot;
    }
}

// Second pass of selection.  Scores are produced untransposed (S = Q K^T: the query fragment
// is the A operand), so a lane holds 16 query rows of ONE key and the sum over rows is in-lane.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void colsum_bf16_kernel(const KernelArgs a)
{
    using G = TileGeom<D>;
    constexpr int KS = D / 16;
    constexpr int BUF_BYTES = G::MAT_BYTES;
    constexpr int NBUF = 3;                                         // LDS tile buffers = prefetch distance + 1
    constexpr int LPT = G::LOADS / NW;                              // loads one wavefront issues per tile
    __shared__ __attribute__((aligned(1024))) unsigned char smem[NBUF * BUF_BYTES];
    __shared__ float red[2][NW][kBf16Tile];

    const int split = blockIdx.x, h = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int row0 = wave * 32;
    const bool wave_active = row0 < a.R;

    const SplitRange sr = split_range(a, split);
    const int ntiles = sr.cache_tiles;
    const long long cache_stride = (long long)a.Hkv * D;
    const u16 *kc = static_cast<const u16 *>(a.kc) + (long long)h * D;

    auto tile_valid = [&](int t) -> int {
        const long long left = sr.c1 - (sr.c0 + (long long)t * kBf16Tile);
        return left < kBf16Tile ? (int)left : kBf16Tile;
    };
    const u16 *kptr[G::LOADS / NW];
    stream_pointers<D, NW>(kc, sr.c0, cache_stride, kptr);
    const long long tile_elems = (long long)kBf16Tile * cache_stride;
    auto issue = [&](int t) {
        const int valid = tile_valid(t);
        unsigned char *buf = smem + (t % NBUF) * BUF_BYTES;
        if (valid == kBf16Tile) {
            issue_tile_stream<D, NW, false>(kptr, tile_elems, 0, t, buf);
        } else {
            const long long base = sr.c0 + (long long)t * kBf16Tile;
            issue_tile<D, NW, false>(kc, kc, cache_stride, buf, [&](int r) -> long long { return base + (r < valid ? r : valid - 1); });
        }
    };
#pragma unroll
    for (int t = 0; t < NBUF - 1; ++t)
        if (t < ntiles) issue(t);

    bf16x8_t qf[KS];
    load_q_frag<D>(a, static_cast<const u16 *>(a.q), h, row0 + l32, qf);

    // per-register row statistics: register v is query row row0 + 8*(v/4) + 4*lg + v%4
    float lse2[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int r = row0 + 8 * (v >> 2) + 4 * lg + (v & 3);
        lse2[v] = r < a.R ? a.lse2[(long long)h * a.rpad + r] : INFINITY;   // exp2(-inf) = 0 for padding rows
    }

    // The cross-wavefront sum of tile t is finished after the barrier of tile t+1 (the `red`
    // buffer alternates), so the loop needs one barrier per tile.
    auto finish = [&](int t) {
        const int valid = tile_valid(t);
        if (threadIdx.x < kBf16Tile && (int)threadIdx.x < valid) {
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) acc += red[t & 1][w][threadIdx.x];
            a.alpha[(long long)h * a.L + sr.c0 + (long long)t * kBf16Tile + threadIdx.x] = acc * a.inv_rows;
        }
    };

    for (int t = 0; t < ntiles; ++t) {
        if (t + NBUF - 2 < ntiles) tile_barrier<(NBUF - 2) * LPT>();
        else tile_barrier<0>();
        if (t + NBUF - 1 < ntiles) issue(t + NBUF - 1);
        if (t > 0) finish(t - 1);
        const unsigned char *kbuf = smem + (t % NBUF) * BUF_BYTES;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            float col = 0.f;
            if (wave_active) {
                f32x16_t sc;
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[v] = 0.f;
                bf16x8_t kf[KS];
#pragma unroll
                for (int s = 0; s < KS; ++s) kf[s] = read_k_frag<D>(kbuf, kt * 32 + l32, s, lg);
#pragma unroll
                for (int s = 0; s < KS; ++s) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[s], kf[s], sc, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; ++v) col += __builtin_amdgcn_exp2f(fmaf(sc[v], a.scale_log2, -lse2[v]));
                col += __shfl_xor(col, 32);
            }
            if (lg == 0) red[t & 1][wave][kt * 32 + l32] = col;
        }
    }
    if (ntiles > 0) {
        __syncthreads();
        finish(ntiles - 1);
    }
}

// ------------------------------------------------------------------------------ launchers
template <int D, int NW, int MODE, bool GATHER>
static hipError_t launch_attn(const KernelArgs &a, int row_groups, hipStream_t stream)
{
    dim3 grid(a.n_split, a.Hkv, row_groups), block(NW * 64);
    hipLaunchKernelGGL((attn_bf16_kernel<D, NW, MODE, GATHER>), grid, block, 0, stream, a);
    return hipGetLastError();
}

template <int D, int NW>
static hipError_t launch_colsum(const KernelArgs &a, hipStream_t stream)
{
    dim3 grid(a.n_split, a.Hkv), block(NW * 64);
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

// Batched sparse step: n_seq independent sequences, one workgroup per (sequence, KV head, row
// group) walks all k + B keys of its head, so every selected row is fetched by exactly one
// workgroup and nothing is merged across workgroups.
hipError_t bf16_attn_batched(const KernelArgs &a, int d, int waves, int row_groups, int n_seq, hipStream_t stream)
{
    dim3 grid(n_seq, a.Hkv, row_groups), block(waves * 64);
    if (d == 128 && waves == 4) hipLaunchKernelGGL((attn_bf16_kernel<128, 4, MODE_ATTN, true>), grid, block, 0, stream, a);
    else if (d == 128 && waves == 8) hipLaunchKernelGGL((attn_bf16_kernel<128, 8, MODE_ATTN, true>), grid, block, 0, stream, a);
    else if (d == 64 && waves == 4) hipLaunchKernelGGL((attn_bf16_kernel<64, 4, MODE_ATTN, true>), grid, block, 0, stream, a);
    else if (d == 64 && waves == 8) hipLaunchKernelGGL((attn_bf16_kernel<64, 8, MODE_ATTN, true>), grid, block, 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
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
