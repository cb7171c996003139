// bf16 MFMA kernels of the MAGE hot path for gfx950 (CDNA4, 64-wide wavefronts).
//
//   attn_bf16_kernel<D,MODE,AHEAD>
//     MODE_ATTN : split-key flash-style attention of the G*B query rows of one KV head over a
//                 slice of keys (contiguous cache rows, then optionally the in-block keys) --
//                 Alg. 1 main stream "Attn(Q,K,V,C)"; also Phase 2 on compacted rows.
//     MODE_STATS: the same score pass without values: per-row reference and normaliser of
//                 softmax(Q1 K^T / sqrt(d)) over the prefix (Alg. 1 select stream, first half).
//     AHEAD     : order of the tile loop (scores one tile ahead of the softmax, or tile by tile).
//   colsum_bf16_kernel<D,NW>
//                 second pass of selection: recomputes the scores, normalises each row with
//                 its final log-sum-exp and averages over the G*B rows (Eq. 5) -> alpha[h,j];
//                 per query head (its B rows, Eq. 2) on request.
//
// Tiling: attention / statistics: one workgroup = 8 wavefronts = 4 row groups of 32 query rows x
// 2 halves of every 64-key tile.  Column sums: 4 or 8 wavefronts, each 32 rows x the whole tile.
//
// Data movement: tiles go HBM -> LDS directly (global_load_lds, 16 bytes per lane, no VGPR
// staging) into a ring of tile buffers, one workgroup barrier per tile.  Rows stay row-major in LDS
// with an XOR swizzle of their 16-byte chunks, so that
//   - the K fragment of a lane (one key row, 8 channels) is one conflict-free ds_read_b128;
//   - the V fragment (8 keys at one channel) is two transposing reads (ds_read_b64_tr_b16), which
//     deliver V^T straight from the row-major tile.
//
// Scores are produced transposed (S^T = K Q^T, v_mfma_f32_32x32x16_bf16 with the K tile as the A
// operand): a lane then holds 16 scores of ONE query row, so the online softmax is in-lane work,
// and the exponentiated scores are already laid out as the B operand of O^T = V^T P^T.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lds_asm.hpp"
#include "ids.hpp"
#include "plan.hpp"

namespace mage {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short u16;

enum { MODE_ATTN = 0, MODE_STATS = 1 };


__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }

// XOR swizzle of the 16-byte chunk index of tile row r.  16 consecutive rows (one ds_read_b128
// phase of the K fragment) and 4 consecutive rows (one half of a transposing V read) both land on
// distinct LDS banks.
template <int D>
__device__ __forceinline__ int swz(int r)
{
    if (D == 256) return r & 15;      // K-only tiles (page-summary rows): any bijection of the low row bits will do
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
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
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

// One matrix of a tile through per-lane element offsets: `rows_to_offsets` works them out from the
// source rows (and keeps them), `issue_offsets` requests the loads.  K and V of a tile share the
// offsets: the V request reuses what the K request of the same tile left behind.
template <int D, int NW, class RowOf>
__device__ __forceinline__ void rows_to_offsets(long long row_stride, RowOf row_of, long long (&off)[TileGeom<D>::LOADS / NW])
{
    using G = TileGeom<D>;
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
#pragma unroll
    for (int n = 0; n < G::LOADS / NW; ++n) {
        const int r = (n * NW + wave) * G::RPI + lane / G::CH;
        off[n] = row_of(r) * row_stride + ((lane % G::CH) ^ swz<D>(r)) * 8;
    }
}

template <int D, int NW>
__device__ __forceinline__ void issue_offsets(const u16 *base, const long long (&off)[TileGeom<D>::LOADS / NW], unsigned char *buf)
{
    using G = TileGeom<D>;
    const int wave = tid_x() >> 6;
#pragma unroll
    for (int n = 0; n < G::LOADS / NW; ++n)
        __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(base + off[n]), MAGE_LDS_PTR(buf + (n * NW + wave) * 1024), 16, 0, 0);
}

// The same for a full tile of contiguous cache rows, written so that the per-tile part of every
// address is wavefront-uniform (scalar registers): `kbase` points at (first row of the tile, this KV
// head, channel 0), `off[n]` is this lane's byte offset inside a tile for load n (constant over the
// tiles), `lds_tile` the LDS byte address of the tile buffer plus this wavefront's 1 KB share.
template <int D, int NW, bool WITH_V>
__device__ __forceinline__ void issue_tile_stream(const unsigned char *kbase, long long v_minus_k_bytes,
                                                  const unsigned (&off)[TileGeom<D>::LOADS / NW], unsigned lds_tile)
{
    using G = TileGeom<D>;
#pragma unroll
    for (int n = 0; n < G::LOADS / NW; ++n) {
        const unsigned dst = lds_tile + n * NW * 1024;
        __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(kbase + off[n]), MAGE_LDS_ADDR(dst), 16, 0, 0);
        if (WITH_V)
            __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(kbase + v_minus_k_bytes + off[n]), MAGE_LDS_ADDR(dst + G::MAT_BYTES), 16, 0, 0);
    }
}

template <int D, int NW>
__device__ __forceinline__ void stream_offsets(long long row_stride, unsigned (&off)[TileGeom<D>::LOADS / NW])
{
    using G = TileGeom<D>;
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
#pragma unroll
    for (int n = 0; n < G::LOADS / NW; ++n) {
        const int r = (n * NW + wave) * G::RPI + lane / G::CH;
        off[n] = (unsigned)(r * row_stride * 2 + ((lane % G::CH) ^ swz<D>(r)) * 16);
    }
}

// Wait until at most PENDING of this wavefront's HBM->LDS loads are outstanding (loads complete in
// issue order, so the oldest tile has landed), then meet the rest of the workgroup.
template <int PENDING>
__device__ __forceinline__ void tile_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(PENDING) : "memory");
    __syncthreads();
}

// Fragment reads.  The swizzle only changes address bits 4..7 (below the row pitch), and so do the
// per-read terms (MFMA k-step for K, O^T tile for V); a row offset leaves those bits alone.  A read
// address is therefore (lane constant) ^ (compile-time constant) + (compile-time offset): one
// VALU op per read and three live address registers for the whole tile loop.
struct FragAddr {
    unsigned k;      // K fragment of key row l32, k-step 0
    unsigned v[2];   // the two transposing reads of a V^T fragment at key block 0, O^T tile 0
};

template <int D>
__device__ __forceinline__ FragAddr frag_addr(int lane)
{
    constexpr int ROW = TileGeom<D>::ROW_BYTES;
    FragAddr f;
    const int l32 = lane & 31, lg = lane >> 5;
    // chunk (2*ks + lg) ^ swz = (2*ks) ^ (lg ^ swz): bit 0 belongs to lg alone
    f.k = (unsigned)(l32 * ROW) | (unsigned)((lg ^ swz<D>(l32)) << 4);
    // V^T: within each 16-lane block, lane i' addresses 4 channels (4*(i' & 3) ..) of key (i' >> 2);
    // the transposing read hands lane i the 4 keys at channel i.  Channel chunk of O^T tile dt is
    // 4*dt + low with low = 2*(blk & 1) + (q >> 1); key = 16*(2*kt + m2) + 8*b + 4*lg + j.
    const int blk = lane >> 4, ip = lane & 15;
    const int j = ip >> 2, q = ip & 3;
    const int low = 2 * (blk & 1) + (q >> 1);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int key = 8 * b + 4 * lg + j;
        f.v[b] = (unsigned)(key * ROW) | (unsigned)((low ^ swz<D>(key)) << 4) | (unsigned)(8 * (q & 1));
    }
    return f;
}

template <int D, bool KEYS_AS_A>
__device__ __forceinline__ void qk_half(unsigned ka, const bf16x8_t (&qf)[D / 16], f32x16_t &sc);

// Scores of one 64-key tile against the wavefront's 32 query rows: two 32-key halves, K fragments
// (key row kt*32 + l32, channels [16*ks + 8*lg, +8)) read KS deep ahead of the MFMA that uses them.
// KEYS_AS_A: S^T = K Q^T (a lane holds 16 keys of one query row); otherwise S = Q K^T.
template <int D, bool KEYS_AS_A>
__device__ __forceinline__ void qk_tile(unsigned ka, const bf16x8_t (&qf)[D / 16], f32x16_t (&sc)[2])
{
    constexpr int KS = D / 16;
    constexpr int HALF = 32 * TileGeom<D>::ROW_BYTES;
    if constexpr (KS > 8) {            // more fragments than the LDS counter can keep apart: one half after the other
        qk_half<D, KEYS_AS_A>(ka, qf, sc[0]);
        qk_half<D, KEYS_AS_A>(ka + HALF, qf, sc[1]);
        return;
    }
    u32x4_t k0[KS], k1[KS];
#pragma unroll
    for (int v = 0; v < 16; ++v) sc[0][v] = sc[1][v] = 0.f;
    static_for<KS>([&](auto S) {
        constexpr int ks = decltype(S)::value;
        k0[ks] = lds_read_b128<0>(ka ^ (unsigned)(ks << 5));
    });
    static_for<KS>([&](auto S) {
        constexpr int ks = decltype(S)::value;
        lds_wait<KS - 1>(k0[ks]);
        const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, k0[ks]);
        sc[0] = KEYS_AS_A ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sc[0], 0, 0, 0)
                          : __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], kf, sc[0], 0, 0, 0);
        k1[ks] = lds_read_b128<HALF>(ka ^ (unsigned)(ks << 5));
    });
    static_for<KS>([&](auto S) {
        constexpr int ks = decltype(S)::value;
        lds_wait<KS - 1 - ks>(k1[ks]);
        const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, k1[ks]);
        sc[1] = KEYS_AS_A ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sc[1], 0, 0, 0)
                          : __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], kf, sc[1], 0, 0, 0);
    });
}

// The same for one 32-key half of a tile (key row l32 of the half that `ka` points at), at most 8
// fragment reads in flight at a time.
template <int D, bool KEYS_AS_A>
__device__ __forceinline__ void qk_half(unsigned ka, const bf16x8_t (&qf)[D / 16], f32x16_t &sc)
{
    constexpr int KS = D / 16;
    constexpr int KB = KS < 8 ? KS : 8;
    static_assert(KS % KB == 0, "k-steps come in whole batches");
#pragma unroll
    for (int v = 0; v < 16; ++v) sc[v] = 0.f;
    static_for<KS / KB>([&](auto BI) {
        constexpr int k0i = decltype(BI)::value * KB;
        u32x4_t k0[KB];
        static_for<KB>([&](auto S) {
            constexpr int i = decltype(S)::value;
            k0[i] = lds_read_b128<0>(ka ^ (unsigned)((k0i + i) << 5));
        });
        static_for<KB>([&](auto S) {
            constexpr int i = decltype(S)::value;
            lds_wait<KB - 1 - i>(k0[i]);
            const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, k0[i]);
            sc = KEYS_AS_A ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[k0i + i], sc, 0, 0, 0)
                           : __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[k0i + i], kf, sc, 0, 0, 0);
        });
    });
}

// V^T fragments of key group g (16 keys: 16*g + 4*lg + {0..3, 8..11}) for all O^T tiles: lane
// holds channel dt*32 + (lane & 31).
template <int D, int GRP>
__device__ __forceinline__ void issue_vt_group(const unsigned (&va)[2], u32x2_t (&vf)[D / 32][2])
{
    constexpr int OFF = GRP * 16 * TileGeom<D>::ROW_BYTES;
    static_for<D / 32>([&](auto T) {
        constexpr int dt = decltype(T)::value;
        vf[dt][0] = lds_read_tr16_b64<OFF>(va[0] ^ (unsigned)(dt << 6));
        vf[dt][1] = lds_read_tr16_b64<OFF>(va[1] ^ (unsigned)(dt << 6));
    });
}

// row / B without a division (inv_B comes from the host)
__device__ __forceinline__ int row_group(const KernelArgs &a, int row)
{
    return a.B == 1 ? row : (int)(((unsigned long long)(unsigned)row * a.inv_B) >> 32);
}

// Query fragment of this lane: row (l % 32) of the wavefront's M tile, 8 consecutive channels
// per MFMA k-step.  Row r of a KV head's row space is (g_local = r / B, q = r % B).
template <int D>
__device__ __forceinline__ void load_q_frag(const KernelArgs &a, const u16 *q, int h, int row, bf16x8_t (&qf)[D / 16])
{
    const int lg = (tid_x() & 63) >> 5;
    if (row < a.R) {
        const int gl = row_group(a, row), qi = row - gl * a.B;
        const u16 *src = q + ((long long)qi * a.Hq + (long long)h * a.G + gl) * D + 8 * lg;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qf[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(src + ks * 16));
    } else {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qf[ks] = as_bf16x8(make_uint4(0, 0, 0, 0));
    }
}

// Which keys does split `s` cover?  Cache tiles are dealt round-robin: split s < n_cyc owns the
// 64-key tiles s, s + n_cyc, s + 2*n_cyc, ...  Workgroups that run at the same time then read one
// moving window of consecutive memory instead of one far-apart stream each, which is the access
// pattern the memory controllers serve fastest.  The block split adds the n_blk in-block keys.
struct SplitRange {
    long long first;      // first key of this split's first tile
    long long step;       // keys between consecutive tiles of this split
    long long nc;         // cache keys in all
    int cache_tiles, blk_tiles;
};

// The tile counts steer every branch of the tile loop; they are the same for all lanes, and
// readfirstlane tells the compiler so (the 64-bit division would otherwise leave them in vector
// registers and turn the loop's control flow into lane masks).
__device__ __forceinline__ SplitRange split_range(const KernelArgs &a, int s)
{
    SplitRange r;
    r.first = (long long)s * kBf16Tile;
    r.step = (long long)a.n_cyc * kBf16Tile;
    r.nc = a.nc;
    // tiles s, s + n_cyc, ... below tiles_q * n_cyc + tiles_r: one more for the first tiles_r splits
    r.cache_tiles = __builtin_amdgcn_readfirstlane(s < a.n_cyc ? a.tiles_q + (s < a.tiles_r ? 1 : 0) : 0);
    r.blk_tiles = __builtin_amdgcn_readfirstlane((s == a.blk_split) ? (a.n_blk + kBf16Tile - 1) / kBf16Tile : 0);
    return r;
}

// Attention / row-statistics pass.  A workgroup is 8 wavefronts: 4 row groups (32 query rows
// each) x 2 key halves of every 64-key tile, one workgroup per CU with a ring of tile buffers that
// fills the LDS, so that four to seven tiles are in flight while one is consumed.  The two
// halves keep separate online-softmax states, merged through LDS after the last tile.
constexpr int kAttnWaves = 8;
constexpr int kAttnRows = 128;   // query rows per workgroup (4 row groups of 32)

template <int D, int MODE>
struct AttnGeom {
    static constexpr bool WITH_V = (MODE == MODE_ATTN);
    // LDS: a ring of NBUF K tiles, then (attention) a ring of NBUF V tiles.  While tile t is
    // consumed, K(t+1) is resident too (its scores are computed one tile ahead) and the next
    // NBUF-1 K tiles / V tiles are in flight.  Attention is register-bound to one workgroup per CU;
    // the K-only pass is lighter on registers and runs two workgroups per CU.
    static constexpr int NBUF = WITH_V ? 4 : 3;
    static constexpr int RING_BYTES = NBUF * TileGeom<D>::MAT_BYTES;
    // the same LDS as NBUF joint K|V tile buffers when scores do not run ahead
    static constexpr int BUF_BYTES = TileGeom<D>::MAT_BYTES * (WITH_V ? 2 : 1);
    static constexpr int TILE_LDS_BYTES = RING_BYTES * (WITH_V ? 2 : 1);
    static constexpr int LPT = (TileGeom<D>::LOADS / kAttnWaves) * (WITH_V ? 2 : 1);            // loads one wavefront issues per tile
    static constexpr int MAX_WAVES_PER_SIMD = (WITH_V || D > 128) ? 2 : 4;
};

template <int D, int MODE, bool AHEAD>
__global__ __launch_bounds__(kAttnWaves * 64) __attribute__((amdgpu_waves_per_eu(2, AttnGeom<D, MODE>::MAX_WAVES_PER_SIMD)))
void attn_bf16_kernel(const KernelArgs a)
{
    using G = TileGeom<D>;
    using AG = AttnGeom<D, MODE>;
    constexpr int NW = kAttnWaves;
    constexpr bool WITH_V = AG::WITH_V;
    constexpr int NBUF = AG::NBUF, LPT = AG::LPT;
    // AHEAD: a ring of K tiles then a ring of V tiles (K runs one tile ahead of V); otherwise a
    // ring of joint K|V buffers
    constexpr int KPITCH = AHEAD ? G::MAT_BYTES : AG::BUF_BYTES;      // bytes between consecutive ring slots
    constexpr int VRING = AHEAD ? AG::RING_BYTES : G::MAT_BYTES;       // where V slots start
    constexpr int KS = D / 16;     // MFMA k-steps over the head dimension
    constexpr int DT = D / 32;     // 32-row tiles of O^T
    constexpr int HALF = 32 * G::ROW_BYTES;
    constexpr int HDT = WITH_V ? DT / 2 : 0;            // O^T tiles each wavefront of a pair finishes
    constexpr int XCH_FLOATS = HDT * 16 * 64;           // accumulators a wavefront hands to its partner
    constexpr int HOST = D / 2 + 4;                     // floats per staged half row
    constexpr int XCH_BYTES = (NW * XCH_FLOATS + NW * 4 * 64) * 4;
    constexpr int STAGE_BYTES = WITH_V ? NW * 32 * HOST * 4 : 0;
    constexpr int TAIL_BYTES = XCH_BYTES > STAGE_BYTES ? XCH_BYTES : STAGE_BYTES;
    constexpr int SMEM_BYTES = AG::TILE_LDS_BYTES > TAIL_BYTES ? AG::TILE_LDS_BYTES : TAIL_BYTES;
    static_assert((NBUF - 1) * LPT < 64, "outstanding loads must fit the counter");

    // tile buffers; after the key loop the same memory carries the merge and the output transposition
    __shared__ __attribute__((aligned(1024))) unsigned char smem[SMEM_BYTES];

    // key splits vary fastest over the grid: consecutive workgroups (dealt round-robin to the XCDs)
    // stream neighbouring tiles of the same head, so every XCD touches every HBM channel.
    const int split = wg_x(), h = wg_y(), rg = wg_z();
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int rgw = wave & 3, kh = wave >> 2;            // row group and key half of this wavefront
    const int row0 = rg * kAttnRows + rgw * 32;              // first row of this wavefront's M tile
    const int row = row0 + l32;
    const bool wave_active = row0 < a.R;

    const SplitRange sr = split_range(a, split);
    const int ntiles = sr.cache_tiles + sr.blk_tiles;

    const long long cache_stride = (long long)a.Hkv * D;
    const u16 *kc = static_cast<const u16 *>(a.kc) + (long long)h * D;
    const u16 *vc = static_cast<const u16 *>(a.vc) + (long long)h * D;
    const u16 *kb = static_cast<const u16 *>(a.kblk) + (long long)h * D;
    const u16 *vb = static_cast<const u16 *>(a.vblk) + (long long)h * D;

    auto tile_valid = [&](int t) -> int {
        if (t < sr.cache_tiles) {
            const long long left = sr.nc - (sr.first + t * sr.step);
            return left < kBf16Tile ? (int)left : kBf16Tile;
        }
        const int left = a.n_blk - (t - sr.cache_tiles) * kBf16Tile;
        return left < kBf16Tile ? left : kBf16Tile;
    };
    unsigned soff[G::LOADS / NW];      // this lane's byte offsets inside a streamed tile
    stream_offsets<D, NW>(cache_stride, soff);
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds_addr(smem) + wave * 1024);
    // Tiles 0 .. n_full-1 are whole tiles of contiguous cache rows: the common case takes one
    // comparison per tile; everything else (a ragged last tile, in-block keys) goes through the
    // general path.
    const int n_full = sr.cache_tiles - ((sr.cache_tiles > 0 && tile_valid(sr.cache_tiles - 1) < kBf16Tile) ? 1 : 0);
    // one matrix (K: IS_V = false, V: true) of tile t into its ring slot; outside the common case
    // the V request of a tile reuses the offsets of its K request, which must be the latest one
    long long goff[G::LOADS / NW];
    auto issue = [&](int t, auto IS_V) {
        constexpr bool is_v = decltype(IS_V)::value;
        const unsigned slot = (is_v ? VRING : 0) + (t % NBUF) * KPITCH;
        const u16 *cache = is_v ? vc : kc, *blk = is_v ? vb : kb;
        if (t < n_full) {
            issue_tile_stream<D, NW, false>(reinterpret_cast<const unsigned char *>(cache + (sr.first + t * sr.step) * cache_stride),
                                            0, soff, lds_wave + slot);
            return;
        }
        if (t >= ntiles) return;
        if constexpr (!is_v) {
            const int valid = tile_valid(t);
            if (t < sr.cache_tiles) {
                const long long base = sr.first + t * sr.step;
                rows_to_offsets<D, NW>(cache_stride, [&](int r) -> long long { return base + (r < valid ? r : valid - 1); }, goff);
            } else {
                const int base = (t - sr.cache_tiles) * kBf16Tile;
                rows_to_offsets<D, NW>(cache_stride, [&](int r) -> long long { return base + (r < valid ? r : valid - 1); }, goff);
            }
        }
        issue_offsets<D, NW>(t < sr.cache_tiles ? cache : blk, goff, smem + slot);
    };
    auto issue_k = [&](int t) { issue(t, std::false_type{}); };
    auto issue_v = [&](int t) { if (WITH_V) issue(t, std::true_type{}); };

    // queries first: waiting for them later (loads retire in order) must not mean waiting for tiles
    bf16x8_t qf[KS];
    load_q_frag<D>(a, static_cast<const u16 *>(a.q), h, row, qf);
    // load order (loads retire in it).  AHEAD: K(0), then pairs [V(j), K(j+1)].  Otherwise pairs
    // [K(j), V(j)].  Either way the V request follows the K request of the same tile directly.
    if constexpr (AHEAD) issue_k(0);
#pragma unroll
    for (int j = 0; j < NBUF - 1; ++j) {
        if constexpr (AHEAD) {
            issue_v(j);
            issue_k(j + 1);
        } else {
            issue_k(j);
            issue_v(j);
        }
    }
    FragAddr fa = frag_addr<D>(lane);
    fa.k += kh * HALF;                 // this wavefront's half of every tile
    fa.v[0] += kh * HALF;
    fa.v[1] += kh * HALF;
    const unsigned smem_addr = lds_addr(smem);

    f32x16_t o[WITH_V ? DT : 1];
#pragma unroll
    for (int i = 0; i < (WITH_V ? DT : 1); ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
    // Online softmax with a lazily raised reference: probabilities are taken against m_run (log2
    // domain), which follows the row maximum only when that has run ahead by more than kLazy, so
    // the accumulators are rescaled on few tiles instead of on almost every one (any reference
    // gives the same ratios; fp32 sums and bf16 probabilities have the exponent range to spare).
    // The reference starts at a finite floor: rows that have seen padding keys only keep it and
    // a zero sum, without any inf - inf.
    constexpr float kLazy = 8.f, kFloor = -3.0e38f;
    float m_run = kFloor, l_run = 0.f;        // reference and this lane's share of the normaliser
    float m_pre = kFloor, l_pre = 0.f;        // the same after the last cache tile (prefix-only statistics)

    // the query fragments must have arrived before the loop: a wait for them inside it would be a
    // wait for every tile load in flight, once per tile
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qf[ks]));

    // AHEAD: scores run one tile ahead of the softmax: S^T(t+1) is accumulated by the matrix cores
    // while the vector ALU exponentiates S^T(t), the two interleaved instruction by instruction.
    // It pays where the loop is long and bound by memory (the tile requests go out earlier in the
    // iteration); short loops and workgroups that share their tiles with a second row group run the
    // plain order, which has fewer instructions per tile.
    // sc[v] = score of query row l32 against key kh*32 + 8*(v/4) + 4*lg + v%4
    f32x16_t sc_cur, sc_nxt;
    if constexpr (AHEAD) {
        if (ntiles >= NBUF) tile_barrier<(NBUF - 1) * LPT>();       // K(0) landed
        else tile_barrier<0>();
        if (wave_active) qk_half<D, true>(smem_addr + fa.k, qf, sc_cur);
    }

    for (int t = 0; t < ntiles; ++t) {
        // AHEAD: V(t) and K(t+1) landed; otherwise K(t) and V(t).  NBUF-2 younger pairs may still be
        // in flight; everyone is done with the tiles before.
        if (t + NBUF - (AHEAD ? 1 : 2) < ntiles) tile_barrier<(NBUF - 2) * LPT>();
        else tile_barrier<0>();
        if constexpr (AHEAD) {
            issue_v(t + NBUF - 1);
            issue_k(t + NBUF);
        } else {
            issue_k(t + NBUF - 1);
            issue_v(t + NBUF - 1);
        }
        // keep the per-read address arithmetic inside the loop: hoisted, it would pin dozens of registers
        asm volatile("" : "+v"(fa.k), "+v"(fa.v[0]), "+v"(fa.v[1]));
        if (WITH_V && t == sr.cache_tiles) {   // first in-block tile: freeze the prefix statistics
            m_pre = m_run;
            l_pre = l_run;
        }

        if (wave_active) {
            // K fragments of the next tile (its ring slot holds stale data after the last tile: the
            // scores computed from it are never used)
            const unsigned ka = smem_addr + ((t + (AHEAD ? 1 : 0)) % NBUF) * KPITCH + fa.k;
            constexpr bool INTERLEAVE = AHEAD && KS <= 8;    // k-steps of the next tile between the pieces of the softmax
            constexpr int KI = INTERLEAVE ? KS : 1;
            u32x4_t kf[KI];
            if constexpr (!AHEAD) qk_half<D, true>(ka, qf, sc_cur);
            if constexpr (INTERLEAVE) {
                static_for<KS>([&](auto S) {
                    constexpr int i = decltype(S)::value;
                    kf[i] = lds_read_b128<0>(ka ^ (unsigned)(i << 5));
                });
            }
            const unsigned vt = smem_addr + VRING + (t % NBUF) * KPITCH;
            const unsigned va[2] = {vt + fa.v[0], vt + fa.v[1]};
            u32x2_t vf[2][DT][2];
            if constexpr (!AHEAD && WITH_V) issue_vt_group<D, 0>(va, vf[0]);      // the first V^T fragments travel while the softmax runs

            if (t >= n_full) {                 // uniform: only the last tile of a slice can have padding keys
                const int valid = tile_valid(t);
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (kh * 32 + 8 * (v >> 2) + 4 * lg + (v & 3) >= valid) sc_cur[v] = -INFINITY;
            }
            float mx = sc_cur[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sc_cur[v]);
            {   // the other 16 keys of this row sit in the other half of the wavefront
                float lo, hi;
                lane_halves(mx, lo, hi);
                mx = fmaxf(lo, hi) * a.scale_log2;
            }
            if (__any(mx > m_run + kLazy)) {      // uniform: some row's maximum has run ahead of its reference
                const float m_new = fmaxf(m_run, mx);
                const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
                m_run = m_new;
                l_run *= corr;
                if constexpr (WITH_V) {
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int v = 0; v < 16; ++v) o[dt][v] *= corr;
                }
            }
            const float m_new = m_run;
            float psum = 0.f;
            if constexpr (INTERLEAVE) {
                constexpr int VPS = 16 / KS;      // scores exponentiated per MFMA k-step
#pragma unroll
                for (int v = 0; v < 16; ++v) sc_nxt[v] = 0.f;
                static_for<KS>([&](auto S) {
                    constexpr int i = decltype(S)::value;
                    constexpr int VR = (WITH_V && i >= 1) ? 2 * DT : 0;     // V^T reads requested behind the K fragments
                    lds_wait<KS - 1 - i + VR>(kf[i]);
                    sc_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[i]), qf[i], sc_nxt, 0, 0, 0);
                    if constexpr (WITH_V && i == 0) issue_vt_group<D, 0>(va, vf[0]);
#pragma unroll
                    for (int e = 0; e < VPS; ++e) {
                        float p = __builtin_amdgcn_exp2f(fmaf(sc_cur[i * VPS + e], a.scale_log2, -m_new));
                        asm volatile("" : "+v"(p));        // computed here, between two MFMAs, not wherever it is first used
                        sc_cur[i * VPS + e] = p;
                        psum += p;
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sc_cur[v], a.scale_log2, -m_new));
                    sc_cur[v] = p;
                    psum += p;
                }
                if constexpr (AHEAD) {
                    if constexpr (WITH_V) issue_vt_group<D, 0>(va, vf[0]);
                    qk_half<D, true>(ka, qf, sc_nxt);
                }
            }
            l_run += psum;

            if constexpr (WITH_V) {
                // key group g (16 keys): P^T fragment from sc_cur[8*g ..]; the V^T fragments of group 1
                // are requested before group 0 is consumed
                static_for<2>([&](auto GI) {
                    constexpr int g = decltype(GI)::value;
                    bf16x8_t pf;
#pragma unroll
                    for (int e = 0; e < 8; ++e) pf[e] = (__bf16)sc_cur[8 * g + e];
                    if constexpr (g == 0) issue_vt_group<D, 1>(va, vf[1]);
                    static_for<DT>([&](auto T) {
                        constexpr int dt = decltype(T)::value;
                        lds_wait<(g == 0 ? 2 * DT : 0) + 2 * (DT - 1 - dt)>(vf[g][dt][0], vf[g][dt][1]);
                        const u32x4_t both = {vf[g][dt][0][0], vf[g][dt][0][1], vf[g][dt][1][0], vf[g][dt][1][1]};
                        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, both), pf, o[dt], 0, 0, 0);
                    });
                });
            }
            if constexpr (AHEAD) sc_cur = sc_nxt;
        }
    }

    float l_tot = l_run + __shfl_xor(l_run, 32);
    float lp_tot = l_pre + __shfl_xor(l_pre, 32);
    if (sr.blk_tiles == 0) {
        m_pre = m_run;
        lp_tot = l_tot;
    }

    // Merge of the two key halves.  Both wavefronts of a row group end up with the merged
    // statistics, and each finishes one half of the channels: it hands the other half of its
    // accumulators to its partner through LDS (16-byte lane-contiguous pieces).
    float *xch = reinterpret_cast<float *>(smem);                      // [wave][HDT * 4][64] x 4 floats
    float *xstat = xch + NW * XCH_FLOATS;                              // [wave][4][64]
    auto hand_over = [&](auto FOREIGN) {                               // FOREIGN: first O^T tile of the half to give away
        constexpr int f0 = decltype(FOREIGN)::value;
#pragma unroll
        for (int i = 0; i < HDT; ++i)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const f32x4_t val = {o[f0 + i][4 * v4], o[f0 + i][4 * v4 + 1], o[f0 + i][4 * v4 + 2], o[f0 + i][4 * v4 + 3]};
                *reinterpret_cast<f32x4_t *>(xch + (((wave * HDT + i) * 4 + v4) * 64 + lane) * 4) = val;
            }
    };
    float fa_ = 1.f, fb_ = 1.f;
    auto take_over = [&](auto OWN) {
        constexpr int o0 = decltype(OWN)::value;
        const int partner = wave ^ 4;
#pragma unroll
        for (int i = 0; i < HDT; ++i)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const f32x4_t ob = *reinterpret_cast<const f32x4_t *>(xch + (((partner * HDT + i) * 4 + v4) * 64 + lane) * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) o[o0 + i][4 * v4 + e] = o[o0 + i][4 * v4 + e] * fa_ + ob[e] * fb_;
            }
    };
    __syncthreads();                    // every wavefront is done reading the last tile
    if (wave_active) {
        if constexpr (WITH_V) {
            if (kh == 0) hand_over(std::integral_constant<int, HDT>{});
            else hand_over(std::integral_constant<int, 0>{});
        }
        float *st = xstat + wave * 4 * 64 + lane;
        st[0] = m_run;
        st[64] = l_tot;
        st[128] = m_pre;
        st[192] = lp_tot;
    }
    __syncthreads();
    if (wave_active) {
        const float *st = xstat + (wave ^ 4) * 4 * 64 + lane;
        const float m_b = st[0], l_b = st[64], mp_b = st[128], lp_b = st[192];
        const float m = fmaxf(m_run, m_b);
        fa_ = m_run == m ? 1.f : __builtin_amdgcn_exp2f(m_run - m);
        fb_ = m_b == m ? 1.f : __builtin_amdgcn_exp2f(m_b - m);
        l_tot = l_tot * fa_ + l_b * fb_;
        m_run = m;
        const float mp = fmaxf(m_pre, mp_b);
        lp_tot = lp_tot * (m_pre == mp ? 1.f : __builtin_amdgcn_exp2f(m_pre - mp)) + lp_b * (mp_b == mp ? 1.f : __builtin_amdgcn_exp2f(mp_b - mp));
        m_pre = mp;
        if constexpr (WITH_V) {
            if (kh == 0) take_over(std::integral_constant<int, 0>{});
            else take_over(std::integral_constant<int, HDT>{});
        }
    }
    const bool owner = kh == 0 && wave_active;      // writes the per-row scalars

    if (WITH_V && a.stat_m != nullptr) {
        if (owner && row < a.R && lg == 0) {
            const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
            a.stat_m[pi] = m_pre;
            a.stat_l[pi] = lp_tot;
        }
    }

    if (MODE == MODE_STATS) {
        if (owner && row < a.R && lg == 0) {
            const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
            a.part_m[pi] = m_run;
            a.part_l[pi] = l_tot;
        }
        return;
    }

    // Output.  O^T register (dt, v) holds channel d = dt*32 + 8*(v/4) + 4*lg + v%4 of query row
    // `row`: every lane owns runs of 4 consecutive channels (16 bytes), and the two lane halves
    // of a row together 32 consecutive bytes, which the L2 merges into full lines.  Written straight
    // from the registers: a transposition through LDS into whole rows costs more time (two more LDS
    // passes and a barrier at the end of every workgroup) than the narrower stores do.
    const bool direct = a.n_split == 1;
    const float inv = direct ? 1.f / l_tot : 1.f;
    auto put_out = [&](auto OWN) {
        constexpr int o0 = decltype(OWN)::value;
        if (row >= a.R) return;
        float *dst;
        if (direct) {
            const int gl = row_group(a, row), qi = row - gl * a.B;
            dst = a.out + ((long long)qi * a.Hq + (long long)h * a.G + gl) * D;
        } else {
            dst = a.part_o + (((long long)h * a.n_split + split) * a.rpad + row) * D;
        }
#pragma unroll
        for (int i = 0; i < HDT; ++i)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const f32x4_t val = {o[o0 + i][4 * v4] * inv, o[o0 + i][4 * v4 + 1] * inv, o[o0 + i][4 * v4 + 2] * inv, o[o0 + i][4 * v4 + 3] * inv};
                *reinterpret_cast<f32x4_t *>(dst + (o0 + i) * 32 + 8 * v4 + 4 * lg) = val;
            }
    };
    if (wave_active) {
        if (kh == 0) put_out(std::integral_constant<int, 0>{});
        else put_out(std::integral_constant<int, HDT>{});
    }
    if (!owner || row >= a.R || lg != 0) return;
    if (direct) {
        if (a.lse_out) {
            const int gl = row_group(a, row), qi = row - gl * a.B;
            a.lse_out[(long long)qi * a.Hq + (long long)h * a.G + gl] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
        }
    } else {
        const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
        a.part_m[pi] = m_run;
        a.part_l[pi] = l_tot;
    }
}

// Second pass of selection.  Scores are produced untransposed (S = Q K^T: the query fragment
// is the A operand), so a lane holds 16 query rows of ONE key and the sum over rows is in-lane.
// Registers are capped so that the LDS, not the register file, decides how many workgroups share
// a CU: three of the 4-wavefront kind, two of the 8-wavefront kind (d = 256: one fewer).
template <int D, int NW>
struct ColsumGeom {
    static constexpr int WAVES_PER_SIMD = D > 128 ? (NW == 8 ? 2 : 1) : (NW == 8 ? 4 : 3);   // d = 256: one workgroup per CU (100 KB of tiles)
};

template <int D, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(ColsumGeom<D, NW>::WAVES_PER_SIMD, ColsumGeom<D, NW>::WAVES_PER_SIMD)))
void colsum_bf16_kernel(const KernelArgs a)
{
    using G = TileGeom<D>;
    constexpr int KS = D / 16;
    constexpr int BUF_BYTES = G::MAT_BYTES;
    constexpr int NBUF = 3;                                         // LDS tile buffers = prefetch distance + 1
    constexpr int LPT = G::LOADS / NW;                              // loads one wavefront issues per tile
    __shared__ __attribute__((aligned(1024))) unsigned char smem[NBUF * BUF_BYTES];
    __shared__ float red[2][NW][kBf16Tile];
    __shared__ float ring[kColsumTiles][kBf16Tile];
    static_assert(kColsumTiles % NW == 0, "flush deals the ring slots to the wavefronts");

    // One grid row per KV head sums all G*B rows of the head (Eq. 5); with head_rows = B there is
    // one grid row per query head, which sums the B rows of that head alone (Eq. 2 per head).
    const int split = wg_x(), hy = wg_y();
    const bool per_head = a.head_rows > 0;
    const int h = per_head ? hy / a.G : hy;                     // KV head whose keys are read
    const int row_lo = per_head ? (hy % a.G) * a.B : 0;         // first row (of the KV head's row space) summed here
    const int R = per_head ? a.head_rows : a.R;
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int row0 = wave * 32;
    const bool wave_active = row0 < R;

    const SplitRange sr = split_range(a, split);
    const int ntiles = sr.cache_tiles;
    const long long cache_stride = (long long)a.Hkv * D;
    const u16 *kc = static_cast<const u16 *>(a.kc) + (long long)h * D;

    // The tiles of a split are walked from the END of the cache towards its start: the pass before this
    // one (row statistics, or the exact attention of the fused step 1) streamed the cache front to back, so
    // its last part is what the memory-side cache (256 MB) still holds, and this pass meets it first.
    auto tile_key = [&](int t) -> long long { return sr.first + (long long)(sr.cache_tiles - 1 - t) * sr.step; };
    auto tile_valid = [&](int t) -> int {
        const long long left = sr.nc - tile_key(t);
        return left < kBf16Tile ? (int)left : kBf16Tile;
    };
    unsigned soff[G::LOADS / NW];
    stream_offsets<D, NW>(cache_stride, soff);
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds_addr(smem) + wave * 1024);
    // all tiles but possibly one (the last of the cache, walked first) are whole
    auto issue = [&](int t) {
        if (tile_valid(t) == kBf16Tile) {
            issue_tile_stream<D, NW, false>(reinterpret_cast<const unsigned char *>(kc + tile_key(t) * cache_stride), 0, soff,
                                            lds_wave + (t % NBUF) * BUF_BYTES);
        } else {
            const int valid = tile_valid(t);
            const long long base = tile_key(t);
            issue_tile<D, NW, false>(kc, kc, cache_stride, smem + (t % NBUF) * BUF_BYTES,
                                     [&](int r) -> long long { return base + (r < valid ? r : valid - 1); });
        }
    };
#pragma unroll
    for (int t = 0; t < NBUF - 1; ++t)
        if (t < ntiles) issue(t);

    bf16x8_t qf[KS];
    load_q_frag<D>(a, static_cast<const u16 *>(a.q), h, row_lo + row0 + l32, qf);
    FragAddr fa = frag_addr<D>(lane);
    const unsigned smem_addr = lds_addr(smem);

    // per-register row statistics: register v is query row row_lo + row0 + 8*(v/4) + 4*lg + v%4
    float lse2[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int r = row0 + 8 * (v >> 2) + 4 * lg + (v & 3);
        lse2[v] = r < R ? a.lse2[(long long)h * a.rpad + row_lo + r] : INFINITY;   // exp2(-inf) = 0 for rows outside the sum
    }

    // The cross-wavefront sum of tile t is finished after the barrier of tile t+1 (the `red`
    // buffer alternates), so the loop needs one barrier per tile.  Finished sums wait in `ring` and
    // leave together: a global store inside the loop would sit in the same counter as the tile
    // loads and hold up the wavefront that issued it at every barrier.  `red` and `ring` are read
    // and written with inline assembly for the same reason as the tiles.
    const unsigned red_addr = lds_addr(red), ring_addr = lds_addr(ring);
    auto finish = [&](int t) {
        if (tid_x() < kBf16Tile) {
            const unsigned src = red_addr + ((t & 1) * NW * kBf16Tile + tid_x()) * 4;
            float part[NW];
            static_for<NW>([&](auto W) {
                constexpr int w = decltype(W)::value;
                part[w] = lds_read_f32<w * kBf16Tile * 4>(src);
            });
            float acc = 0.f;
            static_for<NW>([&](auto W) {
                constexpr int w = decltype(W)::value;
                lds_wait<NW - 1 - w>(part[w]);
                acc += part[w];
            });
            acc *= a.inv_rows;
            const unsigned dst = ring_addr + ((t % kColsumTiles) * kBf16Tile + tid_x()) * 4;
            asm volatile("ds_write_b32 %0, %1" ::"v"(dst), "v"(acc) : "memory");
        }
    };
    // write out the sums of tiles [t0, t0 + n), n <= kColsumTiles; the caller has put a barrier
    // between the last finish() and this
    auto flush = [&](int t0, int n) {
#pragma unroll
        for (int j = 0; j < kColsumTiles / NW; ++j) {
            const int slot = j * NW + wave;
            const int t = t0 + slot;
            if (slot < n) {                                  // uniform per wavefront
                const bool live = lane < tile_valid(t);
                float v = 0.f;
                if (live) {
                    v = lds_read_f32<0>(ring_addr + ((t % kColsumTiles) * kBf16Tile + lane) * 4);
                    lds_wait<0>(v);
                    a.alpha[(long long)hy * a.L + tile_key(t) + lane] = v;
                }
                if (a.gmax != nullptr) {                     // maxima of 16 consecutive keys, for the top-k filter
                    float g = v;
#pragma unroll
                    for (int d = 1; d < kGroupKeys; d <<= 1) g = fmaxf(g, __shfl_xor(g, d));
                    if (live && (lane & (kGroupKeys - 1)) == 0)
                        a.gmax[(long long)hy * ((a.L + kGroupKeys - 1) / kGroupKeys) + (tile_key(t) + lane) / kGroupKeys] = g;
                }
            }
        }
    };
    auto lds_barrier = [] {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __syncthreads();
    };

    int flushed = 0;          // tiles [0, flushed) have left the ring
    for (int t = 0; t < ntiles; ++t) {
        if (t + NBUF - 2 < ntiles) tile_barrier<(NBUF - 2) * LPT>();
        else tile_barrier<0>();
        if (t + NBUF - 1 < ntiles) issue(t + NBUF - 1);
        if (t > flushed) finish(t - 1);
        const unsigned tile_addr = smem_addr + (t % NBUF) * BUF_BYTES;
        asm volatile("" : "+v"(fa.k));
        float col[2] = {0.f, 0.f};
        if (wave_active) {
            // sc[v] = score of query row row0 + 8*(v/4) + 4*lg + v%4 against key kt*32 + l32
            auto sum_rows = [&](const f32x16_t &sc, float &col) {
#pragma unroll
                for (int v = 0; v < 16; ++v) col += __builtin_amdgcn_exp2f(fmaf(sc[v], a.scale_log2, -lse2[v]));
                // the other 16 rows of this key sit in the other half of the wavefront
                float lo, hi;
                lane_halves(col, lo, hi);
                col = lo + hi;
            };
            if constexpr (NW == 8) {
                // one key half after the other: half the fragment and score registers, which is what
                // lets two 8-wavefront workgroups share a CU
                constexpr int HALF = 32 * G::ROW_BYTES;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) {
                    f32x16_t sc;
                    qk_half<D, false>(tile_addr + fa.k + kt * HALF, qf, sc);
                    sum_rows(sc, col[kt]);
                }
            } else {
                f32x16_t sc[2];
                qk_tile<D, false>(tile_addr + fa.k, qf, sc);
                sum_rows(sc[0], col[0]);
                sum_rows(sc[1], col[1]);
            }
        }
        if (lg == 0) {
            const unsigned dst = red_addr + (((t & 1) * NW + wave) * kBf16Tile + l32) * 4;
            asm volatile("ds_write_b32 %0, %1\n\tds_write_b32 %0, %2 offset:128" ::"v"(dst), "v"(col[0]), "v"(col[1]) : "memory");
        }
        if (t - flushed == kColsumTiles - 1 || t == ntiles - 1) {   // ring full, or done: drain it
            lds_barrier();
            finish(t);
            lds_barrier();
            flush(flushed, t + 1 - flushed);
            flushed = t + 1;
        }
    }
}

// ------------------------------------------------------------------------------ launchers
// the division results the kernels would otherwise start with
static KernelArgs fill_split_consts(const KernelArgs &k)
{
    KernelArgs a = k;
    const long long tiles = (a.nc + kBf16Tile - 1) / kBf16Tile;
    const int n = a.n_cyc > 0 ? a.n_cyc : 1;
    a.tiles_q = (int)(tiles / n);
    a.tiles_r = (int)(tiles % n);
    a.inv_B = a.B >= 2 ? (unsigned)(((1ull << 32) + a.B - 1) / a.B) : 0u;
    return a;
}

template <int D, int MODE, bool AHEAD>
static hipError_t launch_attn(const KernelArgs &k, int row_groups, int grid_x, hipStream_t stream)
{
    if ((long long)k.R * k.B >= (1ll << 32)) return hipErrorInvalidValue;      // row_group's precondition
    const KernelArgs a = fill_split_consts(k);
    dim3 grid(grid_x, a.Hkv, row_groups), block(kAttnWaves * 64);
    hipLaunchKernelGGL((attn_bf16_kernel<D, MODE, AHEAD>), grid, block, 0, stream, a);
    return hipGetLastError();
}

template <int D, int NW>
static hipError_t launch_colsum(const KernelArgs &k, hipStream_t stream)
{
    if ((long long)k.R * k.B >= (1ll << 32)) return hipErrorInvalidValue;      // row_group's precondition
    const KernelArgs a = fill_split_consts(k);
    dim3 grid(a.n_split, a.head_rows > 0 ? a.Hq : a.Hkv), block(NW * 64);
    hipLaunchKernelGGL((colsum_bf16_kernel<D, NW>), grid, block, 0, stream, a);
    return hipGetLastError();
}

// Scores one tile ahead (see the kernel) for long, memory-bound tile loops of workgroups that have
// their tiles to themselves; measured on MI355X, the plain order is faster for shorter loops and
// where two row groups stream the same tiles.
static bool scores_ahead(const KernelArgs &a, int row_groups)
{
    const long long tiles = (a.nc + kBf16Tile - 1) / kBf16Tile;
    return row_groups == 1 && tiles / (a.n_cyc > 0 ? a.n_cyc : 1) >= 24;
}

template <int D>
static hipError_t launch_attn_any(const KernelArgs &a, int row_groups, hipStream_t stream)
{
    return scores_ahead(a, row_groups) ? launch_attn<D, MODE_ATTN, true>(a, row_groups, a.n_split, stream)
                                       : launch_attn<D, MODE_ATTN, false>(a, row_groups, a.n_split, stream);
}

// dense keys only (the whole cache, or compacted rows): gathered rows are sparse_bf16.hip's
hipError_t bf16_attn(const KernelArgs &a, int d, int row_groups, hipStream_t stream)
{
    if (d == 128) return launch_attn_any<128>(a, row_groups, stream);
    if (d == 64) return launch_attn_any<64>(a, row_groups, stream);
    return hipErrorInvalidValue;
}

hipError_t bf16_stats(const KernelArgs &a, int d, int row_groups, hipStream_t stream)
{
    // two workgroups per CU already overlap each other's phases: the plain order measured faster
    if (d == 128) return launch_attn<128, MODE_STATS, false>(a, row_groups, a.n_split, stream);
    if (d == 64) return launch_attn<64, MODE_STATS, false>(a, row_groups, a.n_split, stream);
    if (d == 256) return launch_attn<256, MODE_STATS, false>(a, row_groups, a.n_split, stream);   // page-summary rows [max | min] of d = 128
    return hipErrorInvalidValue;
}

hipError_t bf16_colsum(const KernelArgs &a, int d, int waves, hipStream_t stream)
{
    if (d == 128 && waves == 4) return launch_colsum<128, 4>(a, stream);
    if (d == 128 && waves == 8) return launch_colsum<128, 8>(a, stream);
    if (d == 64 && waves == 4) return launch_colsum<64, 4>(a, stream);
    if (d == 64 && waves == 8) return launch_colsum<64, 8>(a, stream);
    if (d == 256 && waves == 4) return launch_colsum<256, 4>(a, stream);
    if (d == 256 && waves == 8) return launch_colsum<256, 8>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace mage
