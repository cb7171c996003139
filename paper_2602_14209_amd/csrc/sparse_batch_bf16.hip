// Batched sparse step for gfx950 (bandwidth mode) -- Alg. 1 Phase 2 "SparseAttn(Q_h,K_h,V_h,C[S])" for
// n_seq independent sequences in one launch: softmax over the k selected cache rows of a KV head plus
// the block's own B keys, for every (sequence, KV head).
//
// A launch carries hundreds of such problems, so the design aims at keeping the memory system busy all
// the time rather than at the latency of one problem:
//   - one workgroup per (sequence, KV head, 128-row group): 8 wavefronts, each owning 16 query rows for
//     ALL keys (no key split, so nothing is merged or exchanged between wavefronts at the end);
//   - v_mfma_f32_16x16x32_bf16 with small per-wavefront state (O^T of 16 rows: 32 registers), so that
//     four wavefronts fit a SIMD and TWO workgroups share a CU: while one runs its prologue (index
//     entries, then rows: two dependent memory round trips), waits at a barrier or writes its output,
//     the other computes;
//   - key positions form one sequence (0..k-1 the selected cache rows, then the in-block rows), cut into
//     32-key tiles that go HBM -> LDS directly (global_load_lds) into a ring of four K|V buffers, three
//     tiles in flight per workgroup, one barrier per tile; every selected row is fetched by exactly
//     one workgroup (R <= 128);
//   - the index entries wait in LDS (fetched in one go at the start): an entry loaded into a register
//     right before its row is requested would sit behind every tile load in flight (loads retire in
//     order), i.e. drain the ring at every tile;
//   - with so little matrix work per tile (16 MFMAs per wavefront) the tile loop is bound by the number
//     of vector-ALU instructions issued around them, so those are kept few: every LDS fragment address
//     is a lane constant plus the ring slot's offset, and what depends on the wavefront number alone
//     stays in scalar registers.  (Unrolling the tile loop over the ring turns the slot into an
//     immediate, twelve additions less per tile, and doubles the code: measured the same, 40.3 us at 64
//     sequences either way, so the loop is rolled.)  What then bounds a workgroup that has its CU to
//     itself is the LDS: every wavefront reads the whole K and V tile (128 KB per tile and workgroup).
// Scores are produced transposed (S^T = K Q^T: a lane holds 4 keys of ONE query row per 16-key block),
// so the probabilities are already the B operand of O^T = V^T P^T; V^T fragments come from transposing
// LDS reads of the row-major tile.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lds_asm.hpp"
#include "ids.hpp"
#include "plan.hpp"

namespace mage {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned short u16;

constexpr int SB_WAVES = 8;
constexpr int SB_ROWS = SB_WAVES * 16;       // query rows per workgroup
constexpr int SB_TK = 32;                    // keys per tile (two 16-key MFMA blocks)
constexpr int SB_NBUF = 4;                   // ring slots
constexpr int SB_IDX_TILES = 64;             // tiles whose index entries LDS holds at a time (2048 entries)

// What the kernel needs of a call, packed: the kernel arguments arrive through scalar loads that the very
// first instructions wait for, so they are few and adjacent, and what the host can work out is worked out
// there (the divisions by Hkv and B become a multiply-high).
struct BatchArgs {
    const void *q, *kc, *vc, *kblk, *vblk;
    const int32_t *idx;
    float *out, *lse_out;
    long long seq_q, seq_kv, seq_idx, seq_blk, seq_out, seq_lse;   // element strides between sequences
    int B, Hq, Hkv, G, R;
    int nk, n_blk;               // selected cache rows, the block's own rows (0 = none)
    int n_units;                 // n_seq * Hkv
    unsigned inv_Hkv;            // ceil(2^32 / Hkv) for Hkv >= 2: unit / Hkv == mulhi(unit, inv_Hkv) while unit * Hkv < 2^32
    unsigned inv_B;              // the same for B (row * B < 2^32)
    float scale_log2;
};

constexpr int SB_GRID_Y = 32768;            // workgroup id: x = place inside a block of ids, (z, y) = block (y < SB_GRID_Y)

// XOR swizzle of the 16-byte chunk index of tile row r (taken modulo 16): the 16 rows of a K fragment
// read and the 8 rows of one phase of a transposing V read land on distinct LDS banks.
__device__ __forceinline__ int sb_swz(int r) { return ((r & 7) << 1) | ((r >> 3) & 1); }

// Tile t has landed once at most N younger row requests of this wavefront are in flight; every LDS read issued so far
// has returned.  a, b: the index-entry registers (the same one twice where a wavefront has a single entry).
template <int N>
__device__ __forceinline__ void sb_tile_wait(float &a, float &b)
{
    if (&a == &b) asm volatile("s_waitcnt vmcnt(%1) lgkmcnt(0)" : "+v"(a) : "n"(N) : "memory");
    else asm volatile("s_waitcnt vmcnt(%2) lgkmcnt(0)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}

template <int D>
__global__ __launch_bounds__(SB_WAVES * 64) __attribute__((amdgpu_waves_per_eu(4, 4)))
void sparse_batch_kernel(const BatchArgs a)
{
    constexpr int NW = SB_WAVES, TK = SB_TK, NBUF = SB_NBUF;
    constexpr int KS = D / 32;                           // MFMA k-steps of the score product
    constexpr int DT = D / 16;                           // 16-channel tiles of O^T
    constexpr int ROW_BYTES = D * 2, CH = D / 8;
    constexpr int MAT_BYTES = TK * ROW_BYTES;            // one 32-key K (or V) tile
    constexpr int RPI = 1024 / ROW_BYTES;                // rows covered by one wavefront-wide load
    constexpr int MAT_UNITS = MAT_BYTES / 1024;          // wavefront-wide loads per matrix
    constexpr int UPW = 2 * MAT_UNITS / NW;              // ... per wavefront and tile (K and V together)
    constexpr int BUF_BYTES = 2 * MAT_BYTES;             // K tile, then V tile
    static_assert(UPW >= 1 && UPW * NW == 2 * MAT_UNITS, "a tile is a whole number of loads per wavefront");
    static_assert((NBUF - 2) * UPW < 64, "outstanding loads must fit the counter");
    __shared__ __attribute__((aligned(1024))) unsigned char smem[NBUF * BUF_BYTES];
    __shared__ int32_t idx_lds[SB_IDX_TILES * TK];

    // Workgroup id -> (unit, row group): a block of 8 * row_groups consecutive ids (the x dimension) holds 8
    // units; the row groups of a unit are 8 ids apart, i.e. on the same XCD (ids are dealt round-robin to
    // the 8 XCDs) and close in time, so the second reader of a selected row finds it in that XCD's L2.
    const int blk = wg_z() * SB_GRID_Y + wg_y(), within = wg_x();
    const int unit = blk * 8 + (within & 7), rg = within >> 3;
    if (unit >= a.n_units) return;                       // uniform: ids past the last unit of a ragged block
    const int zi = a.Hkv == 1 ? unit : (int)(((unsigned long long)(unsigned)unit * a.inv_Hkv) >> 32);
    const int h = unit - zi * a.Hkv;
    const long long z = zi;
    const int lane = tid_x() & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid_x() >> 6);   // scalar: what depends on it alone stays in scalar registers
    const int l16 = lane & 15, lg4 = lane >> 4;
    const int row0 = rg * SB_ROWS + wave * 16, row = row0 + l16;
    const bool wave_active = row0 < a.R;

    const int nk = a.nk;                                  // selected cache rows
    const int n_keys = nk + a.n_blk;
    const int ntiles = __builtin_amdgcn_readfirstlane((n_keys + TK - 1) / TK);
    const long long stride = (long long)a.Hkv * D;
    const u16 *kc = static_cast<const u16 *>(a.kc) + z * a.seq_kv + (long long)h * D;
    const u16 *vc = static_cast<const u16 *>(a.vc) + z * a.seq_kv + (long long)h * D;
    const u16 *kb = static_cast<const u16 *>(a.kblk) + z * a.seq_blk + (long long)h * D;
    const u16 *vb = static_cast<const u16 *>(a.vblk) + z * a.seq_blk + (long long)h * D;
    const int32_t *idx = a.idx + z * a.seq_idx + (long long)h * nk;

    // index entries of the selected rows at key positions [t0*TK, (t0 + SB_IDX_TILES)*TK) into LDS: at
    // most four per thread, all requested before the first is stored
    int idx_t0 = 0;
    constexpr int PER = SB_IDX_TILES * TK / (NW * 64);
    auto fetch_idx = [&](int t0, int (&e)[PER]) {
        const int first = t0 * TK;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int p = first + i * NW * 64 + (int)tid_x();
            e[i] = p < nk ? idx[p] : 0;
        }
    };
    auto store_idx = [&](const int (&e)[PER]) {
#pragma unroll
        for (int i = 0; i < PER; ++i) idx_lds[i * NW * 64 + tid_x()] = e[i];
    };
    auto load_idx = [&](int t0) {
        int e[PER];
        fetch_idx(t0, e);
        store_idx(e);
    };
    const unsigned idx_addr = lds_addr(idx_lds);
    // This wavefront's share of a tile: load unit u = n*NW + wave of the 2*MAT_UNITS units (K matrix,
    // then V matrix); a unit is 1 KB = RPI rows; lane -> row (lane / CH) of the unit, chunk (lane % CH).
    // Positions past the last key repeat it (their scores are masked).
    const u16 *unit_cache[UPW], *unit_blk[UPW];       // cache / block base pointer of each unit (scalar)
    int unit_row[UPW];                                // tile row this lane fetches in each unit
    unsigned unit_chunk[UPW];                         // its (swizzled) source chunk, in bytes
    const unsigned char *unit_src[UPW];               // cache base + chunk: what a selected row's offset is added to
#pragma unroll
    for (int n = 0; n < UPW; ++n) {
        const int u = n * NW + wave;
        const bool is_v = u >= MAT_UNITS;             // uniform per wavefront
        unit_cache[n] = is_v ? vc : kc;
        unit_blk[n] = is_v ? vb : kb;
        unit_row[n] = (u % MAT_UNITS) * RPI + lane / CH;
        unit_chunk[n] = (unsigned)(((lane % CH) ^ (sb_swz(unit_row[n]) & (CH - 1))) * 16);
        unit_src[n] = reinterpret_cast<const unsigned char *>(unit_cache[n]) + unit_chunk[n];
    }
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds_addr(smem) + wave * 1024);
    const unsigned stride_bytes = (unsigned)stride * 2u;
    // The index entries of a tile's rows are read from LDS one tile ahead of the request (request_entries:
    // no wait), so that a tile's requests go out right after the barrier that frees its buffer.
    float ent[UPW];
    auto request_entries = [&](int t) {
        if ((t + 1) * TK <= nk && t >= idx_t0 && t < idx_t0 + SB_IDX_TILES) {   // uniform; the common case: a tile of selected rows, no clamping
            const unsigned base = idx_addr + (unsigned)((t - idx_t0) * TK) * 4;
#pragma unroll
            for (int n = 0; n < UPW; ++n) ent[n] = lds_read_f32<0>(base + (unsigned)unit_row[n] * 4);
            return;
        }
#pragma unroll
        for (int n = 0; n < UPW; ++n) {
            int p = t * TK + unit_row[n];
            p = (p < nk ? p : nk - 1) - idx_t0 * TK;     // in-block positions read some entry and ignore it
            p = p < 0 ? 0 : (p < SB_IDX_TILES * TK ? p : SB_IDX_TILES * TK - 1);   // (a tile past the window is re-read after the refill)
            ent[n] = lds_read_f32<0>(idx_addr + (unsigned)p * 4);
        }
    };
    // wait for the entries just requested: one wait for all of them, in one place -- the registers an LDS read will
    // write must not be named by any instruction before it (the compiler copies a register it is told an assembly
    // statement modifies when the old value has a second reader, and such a copy would read too early)
    auto await_entries = [&] {
        static_for<UPW>([&](auto NI) { lds_wait<UPW - 1 - decltype(NI)::value>(ent[decltype(NI)::value]); });
    };
    // request tile t's rows; its entries have landed (await_entries, or the wait at the top of a loop iteration)
    auto issue = [&](int t) {
        const unsigned dst = lds_wave + (unsigned)(t % NBUF) * BUF_BYTES;
        if ((t + 1) * TK <= nk) {                        // uniform; nearly every tile: selected rows only, one multiply-add per request
            static_for<UPW>([&](auto NI) {
                constexpr int n = decltype(NI)::value;
                const unsigned long long off = (unsigned long long)(unsigned)__builtin_bit_cast(int, ent[n]) * stride_bytes;
                __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(unit_src[n] + off), MAGE_LDS_ADDR(dst + n * NW * 1024), 16, 0, 0);
            });
            return;
        }
        static_for<UPW>([&](auto NI) {
            constexpr int n = decltype(NI)::value;
            int p = t * TK + unit_row[n];
            p = p < n_keys ? p : n_keys - 1;
            const bool cache = p < nk;
            const unsigned src_row = cache ? (unsigned)__builtin_bit_cast(int, ent[n]) : (unsigned)(p - nk);
            const unsigned long long off = (unsigned long long)src_row * stride_bytes + unit_chunk[n];
            const unsigned char *base = reinterpret_cast<const unsigned char *>(cache ? unit_cache[n] : unit_blk[n]);
            __builtin_amdgcn_global_load_lds(MAGE_GLOBAL_PTR(base + off), MAGE_LDS_ADDR(dst + n * NW * 1024), 16, 0, 0);
        });
    };

    // the index entries are requested first: everything else on the way to the first tile waits for them
    int e0[PER];
    fetch_idx(0, e0);
    // query fragment (B operand): row l16 of this wavefront's 16 rows, channels 32*ks + 8*lg4 .. +7
    bf16x8_t qf[KS];
    {
        const int rq = row < a.R ? row : a.R - 1;         // rows past R re-read the last row and are never stored
        const int gl = a.B == 1 ? rq : (int)(((unsigned long long)(unsigned)rq * a.inv_B) >> 32), qi = rq - gl * a.B;
        const u16 *src = static_cast<const u16 *>(a.q) + z * a.seq_q + ((long long)qi * a.Hq + (long long)h * a.G + gl) * D + 8 * lg4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(src + ks * 32));
    }
    store_idx(e0);
    __syncthreads();
#pragma clang loop unroll(disable)
    for (int j = 0; j < NBUF - 1 && j < ntiles; ++j) {
        request_entries(j);
        await_entries();
        issue(j);
    }
    request_entries(NBUF - 1);

    // Fragment read addresses.  The swizzle, the MFMA k-step (K) and the O^T tile (V) all act on address
    // bits 4..7 only, so each read's address is a lane constant plus the ring slot's offset (one
    // addition per read); the 16-key block is an immediate offset.
    const unsigned smem_addr = lds_addr(smem);
    // K fragment (A operand): key row l16 of a block, channels 32*ks + 8*lg4 .. +7 = chunk 4*ks + lg4
    unsigned kaddr[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        kaddr[ks] = smem_addr + (((unsigned)(l16 * ROW_BYTES) | (unsigned)(((lg4 ^ sb_swz(l16)) & (CH - 1)) << 4)) ^ (unsigned)(ks << 6));
    // V^T fragment: within each 16-lane block, lane i' addresses 4 channels (4*(i' & 3) ..) of key
    // 4*lg4 + (i' >> 2); the transposing read hands lane i channel i of those 4 keys
    const int jj = l16 >> 2, q4 = l16 & 3;
    const int vr = 4 * lg4 + jj;
    unsigned vaddr[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
        vaddr[dt] = smem_addr + (((unsigned)(vr * ROW_BYTES + 8 * (q4 & 1)) | (unsigned)((((q4 >> 1) ^ sb_swz(vr)) & (CH - 1)) << 4)) ^ (unsigned)(dt << 5));

    f32x4_t o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // online softmax against a lazily raised reference: probabilities are taken against m_run, which
    // follows the row maximum only when that has run ahead by more than kLazy (log2 units), so the
    // accumulators are rescaled on few tiles; the reference starts at a finite floor (no inf - inf)
    constexpr float kLazy = 8.f, kFloor = -3.0e38f;
    float m_run = kFloor, l_run = 0.f;                    // l_run: this lane's share (its 8 keys per tile)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qf[ks]));

    // one tile, in ring slot t % NBUF.  The loop over the tiles is NOT unrolled over the ring: the slot is
    // one scalar addition per fragment address, while an unrolled body is four times the instructions
    // to fetch into an instruction cache that starts cold at every launch.
    auto step = [&](int t) {
        constexpr int BLK = 16 * ROW_BYTES;
        const unsigned koff = (unsigned)(t % NBUF) * BUF_BYTES, voff = koff + MAT_BYTES;
        // tile t has landed; NBUF-2 younger tiles may still be in flight; everyone is done with tile t-1
        // (the wait names the entry registers: what reads them below depends on it and cannot be moved above it)
        if (t + NBUF - 2 < ntiles) sb_tile_wait<(NBUF - 2) * UPW>(ent[0], ent[UPW - 1]);
        else sb_tile_wait<0>(ent[0], ent[UPW - 1]);
        __syncthreads();
        // ---- scores: sc[b][v] = S^T(key 16*b + 4*lg4 + v of the tile, query row l16) ----
        // The two key blocks accumulate alternately (two independent chains of MFMAs); the fragments are
        // read in batches of KB k-steps (registers: four wavefronts share a SIMD).  The first batch is
        // requested before the next tile's rows are, so that those requests (all wavefronts issue theirs at
        // the same moment, right after the barrier) are made while the fragments travel.
        constexpr int KB = KS < 2 ? KS : 2;
        u32x4_t kf[KB][2];
        auto read_k = [&](auto BT) {
            constexpr int k0 = decltype(BT)::value * KB;
            static_for<KB>([&](auto S) {
                constexpr int i = decltype(S)::value;
                kf[i][0] = lds_read_b128<0>(kaddr[k0 + i] + koff);
                kf[i][1] = lds_read_b128<BLK>(kaddr[k0 + i] + koff);
            });
        };
        if (wave_active) read_k(std::integral_constant<int, 0>{});
        const int tn = t + NBUF - 1;                      // goes into the slot tile t-1 has just left
        if (tn < ntiles) {
            if (tn + 1 > idx_t0 + SB_IDX_TILES && tn * TK < nk) {                 // uniform; rare (k > 2048)
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                // the fragment reads above read LDS, too
                idx_t0 = tn;
                load_idx(tn);
                __syncthreads();
                request_entries(tn);
                await_entries();
            }
            issue(tn);
            request_entries(tn + 1);                      // lands while this tile is computed; waited for at the next barrier
        }
        if (!wave_active) return;
        const int valid = n_keys - t * TK;                // >= 1
        f32x4_t sc[2] = {f32x4_t{0.f, 0.f, 0.f, 0.f}, f32x4_t{0.f, 0.f, 0.f, 0.f}};
        static_for<KS / KB>([&](auto BT) {
            constexpr int k0 = decltype(BT)::value * KB;
            // (the waits of the first batch count the entry reads behind it as if they were fragments: they only wait longer)
            if constexpr (k0 > 0) read_k(BT);
            static_for<KB>([&](auto S) {
                constexpr int i = decltype(S)::value;
                static_for<2>([&](auto BI) {
                    constexpr int b = decltype(BI)::value;
                    lds_wait<2 * KB - 1 - (2 * i + b)>(kf[i][b]);
                    sc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[i][b]), qf[k0 + i], sc[b], 0, 0, 0);
                });
            });
        });
        // V^T fragments of the first O^T tiles travel while the softmax runs
        constexpr int kPre = DT < 2 ? DT : 2;
        u32x2_t lo[DT], hi[DT];
        static_for<kPre>([&](auto T) {
            constexpr int dt = decltype(T)::value;
            lo[dt] = lds_read_tr16_b64<0>(vaddr[dt] + voff);
            hi[dt] = lds_read_tr16_b64<BLK>(vaddr[dt] + voff);
        });
        if (valid < TK) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (16 * b + 4 * lg4 + v >= valid) sc[b][v] = -INFINITY;
        }
        float mx = fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3]));
        mx = fmaxf(mx, fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
        {   // the other keys of this query row sit in the three other 16-lane rows of the wavefront
            float x0, x1;
            lane_rows16(mx, x0, x1);
            mx = fmaxf(x0, x1);
            lane_halves(mx, x0, x1);
            mx = fmaxf(x0, x1) * a.scale_log2;
        }
        if (__any(mx > m_run + kLazy)) {                  // uniform: some row's maximum has run ahead of its reference
            const float m_new = fmaxf(m_run, mx);
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= corr;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt] *= corr;
        }
        bf16x8_t pf;
        float psum = 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sc[b][v], a.scale_log2, -m_run));
                psum += p;
                pf[4 * b + v] = (__bf16)p;
            }
        l_run += psum;
        // ---- O^T += V^T P^T: 32 keys (both blocks) per MFMA, fragments kPre O^T tiles ahead ----
        static_for<DT>([&](auto T) {
            constexpr int dt = decltype(T)::value;
            constexpr int younger = ((dt + kPre < DT ? dt + kPre : DT) - dt - 1) * 2;
            lds_wait<younger>(lo[dt], hi[dt]);
            const u32x4_t both = {lo[dt][0], lo[dt][1], hi[dt][0], hi[dt][1]};
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, both), pf, o[dt], 0, 0, 0);
            if constexpr (dt + kPre < DT) {
                lo[dt + kPre] = lds_read_tr16_b64<0>(vaddr[dt + kPre] + voff);
                hi[dt + kPre] = lds_read_tr16_b64<BLK>(vaddr[dt + kPre] + voff);
            }
        });
    };
#pragma clang loop unroll(disable)
    for (int t = 0; t < ntiles; ++t) step(t);

    if (!wave_active) return;
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (row >= a.R) return;
    const float inv = 1.f / l_tot;
    const int gl = a.B == 1 ? row : (int)(((unsigned long long)(unsigned)row * a.inv_B) >> 32), qi = row - gl * a.B;
    const long long orow = (long long)qi * a.Hq + (long long)h * a.G + gl;
    float *dst = a.out + z * a.seq_out + orow * D;
    // O^T register (dt, v) holds channel 16*dt + 4*lg4 + v of this lane's query row
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4_t *>(dst + 16 * dt + 4 * lg4) = o[dt] * inv;
    if (a.lse_out && lg4 == 0) a.lse_out[z * a.seq_lse + orow] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
}

// n_seq independent sequences, one workgroup per (sequence, KV head, 128-row group).
hipError_t bf16_sparse_batched(const KernelArgs &k, int d, int row_groups, int n_seq, hipStream_t stream)
{
    const long long n_units = (long long)n_seq * k.Hkv;
    const long long n_blocks = (n_units + 7) / 8;
    // the kernel's 32-bit arithmetic: unit / Hkv and row / B by a multiply-high, ids within the grid's limits
    if (n_seq <= 0 || row_groups <= 0 || k.nc <= 0 || k.nc > 0x7fffffff - k.n_blk || (n_units + 8) * k.Hkv >= (1ll << 32) ||
        (long long)k.R * k.B >= (1ll << 32) || n_blocks > (long long)SB_GRID_Y * 65535 || 8ll * row_groups > 0x7fffffff)
        return hipErrorInvalidValue;
    BatchArgs a{};
    a.q = k.q;
    a.kc = k.kc;
    a.vc = k.vc;
    a.kblk = k.kblk;
    a.vblk = k.vblk;
    a.idx = k.idx;
    a.out = k.out;
    a.lse_out = k.lse_out;
    a.seq_q = k.seq_q;
    a.seq_kv = k.seq_kv;
    a.seq_idx = k.seq_idx;
    a.seq_blk = k.seq_blk;
    a.seq_out = k.seq_out;
    a.seq_lse = k.seq_lse;
    a.B = k.B;
    a.Hq = k.Hq;
    a.Hkv = k.Hkv;
    a.G = k.G;
    a.R = k.R;
    a.nk = (int)k.nc;
    a.n_blk = k.n_blk;
    a.n_units = (int)n_units;
    a.inv_Hkv = k.Hkv >= 2 ? (unsigned)(((1ull << 32) + k.Hkv - 1) / k.Hkv) : 0u;
    a.inv_B = k.B >= 2 ? (unsigned)(((1ull << 32) + k.B - 1) / k.B) : 0u;
    a.scale_log2 = k.scale_log2;
    const unsigned gy = (unsigned)(n_blocks < SB_GRID_Y ? n_blocks : SB_GRID_Y);
    const unsigned gz = (unsigned)((n_blocks + SB_GRID_Y - 1) / SB_GRID_Y);
    dim3 grid(8 * row_groups, gy, gz), block(SB_WAVES * 64);
    if (d == 128) hipLaunchKernelGGL((sparse_batch_kernel<128>), grid, block, 0, stream, a);
    else if (d == 64) hipLaunchKernelGGL((sparse_batch_kernel<64>), grid, block, 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace mage
