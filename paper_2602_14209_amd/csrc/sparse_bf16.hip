// bf16 sparse-step attention for gfx950 -- Alg. 1 Phase 2 "SparseAttn(Q_h,K_h,V_h,C[S])":
// softmax over the k selected cache rows of KV head h plus the block's own B keys.
//
// The step moves a few MB, so it is bound by dependent-load latency and by how many compute
// units take part, not by bandwidth.  Layout of the work, chosen for that:
//   - one workgroup per (KV head, 16 query rows, slice of the output channels); its 8 wavefronts
//     split the KEYS (tiles of 16 key positions, round-robin), so no partial result ever leaves
//     the compute unit: the eight partial (max, sum, O) are merged through LDS and every output
//     element is written once;
//   - every load of a pass is in flight at once: the index entries, then K rows into registers
//     (coalesced 64-byte pieces, moved to their MFMA operand lanes by a lane permute) and V rows
//     straight into LDS (global_load_lds), from where transposing reads (ds_read_b64_tr_b16)
//     deliver V^T fragments;
//   - the step has too little work for 256 compute units if a row tile is one workgroup (64 at
//     Hkv = 8, G*B = 128), and keys cannot be split over workgroups without a merge through memory
//     that costs more than it saves.  The OUTPUT CHANNELS can: up to four workgroups share a row
//     tile, each computes the full scores (the softmax statistics are simply computed four times)
//     but fetches and multiplies only its quarter of every V row.  Measured at Hkv = 8, k = 512:
//     9.5 us with one workgroup per row tile, 8.4 with two, 7.8 with four;
//   - the instruction cache is cold at the start of every launch (straight-line code runs at
//     about 13 cycles per instruction the first time, 3 the second), and nearly all of this kernel
//     runs once.  What sits in front of a load on the chain index entry -> row -> scores is
//     therefore kept short: divisions are done on the host, the index entries are requested
//     before anything else, then the queries, then the address arithmetic that does not depend
//     on them; the first pass over the keys is not the body of a loop (see run_pass);
//   - workgroups of one KV head sit on the same XCD when Hkv is a multiple of 8 (linear
//     workgroup id = head + Hkv * (row tile, channel part)), so a gathered row is fetched from HBM
//     once and shared through that XCD's L2.
// Key positions form one sequence: 0..k-1 are cache rows idx[h,p], k..k+B-1 the in-block rows.
// v_mfma_f32_16x16x32_bf16 throughout; scores are produced transposed (S^T = K Q^T) so that a
// lane holds scores of one query row and P^T is already the B operand of O^T = V^T P^T.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lds_asm.hpp"
#include "ids.hpp"
#include "plan.hpp"

namespace mage {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short u16;

constexpr int SP_WAVES = 8;
constexpr int SP_KT = 16;          // key positions per tile
constexpr int SP_TPW = 5;          // tiles per wavefront per pass (register arrays)
constexpr int SP_MAXT = SP_WAVES * SP_TPW;   // tiles per pass: all of LDS holds V (640 key positions at d=128)

// The compiler may not read, copy or move these registers across this point (they are the
// destinations of loads it does not know about).
__device__ __forceinline__ void hold_reg(u32x4_t &r) { asm volatile("" : "+v"(r)); }
__device__ __forceinline__ void hold_int(int &r) { asm volatile("" : "+v"(r)); }
__device__ __forceinline__ int global_load_b32(const void *p)      // a load the compiler keeps no books on (see lds_asm.hpp)
{
    int r;
    asm volatile("global_load_dword %0, %1, off" : "=&v"(r) : "v"(p));
    return r;
}
template <int N>
__device__ __forceinline__ void hold_regs(u32x4_t (&r)[N])
{
    static_for<N>([&](auto I) { hold_reg(r[decltype(I)::value]); });
}

// chunk swizzle of a 16-row V tile: rows 0..7 (one half of a transposing read) spread over all banks
__device__ __forceinline__ int sp_swz(int r) { return ((r & 7) << 1) | (r >> 3); }

// The kernel's own argument block: one launch is so short that the instructions in front of the first
// load are a visible part of it, so everything that needs a division is worked out on the host.
struct SparseArgs {
    const void *q, *kc, *vc, *kblk, *vblk;
    const int32_t *idx;          // [Hkv][nc] (unused when COMPACT)
    float *out, *lse_out;
    int B, Hq, Hkv, G, R;
    int nc, n_blk;               // cache key positions (k) and in-block keys
    int ntiles, npass, tpp;      // tiles of SP_KT key positions, passes over the LDS window, tiles per pass (balanced)
    unsigned inv_B;              // ceil(2^32 / B) for B >= 2: row / B == mulhi(row, inv_B) while row * B < 2^32
    float scale_log2;
};

// COMPACT: the k cache positions are rows 0..k-1 of a compacted cache (no index set to read).
// DS: the output channels of a row tile are dealt to DS workgroups.  Each of them computes the
// full scores (every K row, all D channels) but fetches and multiplies only its D/DS channels of
// V: no result crosses workgroups, the softmax statistics are simply computed DS times, and a
// compute unit has 1/DS of the V bytes to pull through its memory path.
template <int D, int DS, bool COMPACT>
__global__ __launch_bounds__(SP_WAVES * 64) __attribute__((amdgpu_waves_per_eu(2))) void sparse_bf16_kernel(const SparseArgs a)
{
    constexpr int KS = D / 32;                  // MFMA k-steps of the score product
    constexpr int DV = D / DS;                  // V channels (and output channels) of this workgroup
    constexpr int DT = DV / 16;                 // 16-channel tiles of O^T
    constexpr int CH = DV / 8;                  // 16-byte chunks per V row slice
    constexpr int ROW_BYTES = DV * 2;           // V row slice in LDS
    constexpr int TILE_BYTES = SP_KT * ROW_BYTES;
    constexpr int VLOADS = TILE_BYTES / 1024;   // wavefront-wide 1 KB loads per V tile
    constexpr int RPL = 1024 / ROW_BYTES;       // rows per such load
    static_assert(DV % 32 == 0 && VLOADS >= 1, "a V tile is at least one wavefront-wide load");

    // V tiles: slot j*8 + wave belongs to this wavefront alone (distinct compile-time offsets, so
    // the compiler sees that the direct loads never overlap).  After the key loop the same memory
    // holds the eight partial results and their (max, sum) pairs.
    __shared__ __attribute__((aligned(1024))) unsigned char vlds[SP_MAXT * TILE_BYTES];
    constexpr int PART_BYTES = SP_WAVES * DT * 64 * 16;
    static_assert(PART_BYTES + 2 * SP_WAVES * 16 * 4 <= SP_MAXT * TILE_BYTES, "merge buffers must fit in the V tiles");
    float (*ml)[SP_WAVES][16] = reinterpret_cast<float (*)[SP_WAVES][16]>(vlds + PART_BYTES);

    const int h = wg_x(), rt = wg_y() / DS, dpart = wg_y() % DS;
    const int lane = tid_x() & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid_x() >> 6);     // uniform: tile bookkeeping stays on the scalar unit
    const int l16 = lane & 15, lg4 = lane >> 4;
    const int row = rt * 16 + l16;

    const int n_keys = a.nc + a.n_blk;
    const int ntiles = a.ntiles, npass = a.npass, tpp = a.tpp;

    const int32_t *idx = COMPACT ? nullptr : a.idx + (long long)h * a.nc;

    // row of q, out and lse that this lane's query row is (rows past R stand in for the last row and are never stored)
    auto io_row = [&]() {
        const int rq = row < a.R ? row : a.R - 1;
        const int gl = a.B == 1 ? rq : (int)(((unsigned long long)(unsigned)rq * a.inv_B) >> 32), qi = rq - gl * a.B;
        return qi * a.Hq + h * a.G + gl;
    };
    // query fragment: row l16 of this row tile, channels 32*ks + 8*lg4 .. +7; requested in the first pass, right
    // after the index entries
    u32x4_t qraw[KS];

    f32x4_t o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;       // l_run: this lane's share (its 4 keys per tile)

    // One pass over (up to) SP_MAXT tiles.  A function object called for pass 0 on its own: written as the body of a
    // loop, everything in it that does not depend on the pass would be computed in front of the loop, i.e. in front
    // of the index requests.
    auto run_pass = [&](int pass) {
        const int t0 = pass * tpp;
        const int t1 = t0 + tpp < ntiles ? t0 + tpp : ntiles;
        const int first = t0 + wave;                        // this wavefront's tiles: first + 8*j
        if (first >= t1) return;                            // nothing for this wavefront in this pass
        const int my_tiles = (t1 - first + SP_WAVES - 1) / SP_WAVES;

        // ---- issue every load of the pass, branch-free (a branch would make the compiler wait
        // for all outstanding loads at its join).  A tile slot j >= my_tiles repeats the last
        // real tile's rows into its own (unused) LDS slot; its scores are masked below. ----
        // src_row(tile row): source of key position tile*16 + row (cache row >= 0, block row r as
        // -1-r).  Every lane reads the index entries of exactly the rows it will fetch -- row
        // (lane / 4) for its K pieces, rows n*RPL + lane / CH for its V loads -- with all those small
        // loads in flight at once; they hit the same few cache lines.
        // The entries are assembly loads too, issued back to back: left to the compiler, each load sinks below the
        // test "is this position a cache row?" and ends up behind a branch of its own.
        constexpr bool V_AS_K = RPL == SP_KT && CH == 4;    // a 64-byte V slice is fetched by the lane quad that fetches the K row
        int tile_of[SP_TPW], ek[SP_TPW], ev[SP_TPW][VLOADS], pk[SP_TPW], posv[SP_TPW][VLOADS];
        auto key_pos = [&](int tile, int r) {
            const int p = tile * SP_KT + r;
            return p < n_keys ? p : n_keys - 1;             // padding positions re-read the last key (masked below)
        };
        auto request = [&](int p) { return COMPACT ? p : global_load_b32(idx + (p < a.nc ? p : a.nc - 1)); };
        auto resolve = [&](int p, int entry) { return p < a.nc ? entry : -1 - (p - a.nc); };
#pragma unroll
        for (int j = 0; j < SP_TPW; ++j) {
            tile_of[j] = first + SP_WAVES * (j < my_tiles ? j : my_tiles - 1);
            pk[j] = key_pos(tile_of[j], lane >> 2);
            ek[j] = request(pk[j]);
#pragma unroll
            for (int n = 0; n < VLOADS; ++n) {
                posv[j][n] = key_pos(tile_of[j], n * RPL + lane / CH);
                ev[j][n] = V_AS_K ? 0 : request(posv[j][n]);
            }
        }
        // K fragments.  The MFMA wants lane (16*c + r) to hold channels [32*ks + 8*c, +8) of tile row r,
        // but a load in that pattern touches 64 separate 16-byte pieces per instruction.  Load
        // coalesced instead -- lane 4*r + c fetches that same piece, so each lane quad reads 64
        // contiguous bytes of one row -- and move the pieces to their MFMA lanes with a lane permute.
        // The loads are inline assembly so that the waits can be ours: behind the conditional last
        // slot the compiler's own bookkeeping would wait for every outstanding load, V included.
        u32x4_t kraw[SP_TPW][KS];
        __builtin_amdgcn_sched_barrier(0);     // every index entry is requested before anything else: the entries head the
                                               // longest dependent chain of the launch (entry -> row -> scores), and the code
                                               // in front of them is fetched from a cold instruction cache
        const unsigned stride_bytes = (unsigned)a.Hkv * (D * 2);       // bytes from a cache row to the next
        const u16 *kc = static_cast<const u16 *>(a.kc) + h * D;
        const u16 *vc = static_cast<const u16 *>(a.vc) + h * D + dpart * DV;
        const u16 *kb = static_cast<const u16 *>(a.kblk) + h * D;
        const u16 *vb = static_cast<const u16 *>(a.vblk) + h * D + dpart * DV;
        if (pass == 0) {
            // The queries: assembly loads like the K rows (the compiler must not count them: its wait for them would
            // sit in front of the first MFMA and take most of the K and V loads with it).  They are older than every
            // K row, so they have landed when the first K tile has.
            const u16 *src = static_cast<const u16 *>(a.q) + (long long)io_row() * D + 8 * lg4;
            static_for<KS>([&](auto S) {
                constexpr int ks = decltype(S)::value;
                qraw[ks] = global_load_b128<ks * 64>(src);
            });
        }
        // the index entries have landed once nothing but the query loads of the first pass is outstanding
        if (pass == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(KS) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < SP_TPW; ++j) {
            hold_int(ek[j]);
            ek[j] = resolve(pk[j], ek[j]);
#pragma unroll
            for (int n = 0; n < VLOADS; ++n) {
                if (!V_AS_K) hold_int(ev[j][n]);
                ev[j][n] = V_AS_K ? ek[j] : resolve(posv[j][n], ev[j][n]);
            }
        }
        // address of a key row: one 32 x 32 -> 64 bit multiply-add (row and row pitch are both below 2^32)
        auto row_ptr = [&](const u16 *cache, const u16 *blk, int e) {
            const unsigned r = e >= 0 ? (unsigned)e : (unsigned)(-1 - e);
            return reinterpret_cast<const unsigned char *>(e >= 0 ? cache : blk) + (unsigned long long)r * stride_bytes;
        };
        auto load_k = [&](int j) {
            const unsigned char *src = row_ptr(kc, kb, ek[j]) + 16 * (lane & 3);
            static_for<KS>([&](auto S) {
                constexpr int ks = decltype(S)::value;
                kraw[j][ks] = global_load_b128<ks * 64>(src);
            });
            __builtin_amdgcn_sched_barrier(0);     // the next tile's address arithmetic stays behind these loads
        };
        auto load_v = [&](int j) {
            unsigned char *dst = vlds + (j * SP_WAVES + wave) * TILE_BYTES;
#pragma unroll
            for (int n = 0; n < VLOADS; ++n) {
                const int r = n * RPL + lane / CH;                           // tile row this lane fetches
                const int e = ev[j][n];
                const unsigned char *src = row_ptr(vc, vb, e);
                const int chunk = (lane % CH) ^ (sp_swz(r) & (CH - 1));
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + chunk * 16),
                                                 (__attribute__((address_space(3))) void *)(dst + n * 1024), 16, 0, 0);
            }
        };
        // the first SP_TPW-1 tile slots unconditionally; the last slot is filled for few wavefronts
        // only, so it sits behind a branch (nothing right after the branches depends on a pending load)
        // (all K before any V, so that the scores can start while V is still arriving)
#pragma unroll
        for (int j = 0; j < SP_TPW - 1; ++j) load_k(j);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kraw[SP_TPW - 1][ks] = u32x4_t{0u, 0u, 0u, 0u};
        if (my_tiles == SP_TPW) load_k(SP_TPW - 1);
#pragma unroll
        for (int j = 0; j < SP_TPW - 1; ++j) load_v(j);
        if (my_tiles == SP_TPW) load_v(SP_TPW - 1);

        __builtin_amdgcn_sched_barrier(0);     // keep every load ahead of the first MFMA (and its wait)
        // K tile j has landed when at most this many younger loads are outstanding.  The counts assume
        // that the conditional last slot was not issued; with it they only wait a little longer.
        bf16x8_t kf[SP_TPW][KS];
        {
            const int from = 4 * (4 * l16 + lg4);            // byte address of the source lane for ds_bpermute
            static_for<SP_TPW>([&](auto J) {
                constexpr int j = decltype(J)::value;
                constexpr int younger = (j < SP_TPW - 1 ? (SP_TPW - 2 - j) * KS : 0) + (SP_TPW - 1) * VLOADS;
                static_for<KS>([&](auto S) {
                    constexpr int ks = decltype(S)::value;
                    vm_wait<younger + (j < SP_TPW - 1 ? KS - 1 - ks : 0)>(kraw[j][ks]);
                    if constexpr (j == 0 && ks == 0)      // the queries are older than this K piece: landed, and not to be touched before here
                        hold_regs(qraw);
                    u32x4_t t;
                    t.x = __builtin_amdgcn_ds_bpermute(from, kraw[j][ks].x);
                    t.y = __builtin_amdgcn_ds_bpermute(from, kraw[j][ks].y);
                    t.z = __builtin_amdgcn_ds_bpermute(from, kraw[j][ks].z);
                    t.w = __builtin_amdgcn_ds_bpermute(from, kraw[j][ks].w);
                    kf[j][ks] = __builtin_bit_cast(bf16x8_t, t);
                });
            });
        }
        // ---- scores: sc[j][v] = S^T(key 4*lg4 + v of tile j, query row l16) ----
        f32x4_t sc[SP_TPW];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < SP_TPW; ++j) {
            sc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                sc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[j][ks], __builtin_bit_cast(bf16x8_t, qraw[ks]), sc[j], 0, 0, 0);
            const int p0 = tile_of[j] * SP_KT + 4 * lg4;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (j >= my_tiles || p0 + v >= n_keys) sc[j][v] = -INFINITY;
                mx = fmaxf(mx, sc[j][v]);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32)) * a.scale_log2;
        const float m_new = fmaxf(m_run, mx);
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < SP_TPW; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sc[j][v], a.scale_log2, -m_new));
                sc[j][v] = p;
                psum += p;
            }
        l_run = l_run * corr + psum;
        if (pass > 0) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt] *= corr;
        }

        // ---- O^T += V^T P^T, 32 key positions (two tiles) per MFMA ----
        // V tiles are consumed as they land: before the MFMAs of tiles 2s and 2s+1 the wavefront
        // waits only until its direct loads of those tiles are done (loads retire in issue order).
        // V^T fragments by transposing LDS reads (inline assembly, see lds_asm.hpp), kPre O^T tiles
        // ahead of the MFMA that consumes them.  The swizzle and the O^T tile both act on address
        // bits 4..7 only: address = (lane constant + compile-time slot offset) ^ (dt << 5).
        const int jj = l16 >> 2, q = l16 & 3;
        const int vr = 4 * lg4 + jj;                          // tile row this lane addresses in a transposing read
        const unsigned vbase = (lds_addr(vlds) + wave * TILE_BYTES + vr * ROW_BYTES + 8 * (q & 1)) |
                               ((((q >> 1) ^ sp_swz(vr)) & (CH - 1)) << 4);
        constexpr int kPre = DT < 4 ? DT : 4;
        auto pv = [&](auto SLOTS) {     // SLOTS: tile slots this wavefront issued V loads for
          constexpr int issued = decltype(SLOTS)::value * VLOADS;
          static_for<(SP_TPW + 1) / 2>([&](auto SI) {
            constexpr int s = decltype(SI)::value;
            if (2 * s < my_tiles) {   // uniform
                constexpr int need = (2 * s + 2) * VLOADS < issued ? (2 * s + 2) * VLOADS : issued;
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(issued - need) : "memory");
                bf16x8_t pf;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    pf[e] = (__bf16)sc[2 * s][e];
                    pf[4 + e] = (2 * s + 1 < SP_TPW) ? (__bf16)sc[2 * s + 1 < SP_TPW ? 2 * s + 1 : 0][e] : (__bf16)0.f;
                }
                // a missing second tile contributes zeros through P; its slot repeats a real tile
                constexpr int ja = 2 * s, jb = (2 * s + 1 < SP_TPW) ? 2 * s + 1 : 2 * s;
                constexpr int offa = ja * SP_WAVES * TILE_BYTES, offb = jb * SP_WAVES * TILE_BYTES;
                u32x2_t lo[DT], hi[DT];
                static_for<kPre>([&](auto T) {
                    constexpr int dt = decltype(T)::value;
                    lo[dt] = lds_read_tr16_b64<0>((vbase + offa) ^ (unsigned)(dt << 5));
                    hi[dt] = lds_read_tr16_b64<0>((vbase + offb) ^ (unsigned)(dt << 5));
                });
                static_for<DT>([&](auto T) {
                    constexpr int dt = decltype(T)::value;
                    // younger reads outstanding behind this pair: the pairs dt+1 .. min(dt+kPre, DT)-1
                    constexpr int younger = ((dt + kPre < DT ? dt + kPre : DT) - dt - 1) * 2;
                    lds_wait<younger>(lo[dt], hi[dt]);
                    const u32x4_t both = {lo[dt][0], lo[dt][1], hi[dt][0], hi[dt][1]};
                    o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, both), pf, o[dt], 0, 0, 0);
                    if constexpr (dt + kPre < DT) {
                        lo[dt + kPre] = lds_read_tr16_b64<0>((vbase + offa) ^ (unsigned)((dt + kPre) << 5));
                        hi[dt + kPre] = lds_read_tr16_b64<0>((vbase + offb) ^ (unsigned)((dt + kPre) << 5));
                    }
                });
            }
          });
        };
        pv(std::integral_constant<int, SP_TPW - 1>{});       // counts without the conditional last slot: never too lax
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // slots past this wavefront's last tile were loaded too
    };
    run_pass(0);
    for (int pass = 1; pass < npass; ++pass) run_pass(pass);

    // ---- merge the eight wavefronts through LDS ----
    float l_w = l_run + __shfl_xor(l_run, 16);
    l_w += __shfl_xor(l_w, 32);
    __syncthreads();                                         // every wavefront is done reading V
    if (lg4 == 0) {
        ml[0][wave][l16] = m_run;
        ml[1][wave][l16] = l_w;
    }
    f32x4_t *part = reinterpret_cast<f32x4_t *>(vlds);     // [wave][dt][lane]
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) part[(wave * DT + dt) * 64 + lane] = o[dt];
    __syncthreads();

    float M = ml[0][0][l16];
#pragma unroll
    for (int w = 1; w < SP_WAVES; ++w) M = fmaxf(M, ml[0][w][l16]);
    float wgt[SP_WAVES], lt = 0.f;
#pragma unroll
    for (int w = 0; w < SP_WAVES; ++w) {
        wgt[w] = __builtin_amdgcn_exp2f(ml[0][w][l16] - M);
        lt = fmaf(wgt[w], ml[1][w][l16], lt);
    }
    if (row >= a.R) return;
    const int orow = io_row();
    float *out = a.out;
    const float inv = 1.f / lt;
    for (int dt = wave; dt < DT; dt += SP_WAVES) {
        f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < SP_WAVES; ++w) acc += part[(w * DT + dt) * 64 + lane] * wgt[w];
        *reinterpret_cast<f32x4_t *>(out + (long long)orow * D + dpart * DV + 16 * dt + 4 * lg4) = acc * inv;
    }
    if (a.lse_out && dpart == 0 && wave == 0 && lg4 == 0) a.lse_out[orow] = (M + log2f(lt)) * 0.6931471805599453f;
}

// Copies the selected rows into a cache of length k: dst[p,h,:] = src[idx[h,p],h,:] (16 bytes per
// thread, a row per D/8 consecutive threads).  The index set is fixed for steps 2..T, so this is
// done once per block.
template <int ESZ>
__global__ __launch_bounds__(256) void compact_kernel(const unsigned char *__restrict__ k_src, const unsigned char *__restrict__ v_src,
                                                      const int32_t *__restrict__ idx, unsigned char *__restrict__ k_dst,
                                                      unsigned char *__restrict__ v_dst, int Hkv, int d, int k)
{
    const int cpr = d * ESZ / 16;                                // 16-byte chunks per row
    const long long t = (long long)wg_x() * 256 + tid_x();
    const long long rowid = t / cpr;                             // (p, h)
    const int c = (int)(t % cpr);
    if (rowid >= (long long)k * Hkv) return;
    const int p = (int)(rowid / Hkv), h = (int)(rowid % Hkv);
    const long long src = ((long long)idx[(long long)h * k + p] * Hkv + h) * d * ESZ + c * 16;
    const long long dst = rowid * d * ESZ + c * 16;
    *reinterpret_cast<uint4 *>(k_dst + dst) = *reinterpret_cast<const uint4 *>(k_src + src);
    *reinterpret_cast<uint4 *>(v_dst + dst) = *reinterpret_cast<const uint4 *>(v_src + src);
}

hipError_t launch_compact(const void *k_src, const void *v_src, const int32_t *idx, void *k_dst, void *v_dst,
                          int Hkv, int d, int k, int esz, hipStream_t stream)
{
    const long long threads = (long long)k * Hkv * (d * esz / 16);
    dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    if (esz == 2)
        hipLaunchKernelGGL(compact_kernel<2>, grid, block, 0, stream, (const unsigned char *)k_src, (const unsigned char *)v_src, idx,
                           (unsigned char *)k_dst, (unsigned char *)v_dst, Hkv, d, k);
    else
        hipLaunchKernelGGL(compact_kernel<4>, grid, block, 0, stream, (const unsigned char *)k_src, (const unsigned char *)v_src, idx,
                           (unsigned char *)k_dst, (unsigned char *)v_dst, Hkv, d, k);
    return hipGetLastError();
}

template <int D, int DS>
static hipError_t launch_sparse(const SparseArgs &a, bool compact, hipStream_t stream)
{
    dim3 grid(a.Hkv, ((a.R + 15) / 16) * DS), block(SP_WAVES * 64);
    if (compact) hipLaunchKernelGGL((sparse_bf16_kernel<D, DS, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((sparse_bf16_kernel<D, DS, false>), grid, block, 0, stream, a);
    return hipGetLastError();
}

// The output channels are split over as many workgroups (1, 2 or 4 per row tile) as still leaves
// every workgroup a compute unit of its own.
hipError_t bf16_sparse(const KernelArgs &k, int d, bool compact, hipStream_t stream)
{
    if (k.nc <= 0 || k.nc > 0x7fffffff - k.n_blk || k.R <= 0 || (long long)k.R * k.B >= (1ll << 32) ||
        (long long)k.Hkv * d * 2 >= (1ll << 31))
        return hipErrorInvalidValue;
    SparseArgs a{};
    a.q = k.q; a.kc = k.kc; a.vc = k.vc; a.kblk = k.kblk; a.vblk = k.vblk; a.idx = k.idx;
    a.out = k.out; a.lse_out = k.lse_out;
    a.B = k.B; a.Hq = k.Hq; a.Hkv = k.Hkv; a.G = k.G; a.R = k.R;
    a.nc = (int)k.nc; a.n_blk = k.n_blk;
    a.ntiles = (a.nc + a.n_blk + SP_KT - 1) / SP_KT;
    a.npass = (a.ntiles + SP_MAXT - 1) / SP_MAXT;
    a.tpp = (a.ntiles + a.npass - 1) / a.npass;
    a.inv_B = k.B >= 2 ? (unsigned)(((1ull << 32) + k.B - 1) / k.B) : 0u;
    a.scale_log2 = k.scale_log2;
    const long long wgs = (long long)a.Hkv * ((a.R + 15) / 16);
    const int ds = 4 * wgs <= kBf16Workgroups ? 4 : 2 * wgs <= kBf16Workgroups ? 2 : 1;
    if (d == 128) {
        if (ds == 4) return launch_sparse<128, 4>(a, compact, stream);
        if (ds == 2) return launch_sparse<128, 2>(a, compact, stream);
        return launch_sparse<128, 1>(a, compact, stream);
    }
    if (d == 64) {
        if (ds >= 2) return launch_sparse<64, 2>(a, compact, stream);
        return launch_sparse<64, 1>(a, compact, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace mage
