// Exact per-KV-head top-k of alpha[h, 0..L) for gfx950 (Alg. 1 "S <- Top-k(alpha)", Eq. 5):
// the k positions with the largest fp32 value, equal values to the smaller index, indices
// emitted in ascending order.  alpha >= 0, so the order of the fp32 bit patterns as unsigned
// integers is the order of the values.
//
// One workgroup of 1024 threads per KV head.  Two routes, chosen per head at run time:
//   filter route (k small against L, the method's regime): the k-th largest of the maxima of
//     disjoint groups of elements is a lower bound of the k-th largest element, so only the few
//     elements at or above it can belong to the set; a radix select over those candidates in LDS
//     finds the k-th value and the ties to keep, and a bitmap walk emits the positions in order.
//     The whole route is one chain of short dependent phases on a single workgroup, so its time is
//     the sum of their latencies: every radix step has its own pre-zeroed histogram and two
//     barriers, prefix sums inside a wavefront use lane-shift moves, and wavefront-uniform values
//     travel through scalar registers rather than the LDS crossbar.
//     The group maxima either come with the row (the column-sum pass leaves one per kGroupKeys
//     consecutive keys; only the groups at or above the bound are then read at all) or are
//     taken here over 8192 strided groups in a first sweep of the row.
//   radix route (any k, any tie structure; also the overflow exit of the filter route): three
//     MSB-first radix-select steps over the whole row find the k-th value and the number of
//     ties to keep, then an ordered sweep emits the set.
// Near-ties at rank k (filter route): alpha is an fp32 result whose relative error (a few 1e-6 from the
// fp32 dot products, exponentials and sums) is of the order of typical gaps between neighbouring values
// at rank k, so the fp32 ranking can differ from the ranking of the exactly computed averages.  The
// candidates within `eps` (relative) of the k-th value -- usually none, a handful at most -- are therefore
// scored again from the inputs in fp64 (exact dot products, fp64 exponentials, the row normalisers
// merged in fp64 from the per-split statistics), rounded to fp32 once, and ranked among themselves by
// (value, smaller index first); as many of them enter the set as the fp32 ranking had admitted.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ids.hpp"
#include "plan.hpp"

namespace mage {

constexpr int TK_THREADS = 1024;
constexpr int TK_WAVES = TK_THREADS / 64;
constexpr int TK_BINS = 4096;                        // widest digit: 12 bits
constexpr int TK_EPT = 16;                           // consecutive elements per thread in the ordered sweep
constexpr int TK_SLOTS = 8;                          // group maxima per thread = loads in flight per thread
constexpr int TK_GROUPS = TK_THREADS * TK_SLOTS;     // 8192
constexpr int TK_CAND = 4096;                        // candidate capacity of the filter route
constexpr int TK_FILTER_MAX_K = 2048;
constexpr int TK_NEAR_MAX = 32;                      // candidates re-scored at most; more of them (massive ties) keep the fp32 ranking

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive moves
// (row shifts inside rows of 16 lanes, then the row broadcasts of the gfx9 family): eight
// vector-ALU instructions instead of six trips through the LDS crossbar.
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t x)
{
    constexpr int ROW_SHR = 0x110, ROW_BCAST15 = 0x142, ROW_BCAST31 = 0x143;
    uint32_t v = x;
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, ROW_SHR + 1, 0xf, 0xf, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, ROW_SHR + 2, 0xf, 0xf, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, ROW_SHR + 3, 0xf, 0xf, true);      // x[l-3..l] inside the row
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ROW_SHR + 4, 0xf, 0xe, true);      // lanes 4..15 of a row: 8 terms
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ROW_SHR + 8, 0xf, 0xc, true);      // lanes 8..15: the whole row prefix
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ROW_BCAST15, 0xa, 0xf, true);      // rows 1 and 3 take the row before
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ROW_BCAST31, 0xc, 0xf, true);      // rows 2 and 3 take lane 31
    return v;
}

// value of a wavefront-uniform lane
__device__ __forceinline__ uint32_t lane_value(uint32_t v, int lane_uniform)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, __builtin_amdgcn_readfirstlane(lane_uniform));
}

// inclusive scan of one value per thread over the workgroup; returns this thread's inclusive
// prefix and the workgroup total.  `tmp` holds TK_WAVES entries.  Every wavefront adds up the
// per-wavefront totals itself (TK_WAVES <= 64 lanes), so nothing runs on a single thread.
__device__ __forceinline__ uint32_t block_scan_incl(uint32_t v, uint32_t *tmp, uint32_t &total)
{
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
    const uint32_t x = wave_scan_incl(v);
    __syncthreads();                      // tmp may still be read from a previous call
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
    const uint32_t w = lane < TK_WAVES ? tmp[lane] : 0u;
    const uint32_t wi = wave_scan_incl(w);
    total = lane_value(wi, TK_WAVES - 1);
    return x + lane_value(wi - w, wave);
}

// Radix step over elements held in LDS or global memory, for a histogram that is already zero
// and used once: histogram the BITS-wide digit at `shift` of every element whose higher bits
// equal `prefix` (bin = number of larger digits, so bins run from the top digit downwards),
// then find the digit in which the `want`-th largest element falls.  Two barriers: after the
// histogram, and after every wavefront has published the running sums of its threads' bins;
// from those every wavefront works out the answer itself.  On return prefix has the digit
// appended, want is the rank inside the digit's bucket and bucket its size.
// Requires: at least `want` elements match the prefix.
template <int BITS>
__device__ __forceinline__ void radix_count(uint32_t x, bool in, int shift, uint32_t prefix, uint32_t *hist)
{
    constexpr int NB = 1 << BITS;
    const uint32_t hi_mask = (shift + BITS >= 32) ? 0u : (0xffffffffu << (shift + BITS));
    if (in && (x & hi_mask) == prefix) atomicAdd(&hist[NB - 1 - ((x >> shift) & (NB - 1))], 1u);
}

// UNR: independent loads in flight per thread (8 for rows in global memory; 1 for the few
// candidates in LDS, where the instructions of the unused slots would cost more than the latency)
template <int BITS, int UNR = 8>
__device__ __forceinline__ void radix_hist_mem(const uint32_t *u, long long n, int shift, uint32_t prefix, uint32_t *hist)
{
    for (long long j0 = tid_x(); j0 < n; j0 += (long long)TK_THREADS * UNR) {
        uint32_t x[UNR];
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const long long j = j0 + (long long)i * TK_THREADS;
            x[i] = j < n ? u[j] : 0xffffffffu;
        }
#pragma unroll
        for (int i = 0; i < UNR; ++i) radix_count<BITS>(x[i], j0 + (long long)i * TK_THREADS < n, shift, prefix, hist);
    }
}

// the same over TK_SLOTS elements per thread that already sit in registers
// `live` slots only: the slots past the end of a short row hold zeros, and thousands of them would all
// be added, one after the other, to the single bin of the value zero; padding(...) accounts for them with
// one addition.
template <int BITS>
__device__ __forceinline__ void radix_hist_regs(const uint32_t (&x)[TK_SLOTS], int live, int shift, uint32_t prefix, uint32_t *hist)
{
#pragma unroll
    for (int i = 0; i < TK_SLOTS; ++i) radix_count<BITS>(x[i], i < live, shift, prefix, hist);
}

// n_pad elements of value zero, counted by one thread (they match a prefix of zero only)
template <int BITS>
__device__ __forceinline__ void radix_hist_padding(uint32_t n_pad, uint32_t prefix, uint32_t *hist)
{
    if (tid_x() == 0 && n_pad != 0 && prefix == 0) atomicAdd(&hist[(1 << BITS) - 1], n_pad);
}

template <int BITS>
__device__ __forceinline__ void radix_pick(int shift, uint32_t &prefix, uint32_t &want, uint32_t &bucket,
                                           const uint32_t *hist, uint32_t *lscan, uint32_t *wtot)
{
    constexpr int NB = 1 << BITS;
    constexpr int PER = NB > TK_THREADS ? NB / TK_THREADS : 1;       // bins per thread
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
    __syncthreads();
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int b = tid_x() * PER + i;
        mine += b < NB ? hist[b] : 0u;
    }
    const uint32_t incl = wave_scan_incl(mine);
    lscan[tid_x()] = incl;
    if (lane == 63) wtot[wave] = incl;
    __syncthreads();
    // the wavefront, then the thread, in whose bins the running count reaches `want`
    const uint32_t w = lane < TK_WAVES ? wtot[lane] : 0u;
    const uint32_t wi = wave_scan_incl(w);
    const unsigned long long wmask = __ballot(lane < TK_WAVES && wi >= want);
    const int wsel = wmask ? __ffsll((long long)wmask) - 1 : TK_WAVES - 1;      // (never empty when the requirement holds)
    const uint32_t wbase = lane_value(wi - w, wsel);                       // elements in the wavefronts before it
    const uint32_t v = lscan[wsel * 64 + lane];
    const unsigned long long lmask = __ballot(wbase + v >= want);
    const int lsel = lmask ? __ffsll((long long)lmask) - 1 : 63;
    const int tsel = wsel * 64 + lsel;
    uint32_t run = wbase + (lsel > 0 ? lane_value(v, lsel > 0 ? lsel - 1 : 0) : 0u);   // elements in the bins before that thread's
    uint32_t digit_bin = (uint32_t)(tsel * PER), cnt = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int b = tsel * PER + i;
        const uint32_t c = b < NB ? hist[b] : 0u;
        if (cnt == 0) {
            if (run < want && want <= run + c) {
                digit_bin = (uint32_t)b;
                cnt = c;
            } else {
                run += c;
            }
        }
    }
    prefix |= (uint32_t)(NB - 1 - digit_bin) << shift;
    want -= run;
    bucket = cnt;
}

template <int BITS>
__device__ __forceinline__ void radix_step_once(const uint32_t *u, uint32_t n, int shift, uint32_t &prefix, uint32_t &want,
                                                uint32_t &bucket, uint32_t *hist, uint32_t *lscan, uint32_t *wtot)
{
    for (uint32_t j = tid_x(); j < n; j += TK_THREADS) radix_count<BITS>(u[j], true, shift, prefix, hist);
    radix_pick<BITS>(shift, prefix, want, bucket, hist, lscan, wtot);
}

// One radix step over n elements of u (global or LDS): histogram the `bits`-wide digit at
// `shift` of every element whose higher bits equal `prefix`, then pick the digit in which the
// `want`-th largest element falls.  On return prefix has that digit appended and want is the
// rank inside the digit's bucket.
__device__ __forceinline__ void radix_step(const uint32_t *u, long long n, int shift, int bits,
                                           uint32_t &prefix, uint32_t &want,
                                           uint32_t *hist, uint32_t *tmp, uint32_t *bcast)
{
    const int nb = 1 << bits;
    const uint32_t hi_mask = (shift + bits >= 32) ? 0u : (0xffffffffu << (shift + bits));
    for (int b = tid_x(); b < nb; b += TK_THREADS) hist[b] = 0;
    __syncthreads();
    constexpr int UNR = 8;      // independent loads in flight per thread
    for (long long j0 = tid_x(); j0 < n; j0 += (long long)TK_THREADS * UNR) {
        uint32_t x[UNR];
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const long long j = j0 + (long long)i * TK_THREADS;
            x[i] = j < n ? u[j] : 0xffffffffu;
        }
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const long long j = j0 + (long long)i * TK_THREADS;
            if (j < n && (x[i] & hi_mask) == prefix) atomicAdd(&hist[(x[i] >> shift) & (nb - 1)], 1u);
        }
    }
    __syncthreads();
    // thread t owns bins [t*per, (t+1)*per) counted from the TOP digit downwards
    const int per = (nb + TK_THREADS - 1) / TK_THREADS;
    uint32_t mine = 0;
    for (int i = 0; i < per; ++i) {
        const int b = nb - 1 - (tid_x() * per + i);
        if (b >= 0) mine += hist[b];
    }
    uint32_t total;
    const uint32_t incl = block_scan_incl(mine, tmp, total);
    const uint32_t excl = incl - mine;
    if (excl < want && want <= incl) {     // exactly one thread: the bucket lies in its bins
        uint32_t run = excl;
        for (int i = 0; i < per; ++i) {
            const int b = nb - 1 - (tid_x() * per + i);
            if (b < 0) break;
            const uint32_t c = hist[b];
            if (run < want && want <= run + c) {
                bcast[0] = (uint32_t)b;
                bcast[1] = want - run;
                bcast[2] = c;
                break;
            }
            run += c;
        }
    }
    __syncthreads();
    prefix |= bcast[0] << shift;
    want = bcast[1];
    __syncthreads();
}

// ascending bitonic sort of a[0..P) in LDS, P a power of two; every thread of the workgroup calls.
// Thread t owns compare-exchange pairs t, t+1024, ...; for distances j <= 32 the 64 pairs of a
// wavefront touch only that wavefront's own 128 elements, so those stages need no workgroup
// barrier (LDS operations of one wavefront execute in order).
template <class T>
__device__ __forceinline__ void bitonic_sort(T *a, int P)
{
    bool need_barrier = true;
    for (int k2 = 2; k2 <= P; k2 <<= 1)
        for (int j = k2 >> 1; j > 0; j >>= 1) {
            if (j >= 64 || need_barrier) __syncthreads();
            else __builtin_amdgcn_wave_barrier();
            need_barrier = j >= 64;          // the stage after a cross-wavefront stage must see its writes
            for (int i = tid_x(); i < P / 2; i += TK_THREADS) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1)), hi = lo | j;
                const bool up = (lo & k2) == 0;
                const T x = a[lo], y = a[hi];
                if ((x > y) == up) {
                    a[lo] = y;
                    a[hi] = x;
                }
            }
        }
    __syncthreads();
}

// elements j..j+3 of row u (zero past the end); one 16-byte load when the row allows it
__device__ __forceinline__ uint4 load4(const uint32_t *u, long long j, long long L, bool vec_ok)
{
    if (vec_ok) return j < L ? *reinterpret_cast<const uint4 *>(u + j) : make_uint4(0, 0, 0, 0);
    uint4 r;
    r.x = j < L ? u[j] : 0u;
    r.y = j + 1 < L ? u[j + 1] : 0u;
    r.z = j + 2 < L ? u[j + 2] : 0u;
    r.w = j + 3 < L ? u[j + 3] : 0u;
    return r;
}

__device__ __forceinline__ int pow2_at_least(int n)
{
    int p = 2;
    while (p < n) p <<= 1;
    return p;
}

__device__ __forceinline__ double load_elem(const void *p, long long i, int esz)
{
    if (esz == 2) return (double)__uint_as_float((uint32_t)static_cast<const unsigned short *>(p)[i] << 16);
    return (double)static_cast<const float *>(p)[i];
}

// alpha[h, j] in fp64 from the inputs (Eq. 5) for the n listed candidates j = cidx[slot[c]]:
//   1/(G*B) * sum over the R rows of exp2(q_r.k_j * scale - M_r) / L_r,
// with (M_r, L_r) the row's softmax statistics merged in fp64 over the key splits.  Four threads per
// row (a quarter of the channels and of the splits each), 256 rows per pass.  Every thread of the
// workgroup calls; out[c] receives the results rounded to fp32 (valid after the final barrier).
__device__ void rescore_candidates(const RescoreArgs &rs, int h, const uint32_t *cidx, const uint32_t *slot, int n, float *out,
                                   float *rowM, double *rowL, double *acc, double *red)
{
    constexpr int ROWS = TK_THREADS / 4;
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
    const int part = tid_x() & 3, rl = tid_x() >> 2;
    const int cpt = rs.d / 4;
    if (tid_x() < n) acc[tid_x()] = 0.0;
    for (int r0 = 0; r0 < rs.R; r0 += ROWS) {              // uniform trip count (one pass unless R > 256)
        const int r = r0 + rl;
        const bool live = r < rs.R;
        // this row's statistics, merged over the key splits
        float M = -INFINITY;
        const long long base = (long long)h * rs.n_split * rs.rpad + (live ? r : 0);
        for (int s = part; s < rs.n_split; s += 4) M = fmaxf(M, rs.stat_m[base + (long long)s * rs.rpad]);
        M = fmaxf(M, __shfl_xor(M, 1));
        M = fmaxf(M, __shfl_xor(M, 2));
        double Lr = 0.0;
        for (int s = part; s < rs.n_split; s += 4) {
            const long long pi = base + (long long)s * rs.rpad;
            Lr += (double)rs.stat_l[pi] * exp2((double)rs.stat_m[pi] - (double)M);
        }
        Lr += __shfl_xor(Lr, 1);
        Lr += __shfl_xor(Lr, 2);
        __syncthreads();                                   // the previous pass is done with rowM / rowL
        if (part == 0) {
            rowM[rl] = M;
            rowL[rl] = Lr;
        }
        __syncthreads();
        const int gl = live ? r / rs.B : 0, qi = live ? r - gl * rs.B : 0;
        const long long qo = ((long long)qi * rs.Hq + (long long)h * rs.G + gl) * rs.d + part * cpt;
        for (int c = 0; c < n; ++c) {
            const long long j = (long long)cidx[slot[c]];
            const long long ko = (j * rs.Hkv + h) * rs.d + part * cpt;
            double p = 0.0;
            if (live)
                for (int e = 0; e < cpt; ++e) p = fma(load_elem(rs.q, qo + e, rs.esz), load_elem(rs.kc, ko + e, rs.esz), p);
            p += __shfl_xor(p, 1);
            p += __shfl_xor(p, 2);
            double t = (live && part == 0) ? exp2(p * (double)rs.scale_log2 - (double)rowM[rl]) / rowL[rl] : 0.0;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) t += __shfl_xor(t, d);
            __syncthreads();                               // red may still be read from the previous candidate
            if (lane == 0) red[wave] = t;
            __syncthreads();
            if (tid_x() == 0) {
                double tot = 0.0;
                for (int w = 0; w < TK_WAVES; ++w) tot += red[w];      // fixed order
                acc[c] += tot;
            }
        }
    }
    __syncthreads();
    if (tid_x() < n) out[tid_x()] = (float)(acc[tid_x()] * rs.inv_rows);
    __syncthreads();
}

__global__ __launch_bounds__(TK_THREADS) void topk_kernel(const float *alpha, const float *group_max, long long L, int k, int32_t *idx_out,
                                                          const RescoreArgs rs)
{
    // one histogram per radix step of the filter route, zeroed together at the start; the radix
    // route reuses the first TK_BINS entries
    constexpr int H_G1 = 0, H_G2 = H_G1 + 4096, H_C1 = H_G2 + 256, H_C2 = H_C1 + 4096, H_C3 = H_C2 + 1024, H_ALL = H_C3 + 1024;
    __shared__ uint32_t hists[H_ALL];
    static_assert(H_ALL >= TK_BINS, "the radix route histograms 12-bit digits in the same array");
    uint32_t *hist = hists;
    __shared__ uint32_t lscan[TK_THREADS];
    __shared__ uint32_t tmp[TK_WAVES + 1];
    __shared__ uint32_t tmp2[TK_WAVES + 1];
    __shared__ uint32_t bcast[3];                        // chosen digit, rank inside its bucket, bucket size
    __shared__ uint32_t n_cand;
    __shared__ uint32_t gmax[TK_GROUPS];                 // group maxima, later the index sort buffer
    __shared__ uint32_t cval[TK_CAND];                   // candidate values (fp32 bit patterns)
    __shared__ uint32_t cidx[TK_CAND];                   // and their positions
    __shared__ uint32_t glist[TK_CAND];                  // groups at or above the bound (handed-in maxima only)
    __shared__ uint32_t n_hit;
    __shared__ uint32_t n_near, n_near_in;
    __shared__ uint32_t near_slot[TK_NEAR_MAX];          // candidates within eps of the k-th value
    __shared__ float near_val[TK_NEAR_MAX];              // their fp64 score, rounded to fp32
    __shared__ double red64[TK_WAVES], near_acc[TK_NEAR_MAX], rowL[TK_THREADS / 4];
    __shared__ float rowM[TK_THREADS / 4];

    const int h = wg_x();
    const uint32_t *u = reinterpret_cast<const uint32_t *>(alpha) + (long long)h * L;
    int32_t *out = idx_out + (long long)h * k;

    if (k <= TK_FILTER_MAX_K) {
        const bool vec_ok = (L & 3) == 0 && (reinterpret_cast<uintptr_t>(u) & 15) == 0;
        const int lane = tid_x() & 63;
        const long long ng = (L + kGroupKeys - 1) / kGroupKeys;       // handed-in group maxima
        // the maxima buffer serves the last phase only (position bitmap / index sort buffer)
        const bool bitmap = L <= (long long)TK_GROUPS * 32;
        uint32_t *bits = gmax;
        int32_t *sidx = reinterpret_cast<int32_t *>(gmax);
        const int words = (int)((L + 31) >> 5);
        const int P2 = pow2_at_least(k);
        // This thread's group maxima, group = slot * 1024 + thread: handed in (if they fit: up to
        // TK_GROUPS of them, the rest reads as zero) or taken here; ranked and compared from
        // registers.  More handed-in maxima than that are ranked from global memory.
        uint32_t gv[TK_SLOTS];
        const uint32_t *gg = group_max ? reinterpret_cast<const uint32_t *>(group_max) + (long long)h * ng : nullptr;
        const bool in_regs = group_max == nullptr || ng <= TK_GROUPS;
#pragma unroll
        for (int s = 0; s < TK_SLOTS; ++s) gv[s] = 0u;
        if (group_max != nullptr) {
            if (in_regs) {
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    const int g = s * TK_THREADS + tid_x();
                    if (g < ng) gv[s] = gg[g];
                }
            }
        } else {
            // ---- sweep 1: strided group maxima; each thread takes 4 consecutive elements per slot
            // (one 16-byte load when the row is aligned)
            for (long long base0 = 0; base0 < L; base0 += 4ll * TK_GROUPS) {
                uint4 x[TK_SLOTS];
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) x[s] = load4(u, base0 + 4ll * (s * TK_THREADS + tid_x()), L, vec_ok);
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    const uint32_t a = x[s].x > x[s].y ? x[s].x : x[s].y, b = x[s].z > x[s].w ? x[s].z : x[s].w;
                    const uint32_t c = a > b ? a : b;
                    gv[s] = c > gv[s] ? c : gv[s];
                }
            }
        }
        // while the loads travel: every histogram and the buffer of the last phase start at zero
        for (int i = tid_x(); i < H_ALL; i += TK_THREADS) hists[i] = 0u;
        if (bitmap) for (int i = tid_x(); i < words; i += TK_THREADS) bits[i] = 0u;
        else for (int i = tid_x(); i < P2; i += TK_THREADS) sidx[i] = 0x7fffffff;
        if (tid_x() == 0) {
            n_cand = 0;
            n_hit = 0;
            n_near = 0;
            n_near_in = 0;
        }
        __syncthreads();
        // a lower bound of the k-th largest group maximum (its top 20 bits), hence of the k-th
        // largest element: at least k elements are >= floor_bits
        uint32_t floor_bits = 0, rank = (uint32_t)k, bucket;
        // slots of this thread that hold a group (group = slot * 1024 + thread); the zeros behind the end of a
        // short row take part in the ranking as one bulk count
        const long long mine = ng > tid_x() ? (ng - tid_x() + TK_THREADS - 1) / TK_THREADS : 0;
        const int live = (group_max != nullptr && in_regs) ? (int)(mine < TK_SLOTS ? mine : TK_SLOTS) : TK_SLOTS;
        const uint32_t n_pad = (group_max != nullptr && in_regs) ? (uint32_t)(TK_GROUPS - ng) : 0u;
        if (in_regs) {
            radix_hist_regs<12>(gv, live, 20, floor_bits, hists + H_G1);
            radix_hist_padding<12>(n_pad, floor_bits, hists + H_G1);
        } else {
            radix_hist_mem<12>(gg, ng, 20, floor_bits, hists + H_G1);
        }
        radix_pick<12>(20, floor_bits, rank, bucket, hists + H_G1, lscan, tmp);
        if (in_regs) {
            radix_hist_regs<8>(gv, live, 12, floor_bits, hists + H_G2);
            radix_hist_padding<8>(n_pad, floor_bits, hists + H_G2);
        } else {
            radix_hist_mem<8>(gg, ng, 12, floor_bits, hists + H_G2);
        }
        radix_pick<8>(12, floor_bits, rank, bucket, hists + H_G2, lscan, tmp2);

        // appends this thread's `cnt` keepers among x[0..NX) (positions j[i] .. j[i]+3) to the candidates
        auto keep = [&](const uint4 *x, const long long *j, int nx, uint32_t cnt) {
            const uint32_t incl = wave_scan_incl(cnt);
            const uint32_t wave_total = lane_value(incl, 63);
            if (wave_total == 0) return;                   // uniform per wavefront
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&n_cand, wave_total);
            uint32_t pos = lane_value(base, 0) + incl - cnt;
            if (cnt) {
                for (int s = 0; s < nx; ++s) {
                    const uint32_t xs[4] = {x[s].x, x[s].y, x[s].z, x[s].w};
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (j[s] >= 0 && j[s] + c < L && xs[c] >= floor_bits) {
                            if (pos < TK_CAND) {
                                cval[pos] = xs[c];
                                cidx[pos] = (uint32_t)(j[s] + c);
                            }
                            ++pos;
                        }
                }
            }
        };
        bool overflow = false;
        if (group_max != nullptr) {
            // ---- the groups at or above the bound, then only their elements ----
            for (long long g0 = 0; g0 < ng; g0 += (long long)TK_THREADS * TK_SLOTS) {     // uniform trip count (one if in_regs)
                if (!in_regs) {
#pragma unroll
                    for (int s = 0; s < TK_SLOTS; ++s) {
                        const long long g = g0 + (long long)s * TK_THREADS + tid_x();
                        gv[s] = g < ng ? gg[g] : 0u;
                    }
                }
                uint32_t cnt = 0;
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    const long long g = g0 + (long long)s * TK_THREADS + tid_x();
                    cnt += (g < ng && gv[s] >= floor_bits);
                }
                const uint32_t incl = wave_scan_incl(cnt);
                const uint32_t wave_total = lane_value(incl, 63);
                if (wave_total == 0) continue;
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(&n_hit, wave_total);
                uint32_t pos = lane_value(base, 0) + incl - cnt;
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    const long long g = g0 + (long long)s * TK_THREADS + tid_x();
                    if (g < ng && gv[s] >= floor_bits) {
                        if (pos < TK_CAND) glist[pos] = (uint32_t)g;
                        ++pos;
                    }
                }
            }
            __syncthreads();
            const uint32_t nh = n_hit;
            overflow = nh > TK_CAND;
            if (!overflow) {
                constexpr int QPG = kGroupKeys / 4;            // 16-byte pieces per group
                constexpr int NX = 4;                           // pieces in flight per thread
                const uint32_t items = nh * QPG;
                for (uint32_t i0 = 0; i0 < items; i0 += TK_THREADS * NX) {                // uniform trip count
                    uint4 x[NX];
                    long long j[NX];
#pragma unroll
                    for (int s = 0; s < NX; ++s) {
                        const uint32_t i = i0 + s * TK_THREADS + tid_x();
                        j[s] = i < items ? (long long)glist[i / QPG] * kGroupKeys + 4 * (i % QPG) : -1;
                        x[s] = j[s] >= 0 ? load4(u, j[s], L, vec_ok) : make_uint4(0, 0, 0, 0);
                    }
                    uint32_t cnt = 0;
#pragma unroll
                    for (int s = 0; s < NX; ++s)
                        if (j[s] >= 0)
                            cnt += (j[s] < L && x[s].x >= floor_bits) + (j[s] + 1 < L && x[s].y >= floor_bits) +
                                   (j[s] + 2 < L && x[s].z >= floor_bits) + (j[s] + 3 < L && x[s].w >= floor_bits);
                    keep(x, j, NX, cnt);
                }
            }
        } else {
            // ---- sweep 2: keep the elements at or above the bound ----
            for (long long base0 = 0; base0 < L; base0 += 4ll * TK_GROUPS) {      // uniform trip count
                uint4 x[TK_SLOTS];
                long long j[TK_SLOTS];
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    j[s] = base0 + 4ll * (s * TK_THREADS + tid_x());
                    x[s] = load4(u, j[s], L, vec_ok);
                }
                uint32_t cnt = 0;
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s)
                    cnt += (j[s] < L && x[s].x >= floor_bits) + (j[s] + 1 < L && x[s].y >= floor_bits) +
                           (j[s] + 2 < L && x[s].z >= floor_bits) + (j[s] + 3 < L && x[s].w >= floor_bits);
                keep(x, j, TK_SLOTS, cnt);
            }
        }
        __syncthreads();
        const uint32_t nc = n_cand;
        if (!overflow && nc <= TK_CAND) {
            // exact k-th value among the candidates (radix select in LDS) and the number of
            // candidates equal to it that belong to the set (the ones with the smallest positions)
            uint32_t thr = 0, want = (uint32_t)k, n_equal;
            radix_step_once<12>(cval, nc, 20, thr, want, n_equal, hists + H_C1, lscan, tmp);
            radix_step_once<10>(cval, nc, 10, thr, want, n_equal, hists + H_C2, lscan, tmp2);
            radix_step_once<10>(cval, nc, 0, thr, want, n_equal, hists + H_C3, lscan, tmp);
            // n_cand now counts the winners (index-sort route); every thread read nc before the
            // barriers of the radix steps
            if (!bitmap) {
                if (tid_x() == 0) n_cand = 0;
                __syncthreads();
            }
            // who is in by the fp32 ranking (ctake); the candidates within eps of the k-th value are listed
            uint32_t *ctake = glist;                         // (the group list has served its purpose)
            const float thr_f = __uint_as_float(thr);
            const uint32_t near_lo = __float_as_uint(thr_f * (1.f - rs.eps)), near_hi = __float_as_uint(thr_f * (1.f + rs.eps));
            const bool rescoring = rs.q != nullptr;
            for (uint32_t i = tid_x(); i < nc; i += TK_THREADS) {
                const uint32_t v = cval[i], j = cidx[i];
                bool take = v > thr;
                if (v == thr) {
                    take = true;
                    if (n_equal != want) {                   // ties cut: keep the `want` smallest positions
                        uint32_t below = 0;
                        for (uint32_t t = 0; t < nc; ++t) below += (cval[t] == thr && cidx[t] < j);
                        take = below < want;
                    }
                }
                ctake[i] = take;
                if (rescoring && v >= near_lo && v <= near_hi) {
                    const uint32_t slot = atomicAdd(&n_near, 1u);
                    if (slot < TK_NEAR_MAX) near_slot[slot] = i;
                    if (take) atomicAdd(&n_near_in, 1u);
                }
            }
            __syncthreads();
            const uint32_t nn = n_near, nin = n_near_in;
            if (rescoring && nn >= 2 && nn <= TK_NEAR_MAX && nin >= 1 && nin < nn) {   // uniform; rare
                rescore_candidates(rs, h, cidx, near_slot, (int)nn, near_val, rowM, rowL, near_acc, red64);
                if (tid_x() < nn) {                      // rank among the near candidates: value, then smaller position
                    const uint32_t me = near_slot[tid_x()];
                    const float v = near_val[tid_x()];
                    uint32_t rank = 0;
                    for (uint32_t c = 0; c < nn; ++c) {
                        const uint32_t o = near_slot[c];
                        rank += (near_val[c] > v) || (near_val[c] == v && cidx[o] < cidx[me]);
                    }
                    ctake[me] = rank < nin;
                }
                __syncthreads();
            }
            for (uint32_t i = tid_x(); i < nc; i += TK_THREADS) {
                if (ctake[i]) {
                    const uint32_t j = cidx[i];
                    if (bitmap) atomicOr(&bits[j >> 5], 1u << (j & 31));
                    else sidx[atomicAdd(&n_cand, 1u)] = (int32_t)j;
                }
            }
            __syncthreads();
            if (bitmap) {
                // ascending order by walking the bitmap of the L positions
                const int wpt = (words + TK_THREADS - 1) / TK_THREADS;      // consecutive words per thread (<= 8)
                uint32_t mine = 0;
                for (int i = 0; i < wpt; ++i) {
                    const int wi = tid_x() * wpt + i;
                    if (wi < words) mine += __popc(bits[wi]);
                }
                uint32_t total;
                uint32_t pos = block_scan_incl(mine, tmp, total) - mine;
                for (int i = 0; i < wpt; ++i) {
                    const int wi = tid_x() * wpt + i;
                    if (wi < words) {
                        uint32_t b = bits[wi];
                        while (b) {
                            const int bit = __ffs(b) - 1;
                            if (pos < (uint32_t)k) out[pos] = (int32_t)(wi * 32 + bit);
                            ++pos;
                            b &= b - 1;
                        }
                    }
                }
            } else {
                bitonic_sort(sidx, P2);
                for (int i = tid_x(); i < k; i += TK_THREADS) out[i] = sidx[i];
            }
            return;
        }
        __syncthreads();                                 // too many ties at the bound: radix route
    }

    // ---- radix route: threshold = bit pattern of the k-th largest value; want = how many
    // elements equal to it belong to the set (those with the smallest indices) ----
    uint32_t prefix = 0, want = (uint32_t)k;
    radix_step(u, L, 20, 12, prefix, want, hist, tmp, bcast);
    radix_step(u, L, 10, 10, prefix, want, hist, tmp, bcast);
    radix_step(u, L, 0, 10, prefix, want, hist, tmp, bcast);
    const uint32_t thr = prefix;

    // ordered sweep: element j goes to slot (#greater before j) + min(#equal before j, want)
    uint32_t base_gt = 0, base_eq = 0;
    for (long long c0 = 0; c0 < L; c0 += (long long)TK_THREADS * TK_EPT) {
        const long long j0 = c0 + (long long)tid_x() * TK_EPT;
        uint32_t x[TK_EPT];
        uint32_t ngt = 0, neq = 0;
#pragma unroll
        for (int i = 0; i < TK_EPT; ++i) {
            x[i] = (j0 + i < L) ? u[j0 + i] : 0u;
            const bool in = j0 + i < L;
            ngt += (in && x[i] > thr) ? 1u : 0u;
            neq += (in && x[i] == thr) ? 1u : 0u;
        }
        uint32_t tot_gt, tot_eq;
        const uint32_t pre_gt = block_scan_incl(ngt, tmp, tot_gt) - ngt + base_gt;
        const uint32_t pre_eq = block_scan_incl(neq, tmp2, tot_eq) - neq + base_eq;
        uint32_t g = pre_gt, e = pre_eq;
#pragma unroll
        for (int i = 0; i < TK_EPT; ++i) {
            if (j0 + i < L) {
                if (x[i] > thr) {
                    out[g + (e < want ? e : want)] = (int32_t)(j0 + i);
                    ++g;
                } else if (x[i] == thr) {
                    if (e < want) out[g + e] = (int32_t)(j0 + i);
                    ++e;
                }
            }
        }
        base_gt += tot_gt;
        base_eq += tot_eq;
    }
}

// group_max: nullptr, or [Hkv][ceil(L / kGroupKeys)] maxima of alpha over groups of kGroupKeys consecutive positions
hipError_t launch_topk(const float *alpha, const float *group_max, int Hkv, long long L, int k, int32_t *idx_out, const RescoreArgs &rs,
                       hipStream_t stream)
{
    hipLaunchKernelGGL(topk_kernel, dim3(Hkv), dim3(TK_THREADS), 0, stream, alpha, group_max, L, k, idx_out, rs);
    return hipGetLastError();
}

}  // namespace mage
