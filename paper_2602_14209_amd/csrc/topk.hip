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
//     The group maxima either come with the row (the column-sum pass leaves one per kGroupKeys
//     consecutive keys; only the groups at or above the bound are then read at all) or are
//     taken here over 8192 strided groups in a first sweep of the row.
//   radix route (any k, any tie structure; also the overflow exit of the filter route): three
//     MSB-first radix-select steps over the whole row find the k-th value and the number of
//     ties to keep, then an ordered sweep emits the set.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.hpp"
#include "probe.hpp"

namespace mage {

constexpr int TK_THREADS = 1024;
constexpr int TK_WAVES = TK_THREADS / 64;
constexpr int TK_BINS = 4096;                        // widest digit: 12 bits
constexpr int TK_EPT = 16;                           // consecutive elements per thread in the ordered sweep
constexpr int TK_SLOTS = 8;                          // group maxima per thread = loads in flight per thread
constexpr int TK_GROUPS = TK_THREADS * TK_SLOTS;     // 8192
constexpr int TK_CAND = 4096;                        // candidate capacity of the filter route
constexpr int TK_FILTER_MAX_K = 2048;

// inclusive scan of one value per thread over the workgroup; returns this thread's inclusive
// prefix and the workgroup total.  `tmp` holds TK_WAVES+1 entries.
__device__ __forceinline__ uint32_t block_scan_incl(uint32_t v, uint32_t *tmp, uint32_t &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    __syncthreads();                      // tmp may still be read from a previous call
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int w = 0; w < TK_WAVES; ++w) {
            const uint32_t t = tmp[w];
            tmp[w] = run;
            run += t;
        }
        tmp[TK_WAVES] = run;
    }
    __syncthreads();
    total = tmp[TK_WAVES];
    return x + tmp[wave];
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
    for (int b = threadIdx.x; b < nb; b += TK_THREADS) hist[b] = 0;
    __syncthreads();
    constexpr int UNR = 8;      // independent loads in flight per thread
    for (long long j0 = threadIdx.x; j0 < n; j0 += (long long)TK_THREADS * UNR) {
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
        const int b = nb - 1 - (threadIdx.x * per + i);
        if (b >= 0) mine += hist[b];
    }
    uint32_t total;
    const uint32_t incl = block_scan_incl(mine, tmp, total);
    const uint32_t excl = incl - mine;
    if (excl < want && want <= incl) {     // exactly one thread: the bucket lies in its bins
        uint32_t run = excl;
        for (int i = 0; i < per; ++i) {
            const int b = nb - 1 - (threadIdx.x * per + i);
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
            for (int i = threadIdx.x; i < P / 2; i += TK_THREADS) {
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

__global__ __launch_bounds__(TK_THREADS) void topk_kernel(const float *alpha, const float *group_max, long long L, int k, int32_t *idx_out)
{
    __shared__ uint32_t hist[TK_BINS];
    __shared__ uint32_t tmp[TK_WAVES + 1];
    __shared__ uint32_t tmp2[TK_WAVES + 1];
    __shared__ uint32_t bcast[3];                        // chosen digit, rank inside its bucket, bucket size
    __shared__ uint32_t n_cand;
    __shared__ uint32_t gmax[TK_GROUPS];                 // group maxima, later the index sort buffer
    __shared__ uint32_t cval[TK_CAND];                   // candidate values (fp32 bit patterns)
    __shared__ uint32_t cidx[TK_CAND];                   // and their positions
    __shared__ uint32_t glist[TK_CAND];                  // groups at or above the bound (handed-in maxima only)
    __shared__ uint32_t n_hit;

    const int h = blockIdx.x;
    const uint32_t *u = reinterpret_cast<const uint32_t *>(alpha) + (long long)h * L;
    int32_t *out = idx_out + (long long)h * k;

    MAGE_PROBE_DECL;
    MAGE_PROBE_AT(0);
    if (k <= TK_FILTER_MAX_K) {
        const bool vec_ok = (L & 3) == 0 && (reinterpret_cast<uintptr_t>(u) & 15) == 0;
        const int lane = threadIdx.x & 63;
        const long long ng = (L + kGroupKeys - 1) / kGroupKeys;       // handed-in group maxima
        const uint32_t *gsrc = gmax;                                   // where the maxima are ranked from
        long long gcount = TK_GROUPS;
        if (group_max != nullptr) {
            const uint32_t *gg = reinterpret_cast<const uint32_t *>(group_max) + (long long)h * ng;
            if (ng <= TK_GROUPS) {
                for (int i = threadIdx.x; i < TK_GROUPS; i += TK_THREADS) gmax[i] = i < ng ? gg[i] : 0u;
            } else {
                gsrc = gg;
            }
            gcount = ng <= TK_GROUPS ? TK_GROUPS : ng;
        } else {
            // ---- sweep 1: strided group maxima (group = slot * 1024 + thread); each thread takes 4
            // consecutive elements per slot (one 16-byte load when the row is aligned)
            uint32_t gm[TK_SLOTS];
#pragma unroll
            for (int s = 0; s < TK_SLOTS; ++s) gm[s] = 0u;
            for (long long base0 = 0; base0 < L; base0 += 4ll * TK_GROUPS) {
                uint4 x[TK_SLOTS];
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) x[s] = load4(u, base0 + 4ll * (s * TK_THREADS + threadIdx.x), L, vec_ok);
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    const uint32_t a = x[s].x > x[s].y ? x[s].x : x[s].y, b = x[s].z > x[s].w ? x[s].z : x[s].w;
                    const uint32_t c = a > b ? a : b;
                    gm[s] = c > gm[s] ? c : gm[s];
                }
            }
#pragma unroll
            for (int s = 0; s < TK_SLOTS; ++s) gmax[s * TK_THREADS + threadIdx.x] = gm[s];
        }
        if (threadIdx.x == 0) {
            n_cand = 0;
            n_hit = 0;
        }
        __syncthreads();
        MAGE_PROBE_AT(1);
        // a lower bound of the k-th largest group maximum (its top 20 bits), hence of the k-th
        // largest element: at least k elements are >= floor_bits
        uint32_t floor_bits = 0, rank = (uint32_t)k;
        radix_step(gsrc, gcount, 20, 12, floor_bits, rank, hist, tmp, bcast);
        radix_step(gsrc, gcount, 12, 8, floor_bits, rank, hist, tmp, bcast);

        MAGE_PROBE_AT(2);
        // appends this thread's `cnt` keepers among x[0..NX) (positions j[i] .. j[i]+3) to the candidates
        auto keep = [&](const uint4 *x, const long long *j, int nx, uint32_t cnt) {
            uint32_t incl = cnt;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t y = __shfl_up(incl, d);
                if (lane >= d) incl += y;
            }
            const uint32_t wave_total = __shfl(incl, 63);
            if (wave_total == 0) return;                   // uniform per wavefront
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&n_cand, wave_total);
            uint32_t pos = __shfl(base, 0) + incl - cnt;
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
            for (long long g0 = 0; g0 < ng; g0 += (long long)TK_THREADS * TK_SLOTS) {     // uniform trip count
                uint32_t gv[TK_SLOTS];
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    const long long g = g0 + (long long)s * TK_THREADS + threadIdx.x;
                    gv[s] = g < ng ? gsrc[g] : 0u;
                }
                uint32_t cnt = 0;
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    const long long g = g0 + (long long)s * TK_THREADS + threadIdx.x;
                    cnt += (g < ng && gv[s] >= floor_bits);
                }
                uint32_t incl = cnt;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const uint32_t y = __shfl_up(incl, d);
                    if (lane >= d) incl += y;
                }
                const uint32_t wave_total = __shfl(incl, 63);
                if (wave_total == 0) continue;
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(&n_hit, wave_total);
                uint32_t pos = __shfl(base, 0) + incl - cnt;
#pragma unroll
                for (int s = 0; s < TK_SLOTS; ++s) {
                    const long long g = g0 + (long long)s * TK_THREADS + threadIdx.x;
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
                        const uint32_t i = i0 + s * TK_THREADS + threadIdx.x;
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
                    j[s] = base0 + 4ll * (s * TK_THREADS + threadIdx.x);
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
        MAGE_PROBE_AT(3);
        const uint32_t nc = n_cand;
        if (!overflow && nc <= TK_CAND) {
            // exact k-th value among the candidates (radix select in LDS) and the number of
            // candidates equal to it that belong to the set (the ones with the smallest positions)
            uint32_t thr = 0, want = (uint32_t)k;
            radix_step(cval, nc, 20, 12, thr, want, hist, tmp, bcast);
            radix_step(cval, nc, 10, 10, thr, want, hist, tmp, bcast);
            radix_step(cval, nc, 0, 10, thr, want, hist, tmp, bcast);
            const uint32_t n_equal = bcast[2];
            __syncthreads();
            const bool bitmap = L <= (long long)TK_GROUPS * 32;
            uint32_t *bits = gmax;                           // reuses the group-maxima buffer
            int32_t *sidx = reinterpret_cast<int32_t *>(gmax);
            const int words = (int)((L + 31) >> 5);
            const int P2 = pow2_at_least(k);
            if (bitmap) for (int i = threadIdx.x; i < words; i += TK_THREADS) bits[i] = 0u;
            else for (int i = threadIdx.x; i < P2; i += TK_THREADS) sidx[i] = 0x7fffffff;
            if (threadIdx.x == 0) n_cand = 0;                // now counts the winners (index-sort route)
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < nc; i += TK_THREADS) {
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
                if (take) {
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
                    const int wi = threadIdx.x * wpt + i;
                    if (wi < words) mine += __popc(bits[wi]);
                }
                uint32_t total;
                uint32_t pos = block_scan_incl(mine, tmp, total) - mine;
                for (int i = 0; i < wpt; ++i) {
                    const int wi = threadIdx.x * wpt + i;
                    if (wi < words) {
                        uint32_t b = bits[wi];
                        while (b) {
                            const int bit = __ffs(b) - 1;
                            out[pos++] = (int32_t)(wi * 32 + bit);
                            b &= b - 1;
                        }
                    }
                }
            } else {
                bitonic_sort(sidx, P2);
                for (int i = threadIdx.x; i < k; i += TK_THREADS) out[i] = sidx[i];
            }
            MAGE_PROBE_AT(4);
            MAGE_PROBE_FLUSH();
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
        const long long j0 = c0 + (long long)threadIdx.x * TK_EPT;
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
hipError_t launch_topk(const float *alpha, const float *group_max, int Hkv, long long L, int k, int32_t *idx_out, hipStream_t stream)
{
    hipLaunchKernelGGL(topk_kernel, dim3(Hkv), dim3(TK_THREADS), 0, stream, alpha, group_max, L, k, idx_out);
    return hipGetLastError();
}

}  // namespace mage
