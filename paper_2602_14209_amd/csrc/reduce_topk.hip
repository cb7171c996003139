// Small kernels around the attention passes (gfx950):
//   combine_kernel   merges the split-key partials of an attention call into out / lse
//   lse_kernel       merges the statistics partials of selection into one log2-domain
//                    log-sum-exp per query row
//   topk_kernel      per KV head, exact top-k of alpha[h, 0..L) by radix select on the fp32 bit
//                    patterns (alpha >= 0, so unsigned integer order is float order), ties to
//                    the smaller index, output ascending (Alg. 1 "S <- Top-k(alpha)", Eq. 5)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.hpp"

namespace mage {

// One thread per (row, 4 channels).  Split s contributes weight exp2(m_s - M).
template <int D>
__global__ __launch_bounds__(256) void combine_kernel(const KernelArgs a)
{
    constexpr int TPR = D / 4;                 // threads per row
    constexpr int ROWS = 256 / TPR;            // rows per workgroup
    const int h = blockIdx.y;
    const int row = blockIdx.x * ROWS + threadIdx.x / TPR;
    const int c4 = threadIdx.x % TPR;
    if (row >= a.R) return;

    float M = -INFINITY;
#pragma unroll 8
    for (int s = 0; s < a.n_split; ++s) M = fmaxf(M, a.part_m[((long long)h * a.n_split + s) * a.rpad + row]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float lt = 0.f;
#pragma unroll 8
    for (int s = 0; s < a.n_split; ++s) {
        const long long pi = ((long long)h * a.n_split + s) * a.rpad + row;
        const float w = exp2f(a.part_m[pi] - M);
        lt = fmaf(w, a.part_l[pi], lt);
        const float4 v = *reinterpret_cast<const float4 *>(a.part_o + pi * D + c4 * 4);
        acc.x = fmaf(w, v.x, acc.x);
        acc.y = fmaf(w, v.y, acc.y);
        acc.z = fmaf(w, v.z, acc.z);
        acc.w = fmaf(w, v.w, acc.w);
    }
    const float inv = 1.f / lt;
    const int gl = row / a.B, qi = row - gl * a.B;
    const long long orow = (long long)qi * a.Hq + (long long)h * a.G + gl;
    *reinterpret_cast<float4 *>(a.out + orow * D + c4 * 4) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
    if (a.lse_out && c4 == 0) a.lse_out[orow] = (M + log2f(lt)) * 0.6931471805599453f;
}

// lse2[h][row] = M + log2( sum_s l_s * 2^(m_s - M) ): one wavefront per row, lane s takes splits
// s, s+64, ...; the sum is accumulated in fp64 in a fixed order.
__global__ __launch_bounds__(256) void lse_kernel(const KernelArgs a, float *lse2_out)
{
    const int h = blockIdx.y;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= a.R) return;
    float M = -INFINITY;
    for (int s = lane; s < a.n_split; s += 64) M = fmaxf(M, a.part_m[((long long)h * a.n_split + s) * a.rpad + row]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d));
    double lt = 0.0;
    for (int s = lane; s < a.n_split; s += 64) {
        const long long pi = ((long long)h * a.n_split + s) * a.rpad + row;
        lt += (double)a.part_l[pi] * (double)exp2f(a.part_m[pi] - M);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) lt += __shfl_xor(lt, d);
    if (lane == 0) lse2_out[(long long)h * a.rpad + row] = M + (float)log2(lt);
}

// ------------------------------------------------------------------------------ top-k
constexpr int TK_THREADS = 1024;
constexpr int TK_WAVES = TK_THREADS / 64;
constexpr int TK_BINS = 4096;            // widest digit: 12 bits
constexpr int TK_EPT = 16;               // consecutive elements per thread in the emit pass

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

// One radix step: histogram the `bits`-wide digit at `shift` of every element whose higher
// bits equal `prefix`, then pick the digit in which the `want`-th largest element falls.
// On return prefix has that digit appended and want is the rank inside the digit's bucket.
__device__ __forceinline__ void radix_step(const uint32_t *u, long long L, int shift, int bits,
                                           uint32_t &prefix, uint32_t &want,
                                           uint32_t *hist, uint32_t *tmp, uint32_t *bcast)
{
    const int nb = 1 << bits;
    const uint32_t hi_mask = (shift + bits >= 32) ? 0u : (0xffffffffu << (shift + bits));
    for (int b = threadIdx.x; b < nb; b += TK_THREADS) hist[b] = 0;
    __syncthreads();
    constexpr int UNR = 8;      // independent loads in flight per thread
    for (long long j0 = threadIdx.x; j0 < L; j0 += (long long)TK_THREADS * UNR) {
        uint32_t x[UNR];
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const long long j = j0 + (long long)i * TK_THREADS;
            x[i] = j < L ? u[j] : 0xffffffffu;
        }
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const long long j = j0 + (long long)i * TK_THREADS;
            if (j < L && (x[i] & hi_mask) == prefix) atomicAdd(&hist[(x[i] >> shift) & (nb - 1)], 1u);
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

__global__ __launch_bounds__(TK_THREADS) void topk_kernel(const float *alpha, long long L, int k, int32_t *idx_out)
{
    __shared__ uint32_t hist[TK_BINS];
    __shared__ uint32_t tmp[TK_WAVES + 1];
    __shared__ uint32_t bcast[2];
    __shared__ uint32_t tmp2[TK_WAVES + 1];

    const int h = blockIdx.x;
    const uint32_t *u = reinterpret_cast<const uint32_t *>(alpha) + (long long)h * L;
    int32_t *out = idx_out + (long long)h * k;

    // threshold = bit pattern of the k-th largest value; want = how many elements equal to it
    // belong to the set (those with the smallest indices)
    uint32_t prefix = 0, want = (uint32_t)k;
    radix_step(u, L, 20, 12, prefix, want, hist, tmp, bcast);
    radix_step(u, L, 10, 10, prefix, want, hist, tmp, bcast);
    radix_step(u, L, 0, 10, prefix, want, hist, tmp, bcast);
    const uint32_t thr = prefix;

    // ordered emit: element j goes to slot (#greater before j) + min(#equal before j, want)
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

hipError_t launch_combine(const KernelArgs &a, int d, hipStream_t stream)
{
    const int rows_per_wg = 256 / (d / 4);
    dim3 grid((a.R + rows_per_wg - 1) / rows_per_wg, a.Hkv), block(256);
    if (d == 128) hipLaunchKernelGGL((combine_kernel<128>), grid, block, 0, stream, a);
    else if (d == 64) hipLaunchKernelGGL((combine_kernel<64>), grid, block, 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_lse(const KernelArgs &a, float *lse2_out, hipStream_t stream)
{
    dim3 grid((a.R + 3) / 4, a.Hkv), block(256);
    hipLaunchKernelGGL(lse_kernel, grid, block, 0, stream, a, lse2_out);
    return hipGetLastError();
}

hipError_t launch_topk(const float *alpha, int Hkv, long long L, int k, int32_t *idx_out, hipStream_t stream)
{
    hipLaunchKernelGGL(topk_kernel, dim3(Hkv), dim3(TK_THREADS), 0, stream, alpha, L, k, idx_out);
    return hipGetLastError();
}

}  // namespace mage
