// Small kernels around the attention passes (gfx950):
//   combine_kernel   merges the split-key partials of an attention call into out / lse
//                    (and, for the fused step 1, the prefix statistics into selection's lse)
//   lse_kernel       merges the statistics partials of selection into one log2-domain
//                    log-sum-exp per query row
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ids.hpp"
#include "plan.hpp"

namespace mage {

// One workgroup per (query row, KV head): 256 threads = D/4 channel quads x SG split groups.
// Split s contributes weight exp2(m_s - M); group g walks splits g, g+SG, ... with all its loads
// in flight, then the groups are added in a fixed order through LDS.
template <int D>
__global__ __launch_bounds__(256) void combine_kernel(const KernelArgs a)
{
    constexpr int TPR = D / 4;                 // threads per row of channels
    constexpr int SG = 256 / TPR;              // split groups
    __shared__ float red_m[4];
    __shared__ float4 red_o[SG][TPR];
    __shared__ float red_l[SG];
    const int row = wg_x(), h = wg_y();
    const int c4 = tid_x() % TPR, sg = tid_x() / TPR;
    const long long base = (long long)h * a.n_split * a.rpad + row;

    // fused step 1: the last wavefront also merges the prefix-only statistics of this row into the
    // log-sum-exp that the column sums need (as lse_kernel would)
    if (a.lse2_out != nullptr && (tid_x() >> 6) == 3) {
        const int lane = tid_x() & 63;
        float Mp = -INFINITY;
        for (int s = lane; s < a.n_split; s += 64) Mp = fmaxf(Mp, a.stat_m[base + (long long)s * a.rpad]);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) Mp = fmaxf(Mp, __shfl_xor(Mp, d));
        double lp = 0.0;
        for (int s = lane; s < a.n_split; s += 64) {
            const long long pi = base + (long long)s * a.rpad;
            lp += (double)a.stat_l[pi] * (double)exp2f(a.stat_m[pi] - Mp);
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) lp += __shfl_xor(lp, d);
        if (lane == 0) a.lse2_out[(long long)h * a.rpad + row] = Mp + (float)log2(lp);
    }

    float M = -INFINITY;
    for (int s = tid_x(); s < a.n_split; s += 256) M = fmaxf(M, a.part_m[base + (long long)s * a.rpad]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d));
    if ((tid_x() & 63) == 0) red_m[tid_x() >> 6] = M;
    __syncthreads();
    M = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float lt = 0.f;
#pragma unroll 4
    for (int s = sg; s < a.n_split; s += SG) {
        const long long pi = base + (long long)s * a.rpad;
        const float w = exp2f(a.part_m[pi] - M);
        lt = fmaf(w, a.part_l[pi], lt);
        const float4 v = *reinterpret_cast<const float4 *>(a.part_o + pi * D + c4 * 4);
        acc.x = fmaf(w, v.x, acc.x);
        acc.y = fmaf(w, v.y, acc.y);
        acc.z = fmaf(w, v.z, acc.z);
        acc.w = fmaf(w, v.w, acc.w);
    }
    red_o[sg][c4] = acc;
    if (c4 == 0) red_l[sg] = lt;
    __syncthreads();
    if (sg != 0) return;
    acc = red_o[0][c4];
    lt = red_l[0];
#pragma unroll
    for (int g = 1; g < SG; ++g) {
        const float4 v = red_o[g][c4];
        acc.x += v.x;
        acc.y += v.y;
        acc.z += v.z;
        acc.w += v.w;
        lt += red_l[g];
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
    const int h = wg_y();
    const int row = wg_x() * 4 + (tid_x() >> 6);
    const int lane = tid_x() & 63;
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

hipError_t launch_combine(const KernelArgs &a, int d, hipStream_t stream)
{
    dim3 grid(a.R, a.Hkv), block(256);
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

}  // namespace mage
