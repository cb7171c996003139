// Small kernels of the second workload (gfx950): a Quest-style page estimator under per-block
// selection (Sec. 2 "Methods for AR LLMs"; Eq. 2, per-block form, with the estimator's scores) and
// the set-overlap ratio of Eq. 1 / Eq. 3.
//
// The page score sum_c max(q_c Kmax_c, q_c Kmin_c) is linear once the query is split by sign:
// max(q*a, q*b) with a >= b is q*a for q >= 0 and q*b for q < 0, so the score is the dot product of
// [max(q,0) | min(q,0)] with the page's row [Kmax | Kmin] of length 2d.  The summaries are
// therefore stored as such rows, the queries are split here, and the scoring, the softmax over
// pages and the block/group average run on the MFMA selection kernels with head dimension 2d.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "ids.hpp"

namespace mage {

// summary[P][h][0][:] = per-channel max, summary[P][h][1][:] = per-channel min of the key rows of page
// P = [P*p, min((P+1)*p, L)).  One thread per 16-byte piece of a (page, head) row.
template <bool BF16>
__global__ __launch_bounds__(256) void page_summary_kernel(const unsigned char *__restrict__ kc, unsigned char *__restrict__ out,
                                                           long long n_pages, int Hkv, int d, int p, long long L)
{
    constexpr int ESZ = BF16 ? 2 : 4, VEC = 16 / ESZ;
    const int cpr = d / VEC;
    const long long t = (long long)wg_x() * 256 + tid_x();
    if (t >= n_pages * Hkv * cpr) return;
    const long long P = t / ((long long)Hkv * cpr);
    const int rem = (int)(t % ((long long)Hkv * cpr)), h = rem / cpr, c = rem % cpr;
    float mx[VEC], mn[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        mx[e] = -INFINITY;
        mn[e] = INFINITY;
    }
    const long long j1 = (P + 1) * p < L ? (P + 1) * p : L;
    for (long long j = P * p; j < j1; ++j) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(kc + ((j * Hkv + h) * (long long)d + c * VEC) * ESZ);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float v = BF16 ? __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16)) : __uint_as_float(w[e]);
            mx[e] = fmaxf(mx[e], v);
            mn[e] = fminf(mn[e], v);
        }
    }
    uint32_t wx[4], wn[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (BF16) {     // the values are bf16-representable: the upper 16 bits are the number
            wx[i] = (__float_as_uint(mx[2 * i]) >> 16) | (__float_as_uint(mx[2 * i + 1]) & 0xffff0000u);
            wn[i] = (__float_as_uint(mn[2 * i]) >> 16) | (__float_as_uint(mn[2 * i + 1]) & 0xffff0000u);
        } else {
            wx[i] = __float_as_uint(mx[i]);
            wn[i] = __float_as_uint(mn[i]);
        }
    }
    unsigned char *row = out + (((P * Hkv + h) * 2) * (long long)d + c * VEC) * ESZ;
    *reinterpret_cast<uint4 *>(row) = make_uint4(wx[0], wx[1], wx[2], wx[3]);
    *reinterpret_cast<uint4 *>(row + (long long)d * ESZ) = make_uint4(wn[0], wn[1], wn[2], wn[3]);
}

// q2[q][g][0:d] = max(q, 0), q2[q][g][d:2d] = min(q, 0)   (bf16 bit patterns; -0 counts as negative)
__global__ __launch_bounds__(256) void quest_query_kernel(const uint16_t *__restrict__ q, uint16_t *__restrict__ q2, long long rows, int d)
{
    const long long t = (long long)wg_x() * 256 + tid_x();
    if (t >= rows * d) return;
    const long long r = t / d;
    const int c = (int)(t % d);
    const uint16_t v = q[t];
    const bool neg = (v & 0x8000u) != 0;
    q2[r * 2 * d + c] = neg ? (uint16_t)0 : v;
    q2[r * 2 * d + d + c] = neg ? v : (uint16_t)0;
}

// idx[h][i] = pages[h][i / p] * p + i % p: the positions of the selected pages, ascending when the pages are
__global__ __launch_bounds__(256) void expand_pages_kernel(const int32_t *__restrict__ pages, int32_t *__restrict__ idx, int Hkv, int k, int p)
{
    const long long t = (long long)wg_x() * 256 + tid_x();
    if (t >= (long long)Hkv * k) return;
    const int h = (int)(t / k), i = (int)(t % k);
    idx[t] = pages[(long long)h * (k / p) + i / p] * p + i % p;
}

// out[i] = |A_(i % a_rows) intersect B_i| / k.  Rows of `a` ascending (binary search), rows of `b` in any order.
__global__ __launch_bounds__(256) void overlap_kernel(const int32_t *__restrict__ a, const int32_t *__restrict__ b, int k, int a_rows,
                                                      float *__restrict__ out)
{
    __shared__ int part[4];
    const int i = wg_x();
    const int32_t *ar = a + (long long)(i % a_rows) * k, *br = b + (long long)i * k;
    int cnt = 0;
    for (int e = tid_x(); e < k; e += 256) {
        const int32_t v = br[e];
        int lo = 0, hi = k;                 // first position with ar[pos] >= v
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (ar[mid] < v) lo = mid + 1;
            else hi = mid;
        }
        cnt += (lo < k && ar[lo] == v) ? 1 : 0;
    }
#pragma unroll
    for (int dlt = 32; dlt >= 1; dlt >>= 1) cnt += __shfl_xor(cnt, dlt);
    if ((tid_x() & 63) == 0) part[tid_x() >> 6] = cnt;
    __syncthreads();
    if (tid_x() == 0) out[i] = (float)(part[0] + part[1] + part[2] + part[3]) / (float)k;
}

hipError_t launch_page_summary(const void *kc, void *out, long long L, int Hkv, int d, int p, bool bf16, hipStream_t stream)
{
    const long long n_pages = (L + p - 1) / p;
    const long long threads = n_pages * Hkv * (d / (bf16 ? 8 : 4));
    dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    if (bf16)
        hipLaunchKernelGGL(page_summary_kernel<true>, grid, block, 0, stream, (const unsigned char *)kc, (unsigned char *)out, n_pages, Hkv, d, p, L);
    else
        hipLaunchKernelGGL(page_summary_kernel<false>, grid, block, 0, stream, (const unsigned char *)kc, (unsigned char *)out, n_pages, Hkv, d, p, L);
    return hipGetLastError();
}

hipError_t launch_quest_query(const void *q, void *q2, long long rows, int d, hipStream_t stream)
{
    dim3 grid((unsigned)((rows * d + 255) / 256)), block(256);
    hipLaunchKernelGGL(quest_query_kernel, grid, block, 0, stream, (const uint16_t *)q, (uint16_t *)q2, rows, d);
    return hipGetLastError();
}

hipError_t launch_expand_pages(const int32_t *pages, int32_t *idx, int Hkv, int k, int p, hipStream_t stream)
{
    dim3 grid((unsigned)(((long long)Hkv * k + 255) / 256)), block(256);
    hipLaunchKernelGGL(expand_pages_kernel, grid, block, 0, stream, pages, idx, Hkv, k, p);
    return hipGetLastError();
}

hipError_t launch_overlap(const int32_t *a, const int32_t *b, int n_rows, int k, int a_rows, float *out, hipStream_t stream)
{
    hipLaunchKernelGGL(overlap_kernel, dim3(n_rows), dim3(256), 0, stream, a, b, k, a_rows, out);
    return hipGetLastError();
}

}  // namespace mage
