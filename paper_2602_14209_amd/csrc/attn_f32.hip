// fp32 vector-ALU kernels of the MAGE hot path for gfx950: the MAGE_F32 element type.
//
// Same decomposition as the bf16 path (split-key flash-style partials; statistics pass and
// column-sum pass for selection) but with plain fp32 FMA arithmetic: 256 threads cover 64
// query rows, 4 threads per row; a 32-key K / V tile is staged in LDS; thread (row, sub)
// scores keys sub, sub+4, ... and then accumulates a quarter of the head dimension.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ids.hpp"
#include "plan.hpp"

namespace mage {

enum { F32_ATTN = 0, F32_STATS = 1 };

struct F32Range {
    long long c0, c1;
    int cache_tiles, blk_tiles;
};

__device__ __forceinline__ F32Range f32_range(const KernelArgs &a, int s)
{
    F32Range r;
    r.c0 = (long long)s * a.kps;
    r.c1 = r.c0 + a.kps;
    if (r.c1 > a.nc) r.c1 = a.nc;
    if (r.c0 > r.c1) r.c0 = r.c1;
    r.cache_tiles = (int)((r.c1 - r.c0 + kF32Tile - 1) / kF32Tile);
    r.blk_tiles = (s == a.blk_split) ? (a.n_blk + kF32Tile - 1) / kF32Tile : 0;
    return r;
}

// rows [row0, row0+64) of KV head h -> LDS, zero-filled past R
template <int D>
__device__ __forceinline__ void f32_load_q(const KernelArgs &a, int h, int row0, float (*qs)[D + 1], int row_end = 1 << 30)
{
    const float *q = static_cast<const float *>(a.q);
    for (int e = tid_x(); e < kF32Rows * D; e += 256) {
        const int r = e / D, c = e - r * D, row = row0 + r;
        float v = 0.f;
        if (row < a.R && row < row_end) {
            const int gl = row / a.B, qi = row - gl * a.B;
            v = q[((long long)qi * a.Hq + (long long)h * a.G + gl) * D + c];
        }
        qs[r][c] = v;
    }
}

template <int D, int MODE, bool GATHER>
__global__ __launch_bounds__(256) void attn_f32_kernel(const KernelArgs a)
{
    constexpr bool WITH_V = (MODE == F32_ATTN);
    constexpr int DS = D / 4;      // channels per thread in the P.V phase
    __shared__ float qs[kF32Rows][D + 1];
    __shared__ float ks[kF32Tile][D + 1];
    __shared__ float vs[WITH_V ? kF32Tile : 1][D];
    __shared__ float ps[kF32Rows][kF32Tile + 1];

    const int h = wg_x(), split = wg_y(), rg = wg_z();
    const int r = tid_x() >> 2, sub = tid_x() & 3;
    const int row0 = rg * kF32Rows, row = row0 + r;

    const F32Range sr = f32_range(a, split);
    const int ntiles = sr.cache_tiles + sr.blk_tiles;

    f32_load_q<D>(a, h, row0, qs);

    float o[WITH_V ? DS : 1];
#pragma unroll
    for (int c = 0; c < (WITH_V ? DS : 1); ++c) o[c] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const long long stride = (long long)a.Hkv * D;
    const float *kc = static_cast<const float *>(a.kc) + (long long)h * D;
    const float *vc = static_cast<const float *>(a.vc) + (long long)h * D;
    const float *kb = static_cast<const float *>(a.kblk) + (long long)h * D;
    const float *vb = static_cast<const float *>(a.vblk) + (long long)h * D;
    const int32_t *idx = GATHER ? a.idx + (long long)h * a.nc : nullptr;

    for (int t = 0; t < ntiles; ++t) {
        int valid;
        const bool from_cache = t < sr.cache_tiles;
        long long base;
        if (from_cache) {
            base = sr.c0 + (long long)t * kF32Tile;
            const long long left = sr.c1 - base;
            valid = left < kF32Tile ? (int)left : kF32Tile;
        } else {
            base = (long long)(t - sr.cache_tiles) * kF32Tile;
            const int left = a.n_blk - (int)base;
            valid = left < kF32Tile ? left : kF32Tile;
        }
        __syncthreads();      // previous tile fully consumed (also orders the Q load before first use)
        for (int e = tid_x(); e < kF32Tile * D; e += 256) {
            const int key = e / D, c = e - key * D;
            const long long pos = base + (key < valid ? key : valid - 1);
            const long long src = from_cache ? (GATHER ? (long long)idx[pos] : pos) : pos;
            ks[key][c] = (from_cache ? kc : kb)[src * stride + c];
            if (WITH_V) vs[key][c] = (from_cache ? vc : vb)[src * stride + c];
        }
        __syncthreads();

        float s[kF32Tile / 4];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < kF32Tile / 4; ++i) {
            const int key = sub + 4 * i;
            float acc = 0.f;
#pragma unroll 8
            for (int c = 0; c < D; ++c) acc = fmaf(qs[r][c], ks[key][c], acc);
            acc *= a.scale_log2;
            if (key >= valid) acc = -INFINITY;
            s[i] = acc;
            mx = fmaxf(mx, acc);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 1));
        mx = fmaxf(mx, __shfl_xor(mx, 2));
        const float m_new = fmaxf(m_run, mx);
        const float corr = exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < kF32Tile / 4; ++i) {
            const float p = exp2f(s[i] - m_new);
            psum += p;
            if (WITH_V) ps[r][sub + 4 * i] = p;
        }
        l_run = l_run * corr + psum;

        if (WITH_V) {
            __syncthreads();
#pragma unroll
            for (int c = 0; c < DS; ++c) o[c] *= corr;
            for (int key = 0; key < kF32Tile; ++key) {
                const float p = ps[r][key];
#pragma unroll
                for (int c = 0; c < DS; ++c) o[c] = fmaf(p, vs[key][sub * DS + c], o[c]);
            }
        }
    }

    float l_tot = l_run + __shfl_xor(l_run, 1);
    l_tot += __shfl_xor(l_tot, 2);
    if (row >= a.R) return;

    const long long pi = ((long long)h * a.n_split + split) * a.rpad + row;
    if (MODE == F32_STATS) {
        if (sub == 0) {
            a.part_m[pi] = m_run;
            a.part_l[pi] = l_tot;
        }
        return;
    }
    if (a.n_split == 1) {
        const int gl = row / a.B, qi = row - gl * a.B;
        float *dst = a.out + ((long long)qi * a.Hq + (long long)h * a.G + gl) * D + sub * DS;
        const float inv = 1.f / l_tot;
#pragma unroll
        for (int c = 0; c < DS; ++c) dst[c] = o[c] * inv;
        if (a.lse_out && sub == 0)
            a.lse_out[(long long)qi * a.Hq + (long long)h * a.G + gl] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    } else {
        float *dst = a.part_o + pi * D + sub * DS;
#pragma unroll
        for (int c = 0; c < DS; ++c) dst[c] = o[c];
        if (sub == 0) {
            a.part_m[pi] = m_run;
            a.part_l[pi] = l_tot;
        }
    }
}

// Second pass of selection (Eq. 5): alpha[h,j] = 1/(G*B) * sum_rows exp2(score2 - lse2[row]).
// One workgroup owns a slice of keys and walks all row groups itself, so no cross-workgroup
// reduction is needed.
template <int D>
__global__ __launch_bounds__(256) void colsum_f32_kernel(const KernelArgs a)
{
    __shared__ float qs[kF32Rows][D + 1];
    __shared__ float ks[kF32Tile][D + 1];
    __shared__ float ps[kF32Rows][kF32Tile + 1];
    __shared__ float ls[kF32Rows];

    // one grid column per KV head (all G*B rows, Eq. 5), or with head_rows = B per QUERY head (its B rows, Eq. 2)
    const int hy = wg_x(), split = wg_y();
    const bool per_head = a.head_rows > 0;
    const int h = per_head ? hy / a.G : hy;
    const int row_lo = per_head ? (hy % a.G) * a.B : 0;
    const int row_end = per_head ? row_lo + a.head_rows : a.R;
    const int r = tid_x() >> 2, sub = tid_x() & 3;
    const F32Range sr = f32_range(a, split);
    const int row_groups = per_head ? (a.head_rows + kF32Rows - 1) / kF32Rows : a.rpad / kF32Rows;
    const long long stride = (long long)a.Hkv * D;
    const float *kc = static_cast<const float *>(a.kc) + (long long)h * D;

    for (int t = 0; t < sr.cache_tiles; ++t) {
        const long long base = sr.c0 + (long long)t * kF32Tile;
        const long long left = sr.c1 - base;
        const int valid = left < kF32Tile ? (int)left : kF32Tile;
        __syncthreads();
        for (int e = tid_x(); e < kF32Tile * D; e += 256) {
            const int key = e / D, c = e - key * D;
            ks[key][c] = kc[(base + (key < valid ? key : valid - 1)) * stride + c];
        }
        float col = 0.f;      // thread t < 32 accumulates key t over every row group
        for (int rg = 0; rg < row_groups; ++rg) {
            if (rg > 0 || t == 0 || row_groups > 1) {
                __syncthreads();
                f32_load_q<D>(a, h, row_lo + rg * kF32Rows, qs, row_end);
                if (tid_x() < kF32Rows) {
                    const int row = row_lo + rg * kF32Rows + tid_x();
                    ls[tid_x()] = row < row_end ? a.lse2[(long long)h * a.rpad + row] : INFINITY;
                }
            }
            __syncthreads();
            const float lse2 = ls[r];
#pragma unroll
            for (int i = 0; i < kF32Tile / 4; ++i) {
                const int key = sub + 4 * i;
                float acc = 0.f;
#pragma unroll 8
                for (int c = 0; c < D; ++c) acc = fmaf(qs[r][c], ks[key][c], acc);
                ps[r][key] = exp2f(fmaf(acc, a.scale_log2, -lse2));
            }
            __syncthreads();
            if (tid_x() < kF32Tile)
                for (int rr = 0; rr < kF32Rows; ++rr) col += ps[rr][tid_x()];
        }
        if (tid_x() < kF32Tile && (int)tid_x() < valid) a.alpha[(long long)hy * a.L + base + tid_x()] = col * a.inv_rows;
    }
}

hipError_t f32_attn(const KernelArgs &a, int d, int row_groups, bool gather, hipStream_t stream)
{
    dim3 grid(a.Hkv, a.n_split, row_groups), block(256);
    if (d == 128) {
        if (gather) hipLaunchKernelGGL((attn_f32_kernel<128, F32_ATTN, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((attn_f32_kernel<128, F32_ATTN, false>), grid, block, 0, stream, a);
    } else if (d == 64) {
        if (gather) hipLaunchKernelGGL((attn_f32_kernel<64, F32_ATTN, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((attn_f32_kernel<64, F32_ATTN, false>), grid, block, 0, stream, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t f32_stats(const KernelArgs &a, int d, int row_groups, hipStream_t stream)
{
    dim3 grid(a.Hkv, a.n_split, row_groups), block(256);
    if (d == 128) hipLaunchKernelGGL((attn_f32_kernel<128, F32_STATS, false>), grid, block, 0, stream, a);
    else if (d == 64) hipLaunchKernelGGL((attn_f32_kernel<64, F32_STATS, false>), grid, block, 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t f32_colsum(const KernelArgs &a, int d, hipStream_t stream)
{
    dim3 grid(a.head_rows > 0 ? a.Hq : a.Hkv, a.n_split), block(256);
    if (d == 128) hipLaunchKernelGGL((colsum_f32_kernel<128>), grid, block, 0, stream, a);
    else if (d == 64) hipLaunchKernelGGL((colsum_f32_kernel<64>), grid, block, 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace mage
