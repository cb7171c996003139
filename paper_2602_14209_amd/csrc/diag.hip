// Measurement aids of the MAGE library (gfx950): the floors and ceilings that the benchmark prints
// beside the attention kernels' figures.  None of them is part of the method; they exist so that a
// reader of the benchmark line can tell a latency-bound launch from a bandwidth-bound one:
//   empty    one kernel that does nothing           -> cost of a launch slot inside a stream / HIP graph
//   stamp    one lane stores the device's wall clock -> time between two points INSIDE a HIP graph, where no
//            host-side event can be placed (which phase of a captured chain the time goes to)
//   chase    one lane following a chain of loads    -> latency of one dependent memory round trip
//   read     every CU streaming 16-byte loads       -> read bandwidth this GPU reaches
//   copy     the same with a store per load         -> copy bandwidth (read + write)
//   merge    four workgroups hand 8 KB each to the last of them to arrive -> what merging partial results
//            ACROSS workgroups inside one launch would cost (with a device-scope fence, and without one)
//   gather   the sparse step's memory accesses only -> rate at which 2*Hkv*k scattered rows of d elements
//            (index entry, then row) can be fetched at all, with no attention arithmetic behind them
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mage.h"
#include "ids.hpp"

namespace mage {

typedef unsigned v4u __attribute__((ext_vector_type(4)));   // 16 bytes, a type the nontemporal builtins take

__global__ void diag_empty_kernel() {}

// the constant-rate device clock (not the shader clock), stored with an ordinary vector store
__global__ __launch_bounds__(64) void diag_stamp_kernel(unsigned long long *out)
{
    if (tid_x() == 0) *out = wall_clock64();
}

// chain[i] = index of the next entry; lane 0 of one wavefront walks n_hops dependent loads from `start`
__global__ __launch_bounds__(64) void diag_chase_kernel(const int32_t *__restrict__ chain, int start, int n_hops, int32_t *out)
{
    if (tid_x() != 0) return;
    int i = start;
    for (int h = 0; h < n_hops; ++h) i = __builtin_nontemporal_load(chain + i);
    *out = i;
}

constexpr int kDiagThreads = 256;
constexpr int kDiagUnroll = 8;      // 16-byte loads in flight per lane

// grid-stride streaming read; the xor of everything read goes to sink[workgroup] so the loads stay
__global__ __launch_bounds__(kDiagThreads) void diag_read_kernel(const v4u *__restrict__ src, size_t n16, uint32_t *sink, int n_wg)
{
    const size_t stride = (size_t)n_wg * kDiagThreads;     // n_wg = workgroups launched
    size_t i = (size_t)wg_x() * kDiagThreads + tid_x();
    v4u acc = {0u, 0u, 0u, 0u};
    for (; i + (kDiagUnroll - 1) * stride < n16; i += kDiagUnroll * stride) {
        v4u v[kDiagUnroll];
#pragma unroll
        for (int u = 0; u < kDiagUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < kDiagUnroll; ++u) {
            acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w;
        }
    }
    for (; i < n16; i += stride) {
        const v4u v = __builtin_nontemporal_load(src + i);
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    const uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) sink[wg_x()] = r;      // practically never true: the compiler cannot drop the loads
}

__global__ __launch_bounds__(kDiagThreads) void diag_copy_kernel(v4u *__restrict__ dst, const v4u *__restrict__ src, size_t n16, int n_wg)
{
    const size_t stride = (size_t)n_wg * kDiagThreads;     // n_wg = workgroups launched
    size_t i = (size_t)wg_x() * kDiagThreads + tid_x();
    for (; i + (kDiagUnroll - 1) * stride < n16; i += kDiagUnroll * stride) {
        v4u v[kDiagUnroll];
#pragma unroll
        for (int u = 0; u < kDiagUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < kDiagUnroll; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

// The memory accesses of a (batched) sparse step and nothing else: for every sequence z and KV head
// h the k rows idx[z,h,:] of the K and of the V cache, each row read once in 16-byte pieces by
// row_bytes/16 consecutive lanes.  One wavefront handles kGatherLoads wavefront-wide loads of each cache.
constexpr int kGatherLoads = 4;
__global__ __launch_bounds__(kDiagThreads) void diag_gather_kernel(const unsigned char *__restrict__ kc, const unsigned char *__restrict__ vc,
                                                                   const int32_t *__restrict__ idx, int Hkv, int k, long long L, int row_bytes,
                                                                   uint32_t *sink)
{
    const int lanes_per_row = row_bytes / 16;                 // 16 at d = 128 bf16
    const int rows_per_load = 64 / lanes_per_row;             // rows one wavefront-wide load covers
    const int lane = tid_x() & 63, wave = tid_x() >> 6;
    const int z = wg_z(), h = wg_y();
    const int e0 = (wg_x() * (kDiagThreads / 64) + wave) * kGatherLoads * rows_per_load;
    if (e0 >= k) return;
    const int32_t *ix = idx + ((long long)z * Hkv + h) * k;
    const long long seq = (long long)z * L * Hkv * row_bytes;
    const long long stride = (long long)Hkv * row_bytes;
    int row[kGatherLoads];
#pragma unroll
    for (int n = 0; n < kGatherLoads; ++n) {
        const int e = e0 + n * rows_per_load + lane / lanes_per_row;
        row[n] = ix[e < k ? e : k - 1];                        // a ragged tail re-reads the last row
    }
    v4u v[2 * kGatherLoads];
#pragma unroll
    for (int n = 0; n < kGatherLoads; ++n) {
        const long long off = seq + (long long)row[n] * stride + (long long)h * row_bytes + (lane % lanes_per_row) * 16;
        v[2 * n] = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(kc + off));
        v[2 * n + 1] = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(vc + off));
    }
    v4u acc = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 2 * kGatherLoads; ++j) {
        acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w;
    }
    const uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) sink[0] = r;
}

// Cross-workgroup merge protocol: every workgroup writes an 8 KB partial; the last of each group of four
// to arrive (a counter that keeps counting: no reset between launches) adds the four partials up.
//   MODE 0: partials only, written through (sc1), nobody merges
//   MODE 1: plain stores, __threadfence() (device-scope release), counter, __threadfence() (acquire), plain loads
//   MODE 2: no fence instruction: partials written and read with device-scope accesses (sc1, which bypass
//           the per-XCD L2), the writer waits for its stores to complete before it touches the counter
template <int MODE>
__global__ __launch_bounds__(512) void diag_merge_kernel(float *part, unsigned *cnt, float *out, const float *src)
{
    const int wg = wg_x(), grp = wg / 4, t = tid_x();
    float4 v = reinterpret_cast<const float4 *>(src)[(size_t)wg * 512 + t];
    v.x += 1.f;
    float *my = part + (size_t)wg * 2048 + t * 4;
    if (MODE == 1) {
        *reinterpret_cast<float4 *>(my) = v;
    } else {
        __hip_atomic_store(my + 0, v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(my + 1, v.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(my + 2, v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(my + 3, v.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (MODE == 0) return;
    __shared__ unsigned arrival;
    if (MODE == 1) __threadfence();
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (t == 0) arrival = __hip_atomic_fetch_add(cnt + grp, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if ((arrival & 3u) != 3u) return;
    if (MODE == 1) __threadfence();
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int w = 0; w < 4; ++w) {
        const float *p = part + (size_t)(grp * 4 + w) * 2048 + t * 4;
        float4 x;
        if (MODE == 1) {
            x = *reinterpret_cast<const float4 *>(p);
        } else {
            x.x = __hip_atomic_load(p + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            x.y = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            x.z = __hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            x.w = __hip_atomic_load(p + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    reinterpret_cast<float4 *>(out)[(size_t)grp * 512 + t] = acc;
}

}  // namespace mage

using namespace mage;

extern "C" {

int mage_diag_empty(void *hip_stream)
{
    hipLaunchKernelGGL(diag_empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream));
    return hipGetLastError() == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

int mage_diag_stamp(uint64_t *out, void *hip_stream)
{
    if (!out) return MAGE_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(out) & 7u) return MAGE_ERR_ALIGN;
    hipLaunchKernelGGL(diag_stamp_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<unsigned long long *>(out));
    return hipGetLastError() == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

int64_t mage_diag_stamp_hz(void)
{
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return 0;
    return (int64_t)khz * 1000;
}

int mage_diag_chase(const int32_t *chain, int64_t n_entries, int start, int n_hops, int32_t *out, void *hip_stream)
{
    if (!chain || !out) return MAGE_ERR_NULL;
    if (n_entries <= 0 || n_entries > ((int64_t)1 << 31) - 1 || start < 0 || start >= n_entries || n_hops <= 0) return MAGE_ERR_SHAPE;
    hipLaunchKernelGGL(diag_chase_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream), chain, start, n_hops, out);
    return hipGetLastError() == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

static int diag_grid(size_t n16)
{
    const size_t want = (n16 + kDiagThreads - 1) / kDiagThreads;
    const size_t cap = 256 * 16;                              // 16 workgroups of 4 wavefronts per CU
    return (int)(want < cap ? (want ? want : 1) : cap);
}

int mage_diag_read(const void *src, size_t bytes, uint32_t *sink, void *hip_stream)
{
    if (!src || !sink) return MAGE_ERR_NULL;
    if (bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15u)) return bytes < 16 ? MAGE_ERR_SHAPE : MAGE_ERR_ALIGN;
    const size_t n16 = bytes / 16;
    const int n_wg = diag_grid(n16);
    hipLaunchKernelGGL(diag_read_kernel, dim3(n_wg), dim3(kDiagThreads), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const v4u *>(src), n16, sink, n_wg);
    return hipGetLastError() == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

int mage_diag_copy(void *dst, const void *src, size_t bytes, void *hip_stream)
{
    if (!src || !dst) return MAGE_ERR_NULL;
    if (bytes < 16) return MAGE_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return MAGE_ERR_ALIGN;
    const size_t n16 = bytes / 16;
    const int n_wg = diag_grid(n16);
    hipLaunchKernelGGL(diag_copy_kernel, dim3(n_wg), dim3(kDiagThreads), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<v4u *>(dst), static_cast<const v4u *>(src), n16, n_wg);
    return hipGetLastError() == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

int mage_diag_merge(int mode, int n_groups, float *part, unsigned *counters, float *out, const float *src, void *hip_stream)
{
    if (!part || !counters || !out || !src) return MAGE_ERR_NULL;
    if (n_groups <= 0 || n_groups > (1 << 16) || mode < 0 || mode > 2) return MAGE_ERR_SHAPE;
    if (((reinterpret_cast<uintptr_t>(part) | reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(src)) & 15u)) return MAGE_ERR_ALIGN;
    dim3 grid(4 * n_groups), block(512);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (mode == 0) hipLaunchKernelGGL(diag_merge_kernel<0>, grid, block, 0, s, part, counters, out, src);
    else if (mode == 1) hipLaunchKernelGGL(diag_merge_kernel<1>, grid, block, 0, s, part, counters, out, src);
    else hipLaunchKernelGGL(diag_merge_kernel<2>, grid, block, 0, s, part, counters, out, src);
    return hipGetLastError() == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

int mage_diag_gather(const mage_shape *shape, int n_seq, const void *k_cache, const void *v_cache, const int32_t *idx,
                     uint32_t *sink, void *hip_stream)
{
    if (!shape || !k_cache || !v_cache || !idx || !sink) return MAGE_ERR_NULL;
    if (shape->Hkv <= 0 || shape->d <= 0 || shape->L <= 0 || shape->k <= 0 || shape->k > shape->L || n_seq <= 0 || n_seq > 65535)
        return MAGE_ERR_SHAPE;
    const int esz = shape->dtype == MAGE_BF16 ? 2 : 4;
    const int row_bytes = shape->d * esz;
    if ((shape->dtype != MAGE_BF16 && shape->dtype != MAGE_F32) || row_bytes % 16 != 0 || row_bytes > 256 || 64 % (row_bytes / 16) != 0)
        return MAGE_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(k_cache) & 15u) || (reinterpret_cast<uintptr_t>(v_cache) & 15u)) return MAGE_ERR_ALIGN;
    const int per_wg = (kDiagThreads / 64) * kGatherLoads * (64 / (row_bytes / 16));
    dim3 grid((shape->k + per_wg - 1) / per_wg, shape->Hkv, n_seq);
    hipLaunchKernelGGL(diag_gather_kernel, grid, dim3(kDiagThreads), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const unsigned char *>(k_cache), static_cast<const unsigned char *>(v_cache), idx,
                       shape->Hkv, shape->k, (long long)shape->L, row_bytes, sink);
    return hipGetLastError() == hipSuccess ? MAGE_OK : MAGE_ERR_HIP;
}

}  // extern "C"
