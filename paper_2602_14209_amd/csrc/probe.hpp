// Optional timeline probe (compiled out unless MAGE_PROBE is defined): thread 0 of every
// workgroup records the 100 MHz wall clock at a few phase boundaries of a kernel.
#pragma once
#include <hip/hip_runtime.h>

#ifdef MAGE_PROBE
namespace mage {
extern __device__ unsigned long long g_probe[8192 * 8];
}
#define MAGE_PROBE_AT(i)                                                                                           \
    do {                                                                                                           \
        if (threadIdx.x == 0)                                                                                      \
            mage::g_probe[(((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) & 8191) * 8 + (i)] = wall_clock64(); \
    } while (0)
// the same for the first lane of the LAST wavefront, slots 8 workgroups further on
#define MAGE_PROBE_LAST_AT(i)                                                                                      \
    do {                                                                                                           \
        if (threadIdx.x == blockDim.x - 64)                                                                        \
            mage::g_probe[((((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) & 4095) + 4096) * 8 + (i)] = wall_clock64(); \
    } while (0)
#else
#define MAGE_PROBE_AT(i) do { } while (0)
#define MAGE_PROBE_LAST_AT(i) do { } while (0)
#endif
