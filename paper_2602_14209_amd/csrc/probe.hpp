// Optional timeline probe (compiled out unless MAGE_PROBE is defined): the first lane of the first
// and of the last wavefront of every workgroup read the 100 MHz wall clock at a few phase boundaries
// of a kernel into registers and write them out together at the end, so that probing adds no memory
// traffic in the middle of the kernel.
#pragma once
#include <hip/hip_runtime.h>

#ifdef MAGE_PROBE
namespace mage {
extern __device__ unsigned long long g_probe[8192 * 8];
}
#define MAGE_PROBE_DECL unsigned long long mage_probe_t[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define MAGE_PROBE_AT(i) mage_probe_t[(i)] = wall_clock64()
#define MAGE_PROBE_LAST_AT(i) MAGE_PROBE_AT(i)
#define MAGE_PROBE_FLUSH()                                                                                        \
    do {                                                                                                          \
        const unsigned wg = ((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) & 4095;             \
        if (threadIdx.x == 0)                                                                                     \
            for (int i_ = 0; i_ < 8; ++i_) mage::g_probe[wg * 8 + i_] = mage_probe_t[i_];                         \
        if (threadIdx.x == blockDim.x - 64)                                                                       \
            for (int i_ = 0; i_ < 8; ++i_) mage::g_probe[(wg + 4096) * 8 + i_] = mage_probe_t[i_];                \
    } while (0)
#else
#define MAGE_PROBE_DECL do { } while (0)
#define MAGE_PROBE_AT(i) do { } while (0)
#define MAGE_PROBE_LAST_AT(i) do { } while (0)
#define MAGE_PROBE_FLUSH() do { } while (0)
#endif
