// Workgroup and work-item indices read straight from the registers the hardware sets up.
//
// HIP's blockIdx / threadIdx / gridDim go through device-library functions (__ockl_get_group_id and
// friends).  Those are normally inlined away, but LLVM does not inline a callee whose target features
// are not a subset of the caller's, and these sources are compiled with the packed-fp32 feature
// switched off while the device library has it on.  Every use then becomes a real call at the top of
// the kernel -- up to 260 instructions with a switch over the dimension, four of them in a row in the
// sparse-step kernel, about 1.4 us of a launch that takes under 10.  The builtins below are plain
// register reads.
#pragma once
#include <hip/hip_runtime.h>

namespace mage {

__device__ __forceinline__ unsigned wg_x() { return __builtin_amdgcn_workgroup_id_x(); }
__device__ __forceinline__ unsigned wg_y() { return __builtin_amdgcn_workgroup_id_y(); }
__device__ __forceinline__ unsigned wg_z() { return __builtin_amdgcn_workgroup_id_z(); }
__device__ __forceinline__ unsigned tid_x() { return __builtin_amdgcn_workitem_id_x(); }

}  // namespace mage
