// Hand-over of data between workgroups of one launch without a cache write-back fence and without anybody
// waiting for anybody.  The producers store with device-scope stores (written through to memory), every
// wavefront waits for its own stores to complete (a workgroup-scope release fence), the workgroup meets at a
// barrier and then counts itself in with one device-scope atomic add on an arrival counter; the workgroup that
// completes the count reads the data back with device-scope loads (buffer loads carrying the device-scope bit,
// so that several can be in flight), every other workgroup simply ends.  The counter is reset by the workgroup
// that completes it, so counters are zero between launches.
#pragma once
#include "common.hpp"

namespace asx {

__device__ __forceinline__ void st_dev(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(int32_t* p, int32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t dev_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ uint32_t ld_dev(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off) {
  return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, byte_off, 0, 16 /* device scope */);
}

// Called by every thread of the workgroup after its device-scope stores.  True (for every thread) in the one
// workgroup that completes the count of `expected` arrivals on *ctr.  flag_sh: one word of LDS.
__device__ __forceinline__ bool arrive_last(int32_t* ctr, int expected, int* flag_sh) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // this wavefront's device-scope stores have completed
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = old == expected - 1;
    if (last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag_sh = last;
  }
  __syncthreads();
  return *flag_sh != 0;
}

}  // namespace asx
