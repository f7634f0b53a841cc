// Direct global -> LDS loads (buffer_load ... lds) and the waits that go with them; shared by the MFMA
// kernels that stream operand tiles through an LDS ring.  Internal, not part of the C ABI.
#pragma once
#include "common.hpp"

namespace d3tom {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// The buffer-resource type and builtins exist in the device pass only; the host pass sees the kernels
// with an empty body (it only needs the launch stub).
#if defined(__HIP_DEVICE_COMPILE__)
// buffer resource over [p, p + bytes), built from values the compiler can see are wave-uniform
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_uniform_rsrc(const void* p, uint32_t bytes) {
    const uint64_t a = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return __builtin_amdgcn_make_buffer_rsrc((void*)(((uint64_t)hi << 32) | lo), 0, (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}
#endif

template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    // N vector-memory operations of this wave may stay in flight (at most 63: the counter has 6 bits);
    // everything older has landed in LDS
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

}  // namespace d3tom
