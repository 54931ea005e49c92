// Small device helpers shared by the kernel files of libfmtc (wavefront = 64 lanes).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fmtc {

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// exclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t v, int lane) {
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    return incl - v;
}

__device__ __forceinline__ unsigned long long wave_inclusive_scan64(unsigned long long v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        unsigned long long t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    return v;
}

// Words that other workgroups of the same kernel read while it runs go through these: device-scope relaxed
// atomics bypass the caches that are private to a part of the chip, so no fence (a cache write-back here)
// is needed as long as every such word carries its own "valid" mark.
__device__ __forceinline__ void publish64(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long peek64(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One wavefront's 64 x 16 (or 64 x 4) bytes from global memory straight into LDS, lane l to lds_base + 16 l
// (4 l).  Written as assembly because the compiler, which cannot tell the LDS stages apart, would hold every
// later LDS read until all transfers it knows of have landed -- the full latency, in every step; the kernel
// counts its loads in flight itself (s_waitcnt vmcnt, then a barrier) before it reads a stage.
typedef __attribute__((address_space(3))) void lds_void_t;
template <int BYTES>
__device__ __forceinline__ void load_to_lds(const void* src, void* lds_base) {
    const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)(lds_void_t*)lds_base);
    uint32_t keep;
    if constexpr (BYTES == 16)
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep) : "v"(src), "s"(base) : "memory");
    else
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %1, off\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep) : "v"(src), "s"(base) : "memory");
}

// Wait until at most N of this wavefront's loads are in flight (they complete in order); no memory access
// moves across it.  A memory operation the caller's count does not know of (the compiler may add some) can only
// make the wait stricter: issued after the awaited load, it takes one of the N places.
template <int N>
__device__ __forceinline__ void wait_loads() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

}  // namespace fmtc
