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

}  // namespace fmtc
