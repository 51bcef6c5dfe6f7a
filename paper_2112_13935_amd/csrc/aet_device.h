// Device-side helpers used by every kernel file: the counter hash behind the sample
// indices and wave-level reductions for 64-wide wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aet {

// SplitMix64 (Steele, Lea, Flood, OOPSLA 2014): value number `ctr` of the stream with
// state `key` is mix(key + (ctr + 1) * golden_gamma).
__host__ __device__ __forceinline__ uint64_t splitmix_mix(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
__host__ __device__ __forceinline__ uint64_t splitmix_at(uint64_t key, uint64_t ctr) {
    return splitmix_mix(key + (ctr + 1) * 0x9E3779B97F4A7C15ULL);
}
// Algorithm 2, sampling step: the row that sample counter q selects, by multiply-shift of the hash's top 32 bits onto [0, n_samples).
__host__ __device__ __forceinline__ uint32_t sample_row(uint64_t key, uint64_t q, uint32_t n_samples) {
    const uint64_t h = splitmix_at(key, q);
    return (uint32_t)(((h >> 32) * (uint64_t)n_samples) >> 32);
}

// Pointers that kernels read out of a parameter record in memory are "flat" to the
// compiler; these casts tell it they point to global memory, so that it emits global_*
// instead of flat_* accesses (flat accesses also count against the LDS wait counter and
// serialise with LDS traffic).
typedef const float __attribute__((address_space(1))) *gcf_ptr;
typedef float __attribute__((address_space(1))) *gf_ptr;
typedef const int32_t __attribute__((address_space(1))) *gci_ptr;
__device__ __forceinline__ gcf_ptr as_global(const float *p) { return (gcf_ptr)p; }
__device__ __forceinline__ gf_ptr as_global(float *p) { return (gf_ptr)p; }
__device__ __forceinline__ gci_ptr as_global(const int32_t *p) { return (gci_ptr)p; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

}  // namespace aet
