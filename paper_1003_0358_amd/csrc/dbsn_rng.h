// Counter-based random numbers of libdbsn (device and host).
//
// The paper names no generator.  This library defines one so that results depend on
// (seed, stream, counter) only, never on launch shape or chunking:
//   mix(z)          SplitMix64's output function (Steele, Lea, Flood, OOPSLA 2014)
//   key(seed, s)  = mix(seed + (s + 1) * GOLD)
//   draw(key, c)  = mix(key  + (c + 1) * GOLD)
//   unit(r)       = (int(r >> 40) - 2^23) * 2^-23      in [-1, 1), exact in binary32
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dbsn {

__host__ __device__ inline uint64_t rng_mix(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__host__ __device__ inline uint64_t rng_key(uint64_t seed, uint64_t stream) {
    return rng_mix(seed + (stream + 1ull) * 0x9E3779B97F4A7C15ull);
}
__host__ __device__ inline uint64_t rng_draw(uint64_t key, uint64_t counter) {
    return rng_mix(key + (counter + 1ull) * 0x9E3779B97F4A7C15ull);
}
// signed 24-bit integer of a draw, -2^23 .. 2^23 - 1
__host__ __device__ inline int32_t rng_i24(uint64_t r) { return (int32_t)(r >> 40) - (1 << 23); }
__host__ __device__ inline float rng_unit(uint64_t r) { return (float)rng_i24(r) * (1.0f / 8388608.0f); }

}  // namespace dbsn
