// Small device/host helpers: the negative-sampling counter hash and wavefront utilities.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace legend {

// splitmix64 output function; the hash of a tuple absorbs one field at a time:
// h <- mix64(h + golden + field).
__host__ __device__ inline uint64_t hash_mix64(uint64_t z) {
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__host__ __device__ inline uint64_t hash_fold(uint64_t h, uint64_t field) {
    return hash_mix64(h + 0x9E3779B97F4A7C15ull + field);
}

constexpr int kWave = 64;

__device__ inline int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ inline float wave_shfl_xor(float v, int mask) { return __shfl_xor(v, mask, kWave); }

}  // namespace legend
