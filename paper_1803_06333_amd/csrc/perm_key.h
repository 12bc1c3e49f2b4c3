// The counter-based key of the epoch order (Section 3.2: "32-bit pseudo-random numbers", xorshift):
// a 64-bit integer mix of (seed, chunk, c) folded to a non-zero 32-bit state, then four rounds of
// the (13,17,5) xorshift.  Usable on the host (order of the groups) and on the device (keys).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace snap {

__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// 64-bit integer mix of (seed, chunk, c) folded to a non-zero 32-bit state, then four rounds of
// the (13,17,5) xorshift.
__host__ __device__ __forceinline__ uint32_t perm_key(uint64_t seed_chunk_mix, uint32_t c) {
    uint64_t z = mix64(seed_chunk_mix + (uint64_t)c * 0x9E3779B97F4A7C15ull);
    uint32_t x = (uint32_t)(z ^ (z >> 32));
    if (x == 0u) x = 0x6C078965u;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        x ^= x << 13;
        x ^= x >> 17;
        x ^= x << 5;
    }
    return x;
}


__host__ __device__ __forceinline__ uint64_t perm_key_base(uint64_t seed, uint32_t chunk) {
    return mix64(seed ^ mix64((uint64_t)chunk + 0x632BE59BD9B4E019ull));
}

constexpr uint32_t GROUP_ORDER_CHUNK = 0xFFFFFFFFu;   // chunk id under which the order of the groups is drawn

}  // namespace snap
