// Device helpers shared by the sampling kernels: the counter-based random
// generator and the lane-group primitives. Internal header; every translation
// unit that includes it gets its own copy.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// ---- Philox4x32-10 (Salmon et al., SC'11) --------------------------------
__device__ __forceinline__ void philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
    const uint32_t lo0 = 0xD2511F53u * c[0], hi0 = __umulhi(0xD2511F53u, c[0]);
    const uint32_t lo1 = 0xCD9E8D57u * c[2], hi1 = __umulhi(0xCD9E8D57u, c[2]);
    const uint32_t a = hi1 ^ c[1] ^ k0;
    const uint32_t b = hi0 ^ c[3] ^ k1;
    c[0] = a; c[1] = lo1; c[2] = b; c[3] = lo0;
}

// 64 random bits for (seed, hop, root index, slot).
__device__ __forceinline__ uint64_t draw64(uint32_t seed_lo, uint32_t seed_hi, uint32_t hop,
                                           uint64_t root, uint32_t slot) {
    uint32_t c[4] = {(uint32_t)root, (uint32_t)(root >> 32), slot, hop};
    uint32_t k0 = seed_lo, k1 = seed_hi;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        philox_round(c, k0, k1);
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return ((uint64_t)c[1] << 32) | c[0];
}

// ---- group helpers ---------------------------------------------------------
// A wavefront is split into 64/G groups of G consecutive lanes (G = 16, 32 or
// 64), one root per group. `sub` is a lane's index inside its group.
template <int G> __device__ __forceinline__ uint64_t group_bits(uint64_t wave_ballot, int group) {
    if (G == 64) return wave_ballot;
    return (wave_ballot >> (group * G)) & (((uint64_t)1 << G) - 1);
}
template <int G> __device__ __forceinline__ uint32_t group_get(uint32_t v, int sub_lane) {
    return (uint32_t)__shfl((int)v, sub_lane, G);
}
template <int G> __device__ __forceinline__ uint64_t group_get64(uint64_t v, int sub_lane) {
    return ((uint64_t)group_get<G>((uint32_t)(v >> 32), sub_lane) << 32) | group_get<G>((uint32_t)v, sub_lane);
}

}  // namespace
