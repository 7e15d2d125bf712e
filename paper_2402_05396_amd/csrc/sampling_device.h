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

// floor(u * n / 2^64) for a 32-bit n: the high word of the 96-bit product.
__device__ __forceinline__ uint32_t mulhi_64x32(uint64_t u, uint32_t n) {
    const uint64_t low = (uint64_t)(uint32_t)u * n;                    // contributes its high word as a carry
    return (uint32_t)(((u >> 32) * n + (low >> 32)) >> 32);
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

// The 64-bit value of the lane a DPP control points at, 0 where there is no such lane or the
// row is masked out: one cross-lane move per half, a few cycles each, no trip through LDS.
// CTRL: 0x110 + n = the lane n places below inside a row of 16 lanes; 0x142 / 0x143 = lane 15 of
// the row below / lane 31, broadcast to a whole row. Every lane of the wave must be active.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ uint64_t dpp_take64(uint64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, ROW_MASK, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), CTRL, ROW_MASK, 0xf, false);
    return ((uint64_t)hi << 32) | lo;
}

// Inclusive prefix sum of one 64-bit value per lane inside a group: four shifted additions
// inside the rows of 16 lanes, then the rows' totals handed on (to rows 1 and 3 for groups of
// 32, and to the upper half for the whole wave). Every lane of the wave must call it.
template <int G> __device__ __forceinline__ uint64_t group_inclusive_scan64(uint64_t v, int /*sub*/) {
    v += dpp_take64<0x111, 0xf>(v);
    v += dpp_take64<0x112, 0xf>(v);
    v += dpp_take64<0x114, 0xf>(v);
    v += dpp_take64<0x118, 0xf>(v);
    if (G >= 32) v += dpp_take64<0x142, 0xa>(v);
    if (G == 64) v += dpp_take64<0x143, 0xc>(v);
    return v;
}

// The 64-bit value of one lane of the wave; `lane` must be the same in every lane.
__device__ __forceinline__ uint64_t wave_get64(uint64_t v, int lane) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// Inclusive prefix sum over the whole wave, and the wave's total in every lane.
__device__ __forceinline__ uint64_t wave_inclusive_scan64(uint64_t v) { return group_inclusive_scan64<64>(v, 0); }
__device__ __forceinline__ uint64_t wave_sum64(uint64_t v) { return wave_get64(wave_inclusive_scan64(v), 63); }

// One of k successive weighted draws without replacement inside a group whose lane i
// holds candidate i: `run` is the inclusive prefix sum of the weights still in play,
// `total` their sum, `w` this lane's weight (below 2^32; 0 once taken), u the 64 random
// bits of this draw. Returns the lane of the first candidate whose running sum exceeds
// floor(u * total / 2^64), or -1 when nothing is left, and takes that candidate out:
// every running sum from its lane on drops by its weight, which is what summing the
// remaining weights again would give. All lanes of the wave must call this; groups
// with `active` false are left untouched.
template <int G>
__device__ __forceinline__ int group_weighted_pick(uint64_t& run, uint64_t& total, uint64_t& w, uint64_t u, bool active,
                                                   int group, int sub) {
    const uint64_t x = __umul64hi(u, total);
    const uint64_t above = group_bits<G>(__ballot(active && run > x), group);
    const int pick = __ffsll((long long)above) - 1;
    const uint64_t taken = group_get<G>((uint32_t)w, pick < 0 ? 0 : pick);   // executed by every lane
    if (active && pick >= 0) {
        if (sub >= pick) run -= taken;
        total -= taken;
        if (sub == pick) w = 0;
    }
    return pick;
}

}  // namespace
