// Philox4x32-R (Salmon, Moraes, Dror, Shaw 2011), the counter-based generator behind every exponential of a race:
// the words are a function of (counter, key) alone, so the draft race, the target race and the comparison method
// regenerate them wherever they are needed and none is ever stored.  Device code for gfx950; included by both
// kernel sources of the library.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ersd_philox {

#ifndef ERSD_PHILOX_ROUNDS
#define ERSD_PHILOX_ROUNDS 7
#endif
constexpr int kPhiloxRounds = ERSD_PHILOX_ROUNDS;   // 7 by default; 10 is the generator's standard strength
constexpr uint32_t kPhiloxM0 = 0xD2511F53u, kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u, kPhiloxW1 = 0xBB67AE85u;

__device__ __forceinline__ void philox4x32(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < kPhiloxRounds; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        uint32_t n0, n2;
        if (r >= 2) {  // gfx950's three-input bitwise operation (truth table 0x96 = a ^ b ^ c): one instruction each
            n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
            n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
        } else {       // in the first two rounds most operands are wavefront-uniform: left to the scalar unit
            n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
            n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        }
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

}  // namespace ersd_philox
