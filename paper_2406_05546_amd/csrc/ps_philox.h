// Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11), device side.
// Each of the 10 rounds multiplies counter words 0 and 2 by fixed odd constants, routes the high
// and low halves, and mixes in the key, which advances by two Weyl constants per round.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ps {

__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32 x 32 -> 64 bit multiply per product (the integer multiplier runs at a quarter of the
        // vector rate, so a separate high and low multiply would cost twice as much)
        const uint64_t p0 = (uint64_t)M0 * c.x, p1 = (uint64_t)M1 * c.z;
        c = make_uint4((uint32_t)(p1 >> 32) ^ c.y ^ k.x, (uint32_t)p1, (uint32_t)(p0 >> 32) ^ c.w ^ k.y, (uint32_t)p0);
        k.x += W0;
        k.y += W1;
    }
    return c;
}

}  // namespace ps
