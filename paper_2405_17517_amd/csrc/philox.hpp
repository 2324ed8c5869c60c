// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) as a gfx950 device function.
// Ten rounds; each round multiplies counter words 0 and 2 by two fixed odd
// constants, keeps both halves of the 64-bit products and mixes the high halves
// with the other two counter words and the round key; the key advances by two
// Weyl constants per round.  The key is wave-uniform in every caller here, so
// its schedule stays in scalar registers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wash {

struct Words4 {
    uint32_t w0, w1, w2, w3;
};

__device__ __forceinline__ void philox_round(uint32_t &x0, uint32_t &x1, uint32_t &x2, uint32_t &x3,
                                             uint32_t ka, uint32_t kb)
{
    const uint64_t pa = static_cast<uint64_t>(x0) * 0xD2511F53ull;
    const uint64_t pb = static_cast<uint64_t>(x2) * 0xCD9E8D57ull;
    const uint32_t y0 = static_cast<uint32_t>(pb >> 32) ^ x1 ^ ka;
    const uint32_t y2 = static_cast<uint32_t>(pa >> 32) ^ x3 ^ kb;
    x1 = static_cast<uint32_t>(pb);
    x3 = static_cast<uint32_t>(pa);
    x0 = y0;
    x2 = y2;
}

__device__ __forceinline__ Words4 philox4x32_10(uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3,
                                                uint32_t ka, uint32_t kb)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        philox_round(x0, x1, x2, x3, ka, kb);
        ka += 0x9E3779B9u;
        kb += 0xBB67AE85u;
    }
    return Words4{x0, x1, x2, x3};
}

}  // namespace wash
