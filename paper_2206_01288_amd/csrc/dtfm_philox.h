// Counter-based random numbers of the evolutionary search (Sec. 3.4), shared by the kernels that draw
// them. Device code only.
#pragma once

#include <stdint.h>

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds; each round multiplies counter
// words 0 and 2 by the two round multipliers, mixes the high halves with words 1, 3 and the key,
// and the key advances by the two Weyl increments.
struct philox_out {
    uint32_t w[4];
};

__device__ __forceinline__ philox_out philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                    uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int i = 0; i < 10; i++) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    philox_out o;
    o.w[0] = c0;
    o.w[1] = c1;
    o.w[2] = c2;
    o.w[3] = c3;
    return o;
}

enum { STREAM_INIT = 0, STREAM_SELECT = 1, STREAM_CROSSOVER = 2, STREAM_MUTATION = 3 };

__device__ __forceinline__ uint32_t randint(uint32_t x, uint32_t n) { return __umulhi(x, n); }
