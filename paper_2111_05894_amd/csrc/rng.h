// Counter-based random numbers of the sampler: Philox4x32 with 10 rounds
// (Salmon, Moraes, Dror, Shaw, SC'11).  The paper asks only for a uniformly
// random choice of neighbours (Sec. 2.2); a counter-based generator makes each
// draw a pure function of (seed, node, draw, hop), whatever thread computes it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tier {

constexpr uint32_t kTagNeighbour = 1;   // counter word 3 of a neighbour draw
constexpr uint32_t kTagBatch = 2;       // counter word 3 of a mini-batch seed

__host__ __device__ inline void mul_wide(uint32_t a, uint32_t b, uint32_t &hi, uint32_t &lo)
{
#if defined(__HIP_DEVICE_COMPILE__)
    hi = __umulhi(a, b);
    lo = a * b;
#else
    uint64_t p = (uint64_t)a * (uint64_t)b;
    hi = (uint32_t)(p >> 32);
    lo = (uint32_t)p;
#endif
}

// 64 bits (block words 1:0) for counter (c0, c1, c2, c3) under key (k0, k1).
__host__ __device__ inline uint64_t philox_r64(uint32_t k0, uint32_t k1,
                                               uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t h0, l0, h1, l1;
        mul_wide(0xD2511F53u, c0, h0, l0);
        mul_wide(0xCD9E8D57u, c2, h1, l1);
        uint32_t y0 = h1 ^ c1 ^ k0, y2 = h0 ^ c3 ^ k1;
        c0 = y0; c1 = l1; c2 = y2; c3 = l0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return ((uint64_t)c1 << 32) | (uint64_t)c0;
}

}  // namespace tier
