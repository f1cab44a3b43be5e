// Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11)
// and the per-node draw stream of the sampler.
#pragma once
#include "common.hpp"

namespace helios {

struct Philox4 { uint32_t w0, w1, w2, w3; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    return Philox4{c0, c1, c2, c3};
}

// k-th 64-bit draw of (rng_seed, hop, node): block k/2 of the counter
// (node, block, hop, tag); even k takes words 0,1, odd k words 2,3.
__device__ __forceinline__ uint64_t node_draw(uint64_t rng_seed, int32_t node, int32_t hop, uint32_t k) {
    const Philox4 b = philox4x32_10(static_cast<uint32_t>(node), k >> 1, static_cast<uint32_t>(hop),
                                    0x48454C49u, static_cast<uint32_t>(rng_seed),
                                    static_cast<uint32_t>(rng_seed >> 32));
    const uint32_t lo = (k & 1u) ? b.w2 : b.w0;
    const uint32_t hi = (k & 1u) ? b.w3 : b.w1;
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

// draw -> [0, n) by the high half of the 128-bit product
__device__ __forceinline__ uint64_t bounded(uint64_t x, uint64_t n) { return __umul64hi(x, n); }

}  // namespace helios
