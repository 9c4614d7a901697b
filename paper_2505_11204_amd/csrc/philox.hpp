// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) for host and device code of
// the GPU library.  The paper fixes only seeds (App. "Default Experimental
// Setup"); a counter-based generator lets any (seed, layer, column) sign and any
// (seed, group, position) sort key be produced independently, with nothing stored.
#pragma once
#include <stdint.h>

#if defined(__HIP__)
#define RANDES_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define RANDES_HD inline
#endif

namespace randes {

struct u32x4_t { uint32_t w[4]; };

RANDES_HD uint32_t mulhi32(uint32_t a, uint32_t b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(a, b);
#else
    return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32);
#endif
}

// Ten rounds; the round key advances by the two Weyl increments.
RANDES_HD u32x4_t philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                uint32_t k0, uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t h0 = mulhi32(M0, c0), l0 = M0 * c0;
        const uint32_t h1 = mulhi32(M1, c2), l1 = M1 * c2;
        c0 = h1 ^ c1 ^ k0;
        c1 = l1;
        c2 = h0 ^ c3 ^ k1;
        c3 = l0;
        k0 += W0;
        k1 += W1;
    }
    u32x4_t o;
    o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
    return o;
}

// Stream ids in counter word 2 keep the sign and permutation streams apart.
constexpr uint32_t STREAM_SIGN = 0u;
constexpr uint32_t STREAM_PERM = 1u;

// The 128 sign bits of columns [128*block, 128*block + 128) of slot `layer`.
RANDES_HD u32x4_t sign_block(uint32_t key_lo, uint32_t key_hi, uint32_t layer, uint32_t block)
{
    return philox4x32_10(block, layer, STREAM_SIGN, 0u, key_lo, key_hi);
}

}  // namespace randes
