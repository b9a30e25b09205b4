// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3",
// SC'11) and the three coefficient samplers, evaluated per lane in registers.
//
// Counter = (block, ciphertext index, party, domain | limb << 8 | group << 16);
// key = (seed low word, seed high word).  The key schedule is added after every round.
#pragma once
#include <stdint.h>

#ifndef D2_DEV
#define D2_DEV __device__ __forceinline__
#endif

namespace d2 {

enum : uint32_t {
    DOM_SK = 1, DOM_PK_E = 2, DOM_CRS = 3, DOM_ENC_U = 4, DOM_ENC_E0 = 5, DOM_ENC_E1 = 6,
    DOM_DEC_E = 7, DOM_BENCH = 8,
    // MBFV.Convert: a receiver's own key pair and the randomness of a conversion share (mu, e0, e1
    // consecutive, like the three domains of Encrypt)
    DOM_RSK = 0x10, DOM_RPK_A = 0x11, DOM_RPK_E = 0x12, DOM_CVT_U = 0x13, DOM_CVT_E0 = 0x14, DOM_CVT_E1 = 0x15,
    // MBFV.Bootstrap: mask M_k (uniform mod t), e0, e1 of a share, common polynomial alpha (per limb)
    DOM_BS_M = 0x16, DOM_BS_E0 = 0x17, DOM_BS_E1 = 0x18, DOM_BS_A = 0x19
};

struct PhiloxKey { uint32_t k0, k1; };

struct Block4 { uint32_t w[4]; };

// Each round: two full 32 x 32 -> 64 products (one 64-bit multiply-add instruction each) and four
// exclusive-ors; the round keys are scalar.
D2_DEV Block4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, PhiloxKey key)
{
    uint32_t k0 = key.k0, k1 = key.k1;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        c0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        c1 = (uint32_t)p1;
        c2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c3 = (uint32_t)p0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    Block4 b;
    b.w[0] = c0; b.w[1] = c1; b.w[2] = c2; b.w[3] = c3;
    return b;
}

D2_DEV uint32_t counter_tag(uint32_t domain, uint32_t limb, uint32_t group)
{
    return domain | (limb << 8) | (group << 16);
}

// Ternary values of coefficients 4b..4b+3 from block b: floor(3w / 2^32) - 1.
D2_DEV void ternary4(const Block4 &b, int32_t out[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = (int32_t)__umulhi(b.w[i], 3u) - 1;
}

// Centred-binomial values of coefficients 2b, 2b+1 from block b.
D2_DEV void cbd2(const Block4 &b, uint32_t mask, int32_t out[2])
{
    out[0] = __popc(b.w[0] & mask) - __popc(b.w[1] & mask);
    out[1] = __popc(b.w[2] & mask) - __popc(b.w[3] & mask);
}

}  // namespace d2
