// Modular arithmetic on 64-bit residues for gfx950, built from 32x32->64 multiply-adds
// (v_mad_u64_u32 / v_mul_hi_u32 issue at full rate on CDNA4).
//
// All products have one fixed operand w with a precomputed Shoup quotient
// ws = floor(w * 2^64 / q), so a modular product is one high product, two low products
// and a subtraction.  Butterflies keep values lazily reduced: forward values live in
// [0, 4q), inverse values in [0, 2q) (Harvey's butterflies), which needs q < 2^62; the
// library restricts q < 2^61.
#pragma once
#include <stdint.h>

#ifndef D2_DEV
#define D2_DEV __device__ __forceinline__
#endif

namespace d2 {

struct Tw {          // a fixed multiplicand and its Shoup quotient
    uint64_t w;
    uint64_t ws;
};

// w * y mod q, result in [0, 2q), valid for every 64-bit y.
D2_DEV uint64_t mul_shoup_lazy(uint64_t y, uint64_t w, uint64_t ws, uint64_t q)
{
    uint64_t qhat = __umul64hi(ws, y);
    return w * y - qhat * q;
}

// [0, 2q) -> [0, q)
D2_DEV uint64_t csub(uint64_t x, uint64_t q) { return x >= q ? x - q : x; }

// w * y mod q, canonical.
D2_DEV uint64_t mul_shoup(uint64_t y, uint64_t w, uint64_t ws, uint64_t q)
{
    return csub(mul_shoup_lazy(y, w, ws, q), q);
}

// [0, 4q) -> [0, q)
D2_DEV uint64_t reduce4(uint64_t x, uint64_t q) { return csub(csub(x, 2 * q), q); }

D2_DEV uint64_t add_mod(uint64_t a, uint64_t b, uint64_t q) { return csub(a + b, q); }

// Cooley-Tukey butterfly with lazy reduction: x, y in [0, 4q) -> [0, 4q).
D2_DEV void ct_butterfly(uint64_t &x, uint64_t &y, uint64_t w, uint64_t ws, uint64_t q)
{
    uint64_t two_q = 2 * q;
    uint64_t u = csub(x, two_q);
    uint64_t v = mul_shoup_lazy(y, w, ws, q);
    x = u + v;
    y = u - v + two_q;
}

// Gentleman-Sande butterfly with lazy reduction: x, y in [0, 2q) -> [0, 2q).
D2_DEV void gs_butterfly(uint64_t &x, uint64_t &y, uint64_t w, uint64_t ws, uint64_t q)
{
    uint64_t two_q = 2 * q;
    uint64_t s = x + y;
    uint64_t d = x - y + two_q;
    x = csub(s, two_q);
    y = mul_shoup_lazy(d, w, ws, q);
}

// A small signed value as a residue: v >= 0 ? v : q + v.
D2_DEV uint64_t lift_small(int32_t v, uint64_t q)
{
    return v >= 0 ? (uint64_t)v : q - (uint64_t)(uint32_t)(-v);
}

// floor(w * 2^64 / q) for w < q by binary long division (set-up paths only).
D2_DEV uint64_t shoup_quotient(uint64_t w, uint64_t q)
{
    uint64_t rem = w, quo = 0;
    for (int i = 0; i < 64; ++i) {
        // rem < q < 2^61, so 2*rem cannot overflow
        rem <<= 1;
        quo <<= 1;
        if (rem >= q) { rem -= q; quo |= 1; }
    }
    return quo;
}

}  // namespace d2
