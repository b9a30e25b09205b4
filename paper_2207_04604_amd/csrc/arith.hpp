// Modular arithmetic back-ends ("policies") for the transform engine on gfx950.
//
// On CDNA4 v_mad_u64_u32, v_mul_lo/hi_u32, v_lshl_add_u64 and v_fma_f64 all issue at full
// rate, so the cost of a butterfly is its instruction count.  Three formulations, chosen
// per context from the size of the largest modulus:
//
//   ArithF  (moduli < 2^44)  residues as signed doubles.  w*y mod q from an error-free
//           product (mul + fma), one rounded quotient and one fma: 6 instructions, result
//           in about (-q/2, q/2); butterflies add and subtract without any correction.
//   ArithS  (moduli < 2^55)  64-bit integers, Shoup quotient ws = floor(w 2^63 / q).  The
//           quotient estimate drops the low x low partial product (error <= 2), so the
//           product lands in [0, 4q); values grow by at most 4q per forward stage and are
//           never corrected inside a forward transform (65 q < 2^62).
//   ArithB  (moduli < 2^61)  64-bit integers, exact 63-bit Shoup quotient, Harvey's lazy
//           butterflies: forward values in [0, 4q), inverse values in [0, 2q).
//   Arith32 (moduli < 2^30)  32-bit residues (one register and one 4-byte LDS word per
//           coefficient), 32-bit Shoup quotient ws = floor(w 2^32 / q), Harvey's lazy butterflies
//           in 8 instructions.  Used for whole contexts whose primes are below 2^30 and, in every
//           context, for the transforms modulo the plaintext modulus t.
//
// Table entries (twiddles, per-modulus constants) are {w, floor(w 2^63 / q)} for the integer
// policies and {bits of the double w, unused} for ArithF.  Prepared keys cross the library
// boundary as values plus 64-bit quotients floor(v 2^64 / q); the integer policies shift
// those right by one, ArithF converts the value and ignores the quotient.
#pragma once
#include <stdint.h>

#ifndef D2_DEV
#define D2_DEV __device__ __forceinline__
#endif

#pragma clang fp contract(off)

namespace d2 {

struct Tw {          // 16-byte table entry: a fixed multiplicand and its companion word
    uint64_t w;
    uint64_t ws;
};

D2_DEV uint32_t lo32(uint64_t v) { return (uint32_t)v; }
D2_DEV uint32_t hi32(uint64_t v) { return (uint32_t)(v >> 32); }
D2_DEV uint64_t mul32(uint32_t a, uint32_t b) { return (uint64_t)a * b; }

// The hot sequences are pinned with inline assembly on the device: the compiler's own
// selection for the same C spends about 40 % more VALU slots (zero-extension moves, a compare
// in front of every conditional subtraction, 32-bit multiplies split off the 64-bit
// multiply-adds).  The plain C next to each block states what it computes and is what a
// host build of this header runs.
#if defined(__HIP_DEVICE_COMPILE__)
#define D2_GCN_ASM 1
#else
#define D2_GCN_ASM 0
#endif

// x >= m ? x - m : x   (unsigned): subtract, then select on the borrow
D2_DEV uint64_t csub(uint64_t x, uint64_t m)
{
#if D2_GCN_ASM
    uint32_t dlo, dhi;
    const uint32_t xlo = lo32(x), xhi = hi32(x), mlo = lo32(m), mhi = hi32(m);
    asm("v_sub_co_u32 %0, vcc, %2, %4\n\t"
        "v_subb_co_u32 %1, vcc, %3, %5, vcc\n\t"
        "v_cndmask_b32 %0, %0, %2, vcc\n\t"
        "v_cndmask_b32 %1, %1, %3, vcc"
        : "=&v"(dlo), "=&v"(dhi)
        : "v"(xlo), "v"(xhi), "v"(mlo), "v"(mhi)
        : "vcc");
    return ((uint64_t)dhi << 32) | dlo;
#else
    uint64_t d = x - m;
    return x < m ? x : d;
#endif
}

// ---------------------------------------------------------------------------------------
// Global memory access.
//   Per-lane: raw buffer instructions -- a wave-uniform base (descriptor in SGPRs) plus one 32-bit
//   per-lane byte offset and a uniform offset.  Plain 64-bit addressing would hold a VGPR pair per
//   array and slot, and generic pointers become flat instructions, whose completion is counted
//   together with LDS traffic.  The ranges are < 4 GB from the base.
//   Wave-uniform table reads: through the constant address space, which the compiler turns into
//   scalar loads (results in SGPRs) when it can see that the offset is uniform.
// ---------------------------------------------------------------------------------------
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
struct U128 {
    uint64_t lo, hi;
};
D2_DEV uint64_t ld64(const void *base, uint32_t lane_off, uint32_t slot_off)
{
#if D2_GCN_ASM
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, 0xffffffff, 0x00020000);
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, lane_off, slot_off, 0);
    return ((uint64_t)v.y << 32) | v.x;
#else
    return *(const uint64_t *)((const char *)base + lane_off + slot_off);
#endif
}
D2_DEV U128 ld128(const void *base, uint32_t lane_off, uint32_t slot_off)
{
#if D2_GCN_ASM
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, 0xffffffff, 0x00020000);
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, slot_off, 0);
    return U128{((uint64_t)v.y << 32) | v.x, ((uint64_t)v.w << 32) | v.z};
#else
    const uint64_t *p = (const uint64_t *)((const char *)base + lane_off + slot_off);
    return U128{p[0], p[1]};
#endif
}
D2_DEV void st64(void *base, uint32_t lane_off, uint32_t slot_off, uint64_t val)
{
#if D2_GCN_ASM
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(base, 0, 0xffffffff, 0x00020000);
    u32x2 v;
    v.x = (uint32_t)val;
    v.y = (uint32_t)(val >> 32);
    __builtin_amdgcn_raw_buffer_store_b64(v, r, lane_off, slot_off, 0);
#else
    *(uint64_t *)((char *)base + lane_off + slot_off) = val;
#endif
}
// The same load marked non-temporal (streaming): for data read exactly once.
D2_DEV uint64_t ld64_stream(const void *base, uint32_t lane_off, uint32_t slot_off)
{
#if D2_GCN_ASM
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, 0xffffffff, 0x00020000);
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, lane_off, slot_off, 2 /* nt */);
    return ((uint64_t)v.y << 32) | v.x;
#else
    return *(const uint64_t *)((const char *)base + lane_off + slot_off);
#endif
}
// The same store marked non-temporal (streaming): for data the kernel never reads again, so that it
// does not displace what the kernel does re-read (parked words, keys, twiddles) from the caches.
D2_DEV void st64_stream(void *base, uint32_t lane_off, uint32_t slot_off, uint64_t val)
{
#if D2_GCN_ASM
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(base, 0, 0xffffffff, 0x00020000);
    u32x2 v;
    v.x = (uint32_t)val;
    v.y = (uint32_t)(val >> 32);
    __builtin_amdgcn_raw_buffer_store_b64(v, r, lane_off, slot_off, 2 /* nt */);
#else
    *(uint64_t *)((char *)base + lane_off + slot_off) = val;
#endif
}
D2_DEV uint64_t const_ld64(const void *base, uint32_t byte_off)
{
#if D2_GCN_ASM
    typedef const __attribute__((address_space(4))) uint64_t *cptr;
    return *(cptr)((uintptr_t)base + byte_off);
#else
    return *(const uint64_t *)((const char *)base + byte_off);
#endif
}
// a value that is the same in every lane of the wavefront, moved to a scalar register
D2_DEV uint32_t wave_uniform(uint32_t v)
{
#if D2_GCN_ASM
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
#else
    return v;
#endif
}

// floor(w * 2^64 / q) for w < q < 2^61 by binary long division (set-up paths only).
D2_DEV uint64_t shoup_quotient(uint64_t w, uint64_t q)
{
    uint64_t rem = w, quo = 0;
    for (int i = 0; i < 64; ++i) {
        rem <<= 1;
        quo <<= 1;
        if (rem >= q) { rem -= q; quo |= 1; }
    }
    return quo;
}

// ---------------------------------------------------------------------------------------
// Shared pieces of the two integer policies.
// ---------------------------------------------------------------------------------------
struct ModU {
    uint64_t q;     // modulus
    uint64_t nq;    // 2^64 - q
    uint64_t one_s; // floor(2^63 / q): Shoup quotient of the multiplicand 1
};

struct TwU {        // multiplicand and its 63-bit Shoup quotient
    uint64_t w, ws;
};

// w*y - qh*q mod 2^64, written as w*y + qh*(2^64 - q) so that every term is added:
// a chain of four 64-bit multiply-adds for the cross terms (only its low word matters; it is
// shifted up by 32), then two more for the low x low terms on top of it.
// SC: w sits in scalar registers (a multiplicand shared by the whole wavefront).  2^64 - q is the same
// for the whole workgroup and always comes from scalar registers (no instruction here reads both it
// and w, so the one-scalar-operand limit holds).
#define D2_SHOUP_TAIL_ASM(WC)                                                                      \
    asm("v_mad_u64_u32 %1, vcc, %4, %3, 0\n\t"                                                     \
        "v_mad_u64_u32 %1, vcc, %5, %2, %1\n\t"                                                    \
        "v_mad_u64_u32 %1, vcc, %6, %9, %1\n\t"                                                    \
        "v_mad_u64_u32 %1, vcc, %7, %8, %1\n\t"                                                    \
        "v_lshlrev_b64 %1, 32, %1\n\t"                                                             \
        "v_mad_u64_u32 %0, vcc, %4, %2, %1\n\t"                                                    \
        "v_mad_u64_u32 %0, vcc, %6, %8, %0"                                                        \
        : "=&v"(acc), "=&v"(cross)                                                                 \
        : "v"(y0), "v"(y1), WC(w0), WC(w1), "v"(h0), "v"(h1), "s"(n0), "s"(n1)                     \
        : "vcc")
template <bool SC = false>
D2_DEV uint64_t shoup_tail(uint64_t y, uint64_t w, uint64_t qh, uint64_t nq)
{
    const uint32_t y0 = lo32(y), y1 = hi32(y), w0 = lo32(w), w1 = hi32(w);
    const uint32_t h0 = lo32(qh), h1 = hi32(qh), n0 = lo32(nq), n1 = hi32(nq);
#if D2_GCN_ASM
    uint64_t acc, cross;
    if constexpr (SC) D2_SHOUP_TAIL_ASM("s");
    else D2_SHOUP_TAIL_ASM("v");
    return acc;
#else
    uint64_t acc = mul32(w0, y0);
    acc = mul32(h0, n0) + acc;
    const uint32_t cross = w0 * y1 + w1 * y0 + h0 * n1 + h1 * n0;
    return acc + ((uint64_t)cross << 32);
#endif
}

// u + (w*y - qh*q) mod 2^64: the addend rides on the multiply-add chain of the low x low terms, and the
// cross terms, of which only the low word matters, are added to the high word at the end: one
// instruction less than shoup_tail followed by a 64-bit addition, and two independent chains.
#define D2_SHOUP_TAIL_ADD_ASM(WC)                                                                  \
    asm("v_mad_u64_u32 %1, vcc, %4, %3, 0\n\t"                                                     \
        "v_mad_u64_u32 %0, vcc, %4, %2, %10\n\t"                                                   \
        "v_mad_u64_u32 %1, vcc, %5, %2, %1\n\t"                                                    \
        "v_mad_u64_u32 %0, vcc, %6, %8, %0\n\t"                                                    \
        "v_mad_u64_u32 %1, vcc, %6, %9, %1\n\t"                                                    \
        "v_mad_u64_u32 %1, vcc, %7, %8, %1"                                                        \
        : "=&v"(acc), "=&v"(cross)                                                                 \
        : "v"(y0), "v"(y1), WC(w0), WC(w1), "v"(h0), "v"(h1), "s"(n0), "s"(n1), "v"(u)             \
        : "vcc")
template <bool SC = false>
D2_DEV uint64_t shoup_tail_add(uint64_t y, uint64_t w, uint64_t qh, uint64_t nq, uint64_t u)
{
    const uint32_t y0 = lo32(y), y1 = hi32(y), w0 = lo32(w), w1 = hi32(w);
    const uint32_t h0 = lo32(qh), h1 = hi32(qh), n0 = lo32(nq), n1 = hi32(nq);
#if D2_GCN_ASM
    uint64_t acc, cross;
    if constexpr (SC) D2_SHOUP_TAIL_ADD_ASM("s");
    else D2_SHOUP_TAIL_ADD_ASM("v");
    // one 32-bit addition on the high word (written out: as C it comes back as a move plus a 64-bit add)
    uint32_t top = hi32(acc);
    const uint32_t cl = lo32(cross);
    asm("v_add_u32 %0, %0, %1" : "+v"(top) : "v"(cl));
    return ((uint64_t)top << 32) | lo32(acc);
#else
    uint64_t acc = mul32(w0, y0) + u;
    acc = mul32(h0, n0) + acc;
    const uint32_t cross = w0 * y1 + w1 * y0 + h0 * n1 + h1 * n0;
    return acc + ((uint64_t)cross << 32);
#endif
}

// y*1 - qh*q mod 2^64 (reduction of y itself)
D2_DEV uint64_t shoup_tail_one(uint64_t y, uint64_t qh, uint64_t nq)
{
    const uint32_t h0 = lo32(qh), h1 = hi32(qh), n0 = lo32(nq), n1 = hi32(nq);
    uint64_t acc = mul32(h0, n0) + y;
    const uint32_t cross = h0 * n1 + h1 * n0;
    return acc + ((uint64_t)cross << 32);
}

// floor(ws*y / 2^63) up to an error of 2 (too small): drops the low x low partial product.
// Needs ws < 2^63 and y < 2^63 (then the middle sum cannot overflow).
#define D2_QHAT_APPROX_ASM(WC)                                                                     \
    asm("v_mad_u64_u32 %0, vcc, %5, %2, 0\n\t"                                                     \
        "v_mad_u64_u32 %1, vcc, %5, %3, 0\n\t"                                                     \
        "v_mad_u64_u32 %0, vcc, %4, %3, %0\n\t"                                                    \
        "v_lshrrev_b64 %0, 31, %0\n\t"                                                             \
        "v_lshl_add_u64 %0, %1, 1, %0"                                                             \
        : "=&v"(mid), "=&v"(top)                                                                   \
        : "v"(y0), "v"(y1), WC(s0), WC(s1)                                                         \
        : "vcc")
template <bool SC = false>
D2_DEV uint64_t qhat_approx(uint64_t y, uint64_t ws)
{
    const uint32_t y0 = lo32(y), y1 = hi32(y), s0 = lo32(ws), s1 = hi32(ws);
#if D2_GCN_ASM
    uint64_t mid, top;
    if constexpr (SC) D2_QHAT_APPROX_ASM("s");
    else D2_QHAT_APPROX_ASM("v");
    return mid;
#else
    uint64_t mid = mul32(s1, y0);
    mid = mul32(s0, y1) + mid;
    const uint64_t top = mul32(s1, y1);
    return (top << 1) + (mid >> 31);
#endif
}

// floor(ws*y / 2^63) exactly, for ws < 2^63 and y < 2^63.
#define D2_QHAT_EXACT_ASM(WC)                                                                      \
    asm("v_mad_u64_u32 %0, vcc, %4, %2, 0\n\t"                                                     \
        "v_mad_u64_u32 %1, vcc, %5, %3, 0\n\t"                                                     \
        "v_lshrrev_b64 %0, 32, %0\n\t"                                                             \
        "v_mad_u64_u32 %0, vcc, %5, %2, %0\n\t"                                                    \
        "v_mad_u64_u32 %0, vcc, %4, %3, %0\n\t"                                                    \
        "v_lshrrev_b64 %0, 31, %0\n\t"                                                             \
        "v_lshl_add_u64 %0, %1, 1, %0"                                                             \
        : "=&v"(mid), "=&v"(top)                                                                   \
        : "v"(y0), "v"(y1), WC(s0), WC(s1)                                                         \
        : "vcc")
template <bool SC = false>
D2_DEV uint64_t qhat_exact(uint64_t y, uint64_t ws)
{
    const uint32_t y0 = lo32(y), y1 = hi32(y), s0 = lo32(ws), s1 = hi32(ws);
#if D2_GCN_ASM
    uint64_t mid, top;
    if constexpr (SC) D2_QHAT_EXACT_ASM("s");
    else D2_QHAT_EXACT_ASM("v");
    return mid;
#else
    uint64_t mid = mul32(s1, y0) + (uint64_t)__umulhi(s0, y0);
    mid = mul32(s0, y1) + mid;
    const uint64_t top = mul32(s1, y1);
    return (top << 1) + (mid >> 31);
#endif
}

// ---------------------------------------------------------------------------------------
// ArithS: moduli < 2^55, lazy products in [0, 4q).
// ---------------------------------------------------------------------------------------
struct ArithS {
    typedef uint64_t elem;
    typedef uint64_t word;          // LDS word of an exchange
    typedef ModU Mod;
    typedef TwU Twid;
    static constexpr int KIND = 1;

    D2_DEV static Mod mod(uint64_t q) { return Mod{q, 0 - q, 0}; }
    D2_DEV static Mod mod(uint64_t q, uint64_t one_s63) { return Mod{q, 0 - q, one_s63}; }
    D2_DEV static Twid tw(const Tw &t) { return Twid{t.w, t.ws}; }
    D2_DEV static Twid tw(uint64_t w, uint64_t ws64) { return Twid{w, ws64 >> 1}; }
    // element of a prepared key: values at v, 64-bit quotients at vs
    D2_DEV static Twid key(const uint64_t *v, const uint64_t *vs, uint32_t lane_off, uint32_t slot_off)
    {
        return tw(ld64(v, lane_off, slot_off), ld64(vs, lane_off, slot_off));
    }
    // table entry i: per-lane index / wave-uniform index (scalar registers, see mul<true>)
    static constexpr bool SCALAR_TW = true;
    D2_DEV static Twid load_v(const Tw *table, uint32_t i)
    {
        const U128 e = ld128(table, 16u * i, 0);
        return Twid{e.lo, e.hi};
    }
    D2_DEV static Twid load_u(const Tw *table, uint32_t i)
    {
        return Twid{const_ld64(table, 16u * i), const_ld64(table, 16u * i + 8u)};
    }

    // w*y mod q in [0, 4q), for y < 2^62.
    template <bool SC = false>
    D2_DEV static elem mul(elem y, const Twid &w, const Mod &m)
    {
        return shoup_tail<SC>(y, w.w, qhat_approx<SC>(y, w.ws), m.nq);
    }
    // w*y mod q in [0, 4q) for a 32-bit y (a plaintext coefficient): with y's high word zero the
    // quotient estimate is one partial product (s1 y >> 31 < 2^32, at most 2 too small as in mul) and the
    // tail loses its y1 and h1 terms: 7 instructions instead of 12.
    D2_DEV static elem mul_u32(uint32_t y, const Twid &w, const Mod &m)
    {
        const uint32_t h = (uint32_t)(mul32(hi32(w.ws), y) >> 31);
        const uint64_t acc = mul32(lo32(w.w), y) + mul32(h, lo32(m.nq));
        const uint32_t cross = hi32(w.w) * y + h * hi32(m.nq);
        return acc + ((uint64_t)cross << 32);
    }
    D2_DEV static elem from_small(int32_t v, const Mod &m)
    {
        return v >= 0 ? (uint64_t)v : m.q - (uint64_t)(uint32_t)(-v);
    }
    D2_DEV static elem from_canon(uint64_t v, const Mod &) { return v; }
    D2_DEV static elem add(elem a, elem b) { return a + b; }
    // x + v for a small signed v (|v| <= 32), as a forward input: q is added instead of mapping v into
    // [0, q) first (the forward range has room for it)
    D2_DEV static elem add_small(elem x, int32_t v, const Mod &m) { return x + (m.q + (uint64_t)(int64_t)v); }

    // forward: no correction; each stage adds at most 4q to the bound.
    // x' = u + t comes out of the multiply-add chain itself, y' = u + 4q - t = (2u + 4q) - x'.
    template <bool SC = false>
    D2_DEV static void ct(elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const elem u = x;
        x = shoup_tail_add<SC>(y, w.w, qhat_approx<SC>(y, w.ws), m.nq, u);
        y = (2 * u + 4 * m.q) - x;
    }
    // First stage on small signed inputs (|xv|, |yv| <= 32): w*yv is an exact 64-bit product (|w yv| < 32q
    // < 2^60), so nothing is reduced: x' = (xv + 32q) + w yv, y' = (xv + 32q) - w yv, both in (0, 64q + 32).
    // The forward bound becomes 64q + 4q per later stage: 64q + 52q + one lazy product < 128q <= 2^62 for
    // the longest ring (2^14) and q < 2^55.
    template <bool SC = false>
    D2_DEV static void ct_small(int32_t xv, int32_t yv, elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const int64_t t = (int64_t)w.w * (int64_t)yv;
        const uint64_t base = 32 * m.q + (uint64_t)(int64_t)xv;
        x = base + (uint64_t)t;
        y = base - (uint64_t)t;
    }
    D2_DEV static void fwd_pass_begin(elem &, const Mod &) {}
    D2_DEV static void fwd_end(elem &, const Mod &) {}
    // inverse: values in [0, 4q)
    template <bool SC = false>
    D2_DEV static void gs(elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const elem four_q = 4 * m.q;
        const elem s = x + y, d = x + four_q - y;
        x = csub(s, four_q);
        y = mul<SC>(d, w, m);
    }
    template <bool SC = false>
    D2_DEV static void gs_last(elem &x, elem &y, const Twid &ninv, const Twid &wn, const Mod &m)
    {
        const elem s = x + y, d = x + 4 * m.q - y;
        x = mul<SC>(s, ninv, m);
        y = mul<SC>(d, wn, m);
    }
    D2_DEV static void inv_pass_begin(elem &, const Mod &) {}
    D2_DEV static elem inv_input(uint64_t canon, const Mod &) { return canon; }

    // any value < 2^62 -> [0, q)
    D2_DEV static uint64_t canon_wide(elem x, const Mod &m)
    {
        const elem r = shoup_tail_one(x, qhat_exact(x, m.one_s), m.nq);   // [0, 2q)
        return csub(r, m.q);
    }
    // [0, 4q) -> [0, q)
    D2_DEV static uint64_t canon_lazy(elem x, const Mod &m) { return csub(csub(x, 2 * m.q), m.q); }
    D2_DEV static uint64_t canon_fwd(elem x, const Mod &m) { return canon_wide(x, m); }
    D2_DEV static uint64_t canon_inv(elem x, const Mod &m) { return canon_lazy(x, m); }
    // forward output + one lazy product
    D2_DEV static uint64_t canon_acc(elem x, const Mod &m) { return canon_wide(x, m); }
};

// ---------------------------------------------------------------------------------------
// ArithB: moduli < 2^61, Harvey butterflies with an exact quotient.
// ---------------------------------------------------------------------------------------
struct ArithB {
    typedef uint64_t elem;
    typedef uint64_t word;          // LDS word of an exchange
    typedef ModU Mod;
    typedef TwU Twid;
    static constexpr int KIND = 2;

    D2_DEV static Mod mod(uint64_t q) { return Mod{q, 0 - q, 0}; }
    D2_DEV static Mod mod(uint64_t q, uint64_t one_s63) { return Mod{q, 0 - q, one_s63}; }
    D2_DEV static Twid tw(const Tw &t) { return Twid{t.w, t.ws}; }
    D2_DEV static Twid tw(uint64_t w, uint64_t ws64) { return Twid{w, ws64 >> 1}; }
    // element of a prepared key: values at v, 64-bit quotients at vs
    D2_DEV static Twid key(const uint64_t *v, const uint64_t *vs, uint32_t lane_off, uint32_t slot_off)
    {
        return tw(ld64(v, lane_off, slot_off), ld64(vs, lane_off, slot_off));
    }
    // table entry i: per-lane index / wave-uniform index (scalar registers, see mul<true>)
    static constexpr bool SCALAR_TW = true;
    D2_DEV static Twid load_v(const Tw *table, uint32_t i)
    {
        const U128 e = ld128(table, 16u * i, 0);
        return Twid{e.lo, e.hi};
    }
    D2_DEV static Twid load_u(const Tw *table, uint32_t i)
    {
        return Twid{const_ld64(table, 16u * i), const_ld64(table, 16u * i + 8u)};
    }

    // w*y mod q in [0, 2q), for y < 2^63.
    template <bool SC = false>
    D2_DEV static elem mul(elem y, const Twid &w, const Mod &m)
    {
        return shoup_tail<SC>(y, w.w, qhat_exact<SC>(y, w.ws), m.nq);
    }
    D2_DEV static elem from_small(int32_t v, const Mod &m)
    {
        return v >= 0 ? (uint64_t)v : m.q - (uint64_t)(uint32_t)(-v);
    }
    D2_DEV static elem from_canon(uint64_t v, const Mod &) { return v; }
    D2_DEV static elem add(elem a, elem b) { return a + b; }
    D2_DEV static elem mul_u32(uint32_t y, const Twid &w, const Mod &m) { return mul(y, w, m); }
    D2_DEV static elem add_small(elem x, int32_t v, const Mod &m) { return x + from_small(v, m); }

    // x, y in [0, 4q) -> [0, 4q)
    template <bool SC = false>
    D2_DEV static void ct(elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const elem two_q = 2 * m.q;
        const elem u = csub(x, two_q);
        x = shoup_tail_add<SC>(y, w.w, qhat_exact<SC>(y, w.ws), m.nq, u);       // u + t
        y = (2 * u + two_q) - x;                                                // u + 2q - t
    }
    // first stage on small signed inputs: no short cut here (the butterflies need their inputs below 4q)
    template <bool SC = false>
    D2_DEV static void ct_small(int32_t xv, int32_t yv, elem &x, elem &y, const Twid &w, const Mod &m)
    {
        x = from_small(xv, m);
        y = from_small(yv, m);
        ct<SC>(x, y, w, m);
    }
    D2_DEV static void fwd_pass_begin(elem &, const Mod &) {}
    D2_DEV static void fwd_end(elem &, const Mod &) {}
    // x, y in [0, 2q) -> [0, 2q)
    template <bool SC = false>
    D2_DEV static void gs(elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const elem two_q = 2 * m.q;
        const elem s = x + y, d = x + two_q - y;
        x = csub(s, two_q);
        y = mul<SC>(d, w, m);
    }
    template <bool SC = false>
    D2_DEV static void gs_last(elem &x, elem &y, const Twid &ninv, const Twid &wn, const Mod &m)
    {
        const elem s = x + y, d = x + 2 * m.q - y;
        x = mul<SC>(s, ninv, m);
        y = mul<SC>(d, wn, m);
    }
    D2_DEV static void inv_pass_begin(elem &, const Mod &) {}
    D2_DEV static elem inv_input(uint64_t canon, const Mod &) { return canon; }

    D2_DEV static uint64_t canon_lazy(elem x, const Mod &m) { return csub(csub(x, 2 * m.q), m.q); }
    // any value < 2^63 -> [0, q)
    D2_DEV static uint64_t canon_wide(elem x, const Mod &m)
    {
        const elem r = shoup_tail_one(x, qhat_exact(x, m.one_s), m.nq);
        return csub(r, m.q);
    }
    D2_DEV static uint64_t canon_fwd(elem x, const Mod &m) { return canon_lazy(x, m); }
    D2_DEV static uint64_t canon_inv(elem x, const Mod &m) { return csub(x, m.q); }
    // forward output + one lazy product: [0, 6q)
    D2_DEV static uint64_t canon_acc(elem x, const Mod &m) { return canon_lazy(csub(x, 4 * m.q), m); }
};

// ---------------------------------------------------------------------------------------
// ArithF: moduli < 2^44, residues as doubles holding integers (signed representatives).
// ---------------------------------------------------------------------------------------
struct ArithF {
    typedef double elem;
    typedef uint64_t word;          // LDS word of an exchange
    struct Mod {
        double q, qinv;
        uint64_t qi;
    };
    struct Twid {
        double w;
    };
    static constexpr int KIND = 0;

    D2_DEV static double u2d(uint64_t v)    // exact for v < 2^52
    {
        return __longlong_as_double((long long)(v | 0x4330000000000000ull)) - 4503599627370496.0;
    }
    D2_DEV static uint64_t d2u(double r)    // exact for integers 0 <= r < 2^52
    {
        return (uint64_t)__double_as_longlong(r + 4503599627370496.0) & 0x000fffffffffffffull;
    }
    D2_DEV static Mod mod(uint64_t q)
    {
        const double qd = u2d(q);
        return Mod{qd, 1.0 / qd, q};
    }
    // aux: bits of the double 1/q (what the per-modulus table holds for this policy)
    D2_DEV static Mod mod(uint64_t q, uint64_t aux) { return Mod{u2d(q), __longlong_as_double((long long)aux), q}; }
    D2_DEV static Twid tw(const Tw &t) { return Twid{__longlong_as_double((long long)t.w)}; }
    D2_DEV static Twid tw(uint64_t w, uint64_t) { return Twid{u2d(w)}; }
    // element of a prepared key: only the values are read
    D2_DEV static Twid key(const uint64_t *v, const uint64_t *, uint32_t lane_off, uint32_t slot_off)
    {
        return Twid{u2d(ld64(v, lane_off, slot_off))};
    }
    // table entry i: per-lane index / wave-uniform index (scalar registers feed the f64 ALU directly)
    static constexpr bool SCALAR_TW = true;
    D2_DEV static Twid load_v(const Tw *table, uint32_t i)
    {
        return Twid{__longlong_as_double((long long)ld64(table, 16u * i, 0))};
    }
    D2_DEV static Twid load_u(const Tw *table, uint32_t i)
    {
        return Twid{__longlong_as_double((long long)const_ld64(table, 16u * i))};
    }

    // x - round(x/q) q: about (-q/2, q/2)
    D2_DEV static elem reduce(elem x, const Mod &m)
    {
        const double b = __builtin_rint(x * m.qinv);
        return __builtin_fma(-b, m.q, x);
    }
    // w*y mod q as a signed representative, for |w y| < 2^96.  Its magnitude is at most
    // q/2 + 1.5 |w y| 2^-52: the quotient is rounded from h/q computed with a relative error of 2^-52, and
    // the low part l of the product (|l| <= |w y| 2^-53) is added after the reduction.  That is q/2 + 1 for
    // canonical operands and up to 0.75 q for |y| = 42 q at the largest modulus.
    template <bool SC = false>
    D2_DEV static elem mul(elem y, const Twid &w, const Mod &m)
    {
        const double h = w.w * y;
        const double l = __builtin_fma(w.w, y, -h);
        const double b = __builtin_rint(h * m.qinv);
        const double r = __builtin_fma(-b, m.q, h);
        return r + l;
    }
    D2_DEV static elem from_small(int32_t v, const Mod &) { return (double)v; }
    D2_DEV static elem from_canon(uint64_t v, const Mod &) { return u2d(v); }
    D2_DEV static elem mul_u32(uint32_t y, const Twid &w, const Mod &m) { return mul((double)y, w, m); }
    D2_DEV static elem add_small(elem x, int32_t v, const Mod &) { return x + (double)v; }
    D2_DEV static elem add(elem a, elem b) { return a + b; }

    template <bool SC = false>
    D2_DEV static void ct(elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const elem t = mul<SC>(y, w, m);
        const elem u = x;
        x = u + t;
        y = u - t;
    }
    // First stage on small signed inputs (|xv|, |yv| <= 32): w*yv is exact in a double (< 2^49), so the
    // stage is one multiplication and two additions.  The values then reach 32q; every later stage adds one
    // product (see mul), i.e. takes a bound of c q to (1 + 1.5 q 2^-52) c q + q/2: 41.3 q after the 13 further
    // stages of the longest ring that starts this way (2^14) at q = 2^44, 42.1 q with one more lazy product
    // on top -- inside what canon_wide accepts (64 q) and far inside the 2^53 of exact integers.
    template <bool SC = false>
    D2_DEV static void ct_small(int32_t xv, int32_t yv, elem &x, elem &y, const Twid &w, const Mod &)
    {
        const double t = w.w * (double)yv, u = (double)xv;
        x = u + t;
        y = u - t;
    }
    D2_DEV static void fwd_pass_begin(elem &, const Mod &) {}
    D2_DEV static void fwd_end(elem &, const Mod &) {}
    template <bool SC = false>
    D2_DEV static void gs(elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const elem s = x + y, d = x - y;
        x = s;
        y = mul<SC>(d, w, m);
    }
    template <bool SC = false>
    D2_DEV static void gs_last(elem &x, elem &y, const Twid &ninv, const Twid &wn, const Mod &m)
    {
        const elem s = x + y, d = x - y;
        x = mul<SC>(s, ninv, m);
        y = mul<SC>(d, wn, m);
    }
    // the sum path of the inverse doubles every stage: bring it back once per pass
    D2_DEV static void inv_pass_begin(elem &x, const Mod &m) { x = reduce(x, m); }
    D2_DEV static elem inv_input(uint64_t canon, const Mod &) { return u2d(canon); }

    // |x| <= 64 q -> [0, q).  x/q is either an integer or at least 1/q > 2^-44 away from one; the
    // computed quotient is off by at most 2 * 64 * 2^-53 = 2^-46 (the rounding of 1/q and of the
    // fused multiply-add), so with a bias of 2^-46 floor() is exact and the remainder needs no correction.
    D2_DEV static uint64_t canon_wide(elem x, const Mod &m)
    {
        const double b = __builtin_floor(__builtin_fma(x, m.qinv, 0x1p-46));
        return d2u(__builtin_fma(-b, m.q, x));
    }
    D2_DEV static uint64_t canon_lazy(elem x, const Mod &m) { return canon_wide(x, m); }
    D2_DEV static uint64_t canon_fwd(elem x, const Mod &m) { return canon_wide(x, m); }
    D2_DEV static uint64_t canon_inv(elem x, const Mod &m) { return canon_wide(x, m); }
    D2_DEV static uint64_t canon_acc(elem x, const Mod &m) { return canon_wide(x, m); }
};

// ---------------------------------------------------------------------------------------
// Arith32: moduli < 2^30, 32-bit residues, Harvey butterflies with a 32-bit Shoup quotient.
// Forward values in [0, 4q) (< 2^32), a finished forward transform in [0, 2q) so that one more lazy
// product can be added without overflow; inverse values in [0, 2q).
// Table entries hold {w | floor(w 2^32 / q) << 32, -} (8 bytes are read per twiddle).
// ---------------------------------------------------------------------------------------
struct Arith32 {
    typedef uint32_t elem;
    typedef uint32_t word;          // LDS word of an exchange
    struct Mod {
        uint32_t q, two_q, nq;      // nq = 2^32 - q
        uint32_t one_s;             // floor(2^32 / q)
    };
    struct Twid {
        uint32_t w, ws;
    };
    static constexpr int KIND = 3;

    D2_DEV static Mod mod(uint64_t q, uint64_t one_s32) { return Mod{(uint32_t)q, 2u * (uint32_t)q, 0u - (uint32_t)q, (uint32_t)one_s32}; }
    D2_DEV static Mod mod(uint64_t q) { return mod(q, (1ull << 32) / q); }
    D2_DEV static Twid tw(const Tw &t) { return Twid{lo32(t.w), hi32(t.w)}; }
    D2_DEV static Twid tw(uint64_t w, uint64_t ws64) { return Twid{(uint32_t)w, hi32(ws64)}; }
    // element of a prepared key: values at v, 64-bit quotients at vs (their high words are the 32-bit quotients)
    D2_DEV static Twid key(const uint64_t *v, const uint64_t *vs, uint32_t lane_off, uint32_t slot_off)
    {
        return tw(ld64(v, lane_off, slot_off), ld64(vs, lane_off, slot_off));
    }
    static constexpr bool SCALAR_TW = true;
    D2_DEV static Twid load_v(const Tw *table, uint32_t i)
    {
        const uint64_t e = ld64(table, 16u * i, 0);
        return Twid{lo32(e), hi32(e)};
    }
    D2_DEV static Twid load_u(const Tw *table, uint32_t i)
    {
        const uint64_t e = const_ld64(table, 16u * i);
        return Twid{lo32(e), hi32(e)};
    }

    // x >= m ? x - m : x for x < 2m: the smaller of x and x - m as unsigned numbers
    D2_DEV static uint32_t csub32(uint32_t x, uint32_t m)
    {
        const uint32_t d = x - m;
        return d < x ? d : x;
    }
    // w*y mod q in [0, 2q), for any 32-bit y: the low word of w y + floor(ws y / 2^32) (2^32 - q)
    template <bool SC = false>
    D2_DEV static elem mul(elem y, const Twid &w, const Mod &m)
    {
        const uint32_t qh = __umulhi(y, w.ws);
        return (uint32_t)(mul32(w.w, y) + mul32(qh, m.nq));
    }
    D2_DEV static elem from_small(int32_t v, const Mod &m) { return v >= 0 ? (uint32_t)v : m.q - (uint32_t)(-v); }
    D2_DEV static elem from_canon(uint64_t v, const Mod &) { return (uint32_t)v; }
    D2_DEV static elem add(elem a, elem b) { return a + b; }
    D2_DEV static elem mul_u32(uint32_t y, const Twid &w, const Mod &m) { return mul(y, w, m); }
    D2_DEV static elem add_small(elem x, int32_t v, const Mod &m) { return x + from_small(v, m); }

    // x, y in [0, 4q) -> [0, 4q)
    template <bool SC = false>
    D2_DEV static void ct(elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const elem u = csub32(x, m.two_q);
        const elem t = mul<SC>(y, w, m);
        x = u + t;
        y = u + m.two_q - t;
    }
    // first stage on small signed inputs: no short cut (8 instructions per butterfly as it is)
    template <bool SC = false>
    D2_DEV static void ct_small(int32_t xv, int32_t yv, elem &x, elem &y, const Twid &w, const Mod &m)
    {
        x = from_small(xv, m);
        y = from_small(yv, m);
        ct<SC>(x, y, w, m);
    }
    D2_DEV static void fwd_pass_begin(elem &, const Mod &) {}
    // the last step of a forward transform: [0, 4q) -> [0, 2q)
    D2_DEV static void fwd_end(elem &x, const Mod &m) { x = csub32(x, m.two_q); }
    // x, y in [0, 2q) -> [0, 2q)
    template <bool SC = false>
    D2_DEV static void gs(elem &x, elem &y, const Twid &w, const Mod &m)
    {
        const elem s = x + y, d = x + m.two_q - y;
        x = csub32(s, m.two_q);
        y = mul<SC>(d, w, m);
    }
    template <bool SC = false>
    D2_DEV static void gs_last(elem &x, elem &y, const Twid &ninv, const Twid &wn, const Mod &m)
    {
        const elem s = x + y, d = x + m.two_q - y;
        x = mul<SC>(s, ninv, m);
        y = mul<SC>(d, wn, m);
    }
    D2_DEV static void inv_pass_begin(elem &, const Mod &) {}
    D2_DEV static elem inv_input(uint64_t canon, const Mod &) { return (uint32_t)canon; }

    // [0, 4q) -> [0, q)
    D2_DEV static uint64_t canon_lazy(elem x, const Mod &m) { return csub32(csub32(x, m.two_q), m.q); }
    // any 32-bit value -> [0, q)
    D2_DEV static uint64_t canon_wide(elem x, const Mod &m)
    {
        const uint32_t r = x - __umulhi(x, m.one_s) * m.q;        // [0, 2q)
        return csub32(r, m.q);
    }
    D2_DEV static uint64_t canon_fwd(elem x, const Mod &m) { return canon_lazy(x, m); }
    D2_DEV static uint64_t canon_inv(elem x, const Mod &m) { return csub32(x, m.q); }
    // finished forward transform ([0, 2q)) + one lazy product ([0, 2q))
    D2_DEV static uint64_t canon_acc(elem x, const Mod &m) { return canon_lazy(x, m); }
};

// canonical u64 helpers used outside the transforms
D2_DEV uint64_t add_mod(uint64_t a, uint64_t b, uint64_t q) { return csub(a + b, q); }
// w*y mod q, canonical, with the 64-bit Shoup quotient ws64 = floor(w 2^64 / q); any 64-bit y
D2_DEV uint64_t mul_shoup64(uint64_t y, uint64_t w, uint64_t ws64, uint64_t q)
{
    const uint64_t r = w * y - __umul64hi(ws64, y) * q;
    return csub(r, q);
}

// uint64 <-> element bit patterns for lazily stored intermediates and 8-byte LDS words; a policy with
// 4-byte LDS words (Arith32) stores its elements as they are
template <class A>
D2_DEV uint64_t to_bits(typename A::elem v);
template <>
D2_DEV uint64_t to_bits<ArithS>(uint64_t v) { return v; }
template <>
D2_DEV uint64_t to_bits<ArithB>(uint64_t v) { return v; }
template <>
D2_DEV uint64_t to_bits<ArithF>(double v) { return (uint64_t)__double_as_longlong(v); }

template <>
D2_DEV uint64_t to_bits<Arith32>(uint32_t v) { return v; }

template <class A>
D2_DEV typename A::elem from_bits(uint64_t v);
template <>
D2_DEV uint32_t from_bits<Arith32>(uint64_t v) { return (uint32_t)v; }
template <>
D2_DEV uint64_t from_bits<ArithS>(uint64_t v) { return v; }
template <>
D2_DEV uint64_t from_bits<ArithB>(uint64_t v) { return v; }
template <>
D2_DEV double from_bits<ArithF>(uint64_t v) { return __longlong_as_double((long long)v); }

template <class A>
D2_DEV typename A::word to_word(typename A::elem v)
{
    if constexpr (sizeof(typename A::word) == 8) return to_bits<A>(v);
    else return v;
}
template <class A>
D2_DEV typename A::elem from_word(typename A::word v)
{
    if constexpr (sizeof(typename A::word) == 8) return from_bits<A>(v);
    else return v;
}

}  // namespace d2
