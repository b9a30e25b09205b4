// HIP kernels of the exchange round.  One workgroup owns one polynomial (or one ciphertext
// and walks over its RNS limbs); transforms run in registers + LDS (ntt_engine.hpp).
#pragma once
#include "ntt_engine.hpp"
#include "philox.hpp"
#include <stddef.h>

// no fused multiply-add unless written out: float results here are compared bit for bit
#pragma clang fp contract(off)

namespace d2 {

constexpr int MAX_LIMBS = 16;
constexpr int MAX_GROUP = 64;

// Per-modulus constants; entry L of the table array describes the plaintext modulus t.
// Tw entries are in the context's arithmetic format ({w, floor(w 2^63/q)} for the 64-bit integer
// policies, {bits of the double w, -} for the floating-point policy, {w | floor(w 2^32/q) << 32, -} for
// the 32-bit policy; the entry of the plaintext modulus is always in the 32-bit format), except
// `gamma` and `pow32`, which are always {w, floor(w 2^64/q)} (they work on canonical 64-bit integers).
struct LimbTab {
    uint64_t q;
    uint64_t one_s;     // floor(2^63 / q); floating-point policy: bits of the double 1/q; 32-bit policy: floor(2^32 / q)
    Tw ninv;            // N^-1 mod q
    Tw wn;              // (inverse twiddle 1) * N^-1 mod q
    Tw lambda;          // floor(Q/t) mod q
    Tw gamma;           // (Q/q)^-1 mod q, integer pair
    uint64_t theta_hi;  // floor(t * 2^128 / q), high and low words
    uint64_t theta_lo;
    Tw pow32;           // 2^32 mod q, integer pair like gamma (reduction of 128-bit uniform blocks)
    uint64_t inv64;     // floor(2^64 / q)
    const Tw *fwd;      // forward twiddles, N entries
    const Tw *inv;      // inverse twiddles, N entries
};

// Entry i (uniform over the workgroup) of the table array, fetched with scalar loads so that the
// constants and the table pointers stay in scalar registers.
D2_DEV LimbTab load_tab(const LimbTab *tabs, uint32_t i)
{
    const LimbTab *e = tabs + i;
    LimbTab r;
    r.q = const_ld64(e, offsetof(LimbTab, q));
    r.one_s = const_ld64(e, offsetof(LimbTab, one_s));
    r.ninv = Tw{const_ld64(e, offsetof(LimbTab, ninv)), const_ld64(e, offsetof(LimbTab, ninv) + 8)};
    r.wn = Tw{const_ld64(e, offsetof(LimbTab, wn)), const_ld64(e, offsetof(LimbTab, wn) + 8)};
    r.lambda = Tw{const_ld64(e, offsetof(LimbTab, lambda)), const_ld64(e, offsetof(LimbTab, lambda) + 8)};
    r.gamma = Tw{const_ld64(e, offsetof(LimbTab, gamma)), const_ld64(e, offsetof(LimbTab, gamma) + 8)};
    r.theta_hi = const_ld64(e, offsetof(LimbTab, theta_hi));
    r.theta_lo = const_ld64(e, offsetof(LimbTab, theta_lo));
    r.pow32 = Tw{const_ld64(e, offsetof(LimbTab, pow32)), const_ld64(e, offsetof(LimbTab, pow32) + 8)};
    r.inv64 = const_ld64(e, offsetof(LimbTab, inv64));
    r.fwd = (const Tw *)const_ld64(e, offsetof(LimbTab, fwd));
    r.inv = (const Tw *)const_ld64(e, offsetof(LimbTab, inv));
    return r;
}

// The 128-bit little-endian value of a Philox block reduced mod q (uniform sampling): Horner over
// its four words, r <- r * 2^32 + w, with 2^32 mod q as a prepared multiplicand and floor(2^64 / q)
// to reduce the words themselves (they can exceed a modulus below 2^32).
D2_DEV uint64_t uniform_mod(const Block4 &b, const LimbTab &tb)
{
    const uint64_t q = tb.q;
    uint64_t r = mul_shoup64(b.w[3], 1, tb.inv64, q);
#pragma unroll
    for (int i = 2; i >= 0; --i)
        r = add_mod(mul_shoup64(r, tb.pow32.w, tb.pow32.ws, q), mul_shoup64(b.w[i], 1, tb.inv64, q), q);
    return r;
}

struct RoundConst {
    uint64_t t;
    uint32_t L;
    uint32_t eta_mask;   // low eta bits set
    int32_t clamp;       // floor(((t-1)/2) / K_max)
    float scale;         // 2^f
    float inv_scale;     // 2^-f
    PhiloxKey key;
    uint32_t coeff_packing;   // 0: value j of a ciphertext is slot j (default); 1: it is coefficient j
};

struct PtrList {
    const void *p[MAX_GROUP];
};

// Job tables passed by value in the kernel arguments; grid.y indexes the job.
constexpr int JOB_CHUNK = 112;   // 112 * 32 B of table + the other arguments stay under the 4 KB argument limit
struct EncJobs {                       // one job = one (party, group) pair encrypting C ciphertexts
    const void *src[JOB_CHUNK];        // gradient (float) or plaintext polynomials (uint64)
    const uint64_t *pk[JOB_CHUNK];     // prepared public key of the group
    uint64_t *out[JOB_CHUNK];          // ciphertexts [C][2][L][N]
    uint32_t party[JOB_CHUNK];
    uint32_t group[JOB_CHUNK];
};
struct ShareJobs {                     // one job = one member's shares of C aggregated ciphertexts
    const uint64_t *sk[JOB_CHUNK];     // prepared secret share
    const uint64_t *ct[JOB_CHUNK];     // aggregate [C][2][L][N]
    uint64_t *out[JOB_CHUNK];          // shares [C][L][N]
    uint32_t party[JOB_CHUNK];
    uint32_t group[JOB_CHUNK];
};
constexpr int CONV_CHUNK = 80;         // 80 * 40 B of table
struct ConvJobs {                      // one job = one member's conversion shares towards one receiver
    const uint64_t *sk[CONV_CHUNK];    // the member's prepared secret share
    const uint64_t *pk[CONV_CHUNK];    // the receiver's prepared public key
    const uint64_t *ct[CONV_CHUNK];    // aggregate [C][2][L][N]
    uint64_t *out[CONV_CHUNK];         // shares [C][2][L][N]
    uint32_t who[CONV_CHUNK];          // member | receiver << 16: the party word of the counters
    uint32_t group[CONV_CHUNK];
};
struct GroupJobs {                     // one job = one group: K buffers laid out at a fixed stride
    const uint64_t *first[JOB_CHUNK];  // buffer of the group's first member
    const uint64_t *ct[JOB_CHUNK];     // aggregate (combine) / unused (sum)
    void *out[JOB_CHUNK];              // aggregate (sum) / decoded floats (combine)
    uint32_t K[JOB_CHUNK];
};
struct RecvJobs {                      // one job = one receiver of one group (MBFV.Convert)
    const uint64_t *first[CONV_CHUNK]; // conversion shares of the group's first member for this receiver
    const uint64_t *ct[CONV_CHUNK];    // aggregate
    const uint64_t *sk[CONV_CHUNK];    // the receiver's prepared secret key
    void *out[CONV_CHUNK];             // decoded floats
    uint32_t K[CONV_CHUNK];
};

D2_DEV uint32_t bitrev(uint32_t v, int bits) { return __brev(v) >> (32 - bits); }

// Returns v unchanged but opaque to the optimiser.  Used at the top of per-limb loops so that
// per-thread addresses and sample conversions are recomputed per iteration (a few
// instructions) instead of being hoisted and kept in ~100 registers across the whole loop.
D2_DEV int opaque(int v)
{
#if D2_GCN_ASM
    asm volatile("" : "+v"(v));
#endif
    return v;
}
D2_DEV uint32_t opaque(uint32_t v) { return (uint32_t)opaque((int)v); }

// -------------------------------------------------------------------------------------
// Plain batched transforms: polys [B][L][N] in place, one workgroup per (b, limb).
// -------------------------------------------------------------------------------------
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_ntt_forward(uint64_t *polys, const LimbTab *tabs, uint32_t L)
{
    typedef typename ENG::A A;
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const int tid = threadIdx.x;
    const LimbTab tb = load_tab(tabs, blockIdx.x % L);
    const typename A::Mod md = A::mod(tb.q, tb.one_s);
    uint64_t *p = polys + (size_t)blockIdx.x * ENG::NB;
    typename A::elem x[ENG::E];
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) x[k] = A::from_canon(p[ENG::coef_pos(k, tid)], md);
    ENG::forward(x, lds, tid, 0, tb.fwd, md);
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) p[ENG::eval_pos(k, tid)] = A::canon_fwd(x[k], md);
}

template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_ntt_inverse(uint64_t *polys, const LimbTab *tabs, uint32_t L)
{
    typedef typename ENG::A A;
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const int tid = threadIdx.x;
    const LimbTab tb = load_tab(tabs, blockIdx.x % L);
    const typename A::Mod md = A::mod(tb.q, tb.one_s);
    uint64_t *p = polys + (size_t)blockIdx.x * ENG::NB;
    typename A::elem x[ENG::E];
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) x[k] = A::inv_input(p[ENG::eval_pos(k, tid)], md);
    ENG::template inverse<true>(x, lds, tid, 0, tb.inv, md, A::tw(tb.ninv), A::tw(tb.wn));
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) p[ENG::coef_pos(k, tid)] = A::canon_inv(x[k], md);
}

// -------------------------------------------------------------------------------------
// Transforms longer than one workgroup can hold: the top LOGH = LOGN - LOGB stages couple
// the 2^LOGH blocks of NB coefficients ("head", register-only, strided global access); the
// remaining LOGB stages are independent per block ("tail", the engine with a block id).
// Between the two kernels the data stays in the policy's lazy representation.
// -------------------------------------------------------------------------------------
template <class A, int LOGN, int LOGH>
__global__ void __launch_bounds__(256) k_head_forward(uint64_t *polys, const LimbTab *tabs, uint32_t L,
                                                        uint32_t poly0)
{
    constexpr int H = 1 << LOGH;
    constexpr int STRIDE = 1 << (LOGN - LOGH);
    const uint32_t poly = blockIdx.y;
    const LimbTab tb = load_tab(tabs, (poly0 + poly) % L);
    const typename A::Mod md = A::mod(tb.q, tb.one_s);
    const Tw *tw = tb.fwd;
    uint64_t *p = polys + ((size_t)poly << LOGN) + (size_t)blockIdx.x * 256 + threadIdx.x;
    typename A::elem x[H];
#pragma unroll
    for (int k = 0; k < H; ++k) x[k] = A::from_canon(p[(size_t)k * STRIDE], md);
#pragma unroll
    for (int kb = LOGH - 1; kb >= 0; --kb) {
        const int s = LOGH - 1 - kb;
#pragma unroll
        for (int g = 0; g < (H >> (kb + 1)); ++g) {
            const typename A::Twid w = load_tw_uniform<A>(tw, (1u << s) + g);
#pragma unroll
            for (int j = 0; j < (1 << kb); ++j) {
                const int k0 = (g << (kb + 1)) | j;
                A::template ct<A::SCALAR_TW>(x[k0], x[k0 | (1 << kb)], w, md);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < H; ++k) p[(size_t)k * STRIDE] = to_bits<A>(x[k]);   // stays lazy
}

template <class A, int LOGN, int LOGH>
__global__ void __launch_bounds__(256) k_head_inverse(uint64_t *polys, const LimbTab *tabs, uint32_t L,
                                                        uint32_t poly0)
{
    constexpr int H = 1 << LOGH;
    constexpr int STRIDE = 1 << (LOGN - LOGH);
    const uint32_t poly = blockIdx.y;
    const LimbTab tb = load_tab(tabs, (poly0 + poly) % L);
    const typename A::Mod md = A::mod(tb.q, tb.one_s);
    const Tw *tw = tb.inv;
    uint64_t *p = polys + ((size_t)poly << LOGN) + (size_t)blockIdx.x * 256 + threadIdx.x;
    typename A::elem x[H];
#pragma unroll
    for (int k = 0; k < H; ++k) {
        x[k] = from_bits<A>(p[(size_t)k * STRIDE]);               // lazy, from the tail kernel
        A::inv_pass_begin(x[k], md);
    }
#pragma unroll
    for (int kb = 0; kb < LOGH; ++kb) {
        const int s = LOGH - 1 - kb;
        if (kb == LOGH - 1) {                                    // last stage: fold N^-1
#pragma unroll
            for (int j = 0; j < (1 << kb); ++j) A::template gs_last<true>(x[j], x[j | (1 << kb)], A::tw(tb.ninv), A::tw(tb.wn), md);
        } else {
#pragma unroll
            for (int g = 0; g < (H >> (kb + 1)); ++g) {
                const typename A::Twid w = load_tw_uniform<A>(tw, (1u << s) + g);
#pragma unroll
                for (int j = 0; j < (1 << kb); ++j) {
                    const int k0 = (g << (kb + 1)) | j;
                    A::template gs<A::SCALAR_TW>(x[k0], x[k0 | (1 << kb)], w, md);
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < H; ++k) p[(size_t)k * STRIDE] = A::canon_inv(x[k], md);
}

// Tail of a long transform over polys [B][L][N].  Tiles that share twiddles -- the same (limb, block)
// of every polynomial of the batch, a "group" of B members -- are given to one workgroup TAIL_TILES
// members at a time: it fetches the twiddles once (scalar registers for the uniform passes, 56
// vector registers for the rest with 16-byte entries) and walks its members with the next member's
// coefficients already requested.  Without this the twiddles are twice the bytes of the data.
// Workgroups are handed to the 8 XCDs round-robin by linear id: XCD x = i % 8 walks the contiguous
// slot range [x * grid/8, (x+1) * grid/8), so that the workgroups of a group also share an L2.
constexpr int TAIL_TILES = 8;

struct TailTile {
    uint32_t limb, blk, m0, m1;       // members [m0, m1) of group (limb, blk)
};
D2_DEV TailTile tail_tile(uint32_t i, uint32_t grid, uint32_t B, uint32_t nblk)
{
    const uint32_t wpg = (B + TAIL_TILES - 1) / TAIL_TILES;      // workgroups per group
    uint32_t slot = i;
    if ((grid & 7u) == 0) slot = (i & 7u) * (grid >> 3) + (i >> 3);
    const uint32_t group = slot / wpg, part = slot % wpg;
    // the same in every lane (they depend on the workgroup id only): keep them in scalar registers,
    // the divisions above went through the vector ALU
    TailTile t;
    t.limb = wave_uniform(group / nblk);
    t.blk = wave_uniform(group % nblk);
    t.m0 = wave_uniform(part * TAIL_TILES);
    t.m1 = t.m0 + TAIL_TILES < B ? t.m0 + TAIL_TILES : B;
    return t;
}

// grid = L * 2^(LOGN - LOGB) * ceil(B / TAIL_TILES)
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_tail_forward(uint64_t *polys, const LimbTab *tabs, uint32_t L,
                                                        uint32_t B)
{
    typedef typename ENG::A A;
    constexpr int E = ENG::E;
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const int tid = threadIdx.x;
    const TailTile tt = tail_tile(blockIdx.x, gridDim.x, B, 1u << (ENG::LOGN - ENG::LOGB));
    if (tt.limb >= L || tt.m0 >= tt.m1) return;
    const LimbTab tb = load_tab(tabs, tt.limb);
    const typename A::Mod md = A::mod(tb.q, tb.one_s);
    typename ENG::Twiddles tw;
    ENG::template load_all<false, false>(tw, tid, tt.blk, tb.fwd);
    const size_t stride = (size_t)L << ENG::LOGN;        // words between members
    uint64_t *p = polys + (((size_t)tt.m0 * L + tt.limb) << ENG::LOGN) + ((size_t)tt.blk << ENG::LOGB);
    uint64_t nx[E];
#pragma unroll
    for (int k = 0; k < E; ++k) nx[k] = ld64(p, 8u * (uint32_t)tid, 8u * ENG::T * k);
    for (uint32_t m = tt.m0; m < tt.m1; ++m, p += stride) {
        typename A::elem x[E];
#pragma unroll
        for (int k = 0; k < E; ++k) x[k] = from_bits<A>(nx[k]);
        if (m + 1 < tt.m1) {
#pragma unroll
            for (int k = 0; k < E; ++k) nx[k] = ld64(p + stride, 8u * (uint32_t)tid, 8u * ENG::T * k);
        }
        ENG::forward(x, lds, tid, tw, md);
#pragma unroll
        for (int k = 0; k < E; ++k) st64(p, 8u * (uint32_t)tid, 8u * ENG::T * k, A::canon_fwd(x[k], md));
    }
}

template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_tail_inverse(uint64_t *polys, const LimbTab *tabs, uint32_t L,
                                                        uint32_t B)
{
    typedef typename ENG::A A;
    constexpr int E = ENG::E;
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const int tid = threadIdx.x;
    const TailTile tt = tail_tile(blockIdx.x, gridDim.x, B, 1u << (ENG::LOGN - ENG::LOGB));
    if (tt.limb >= L || tt.m0 >= tt.m1) return;
    const LimbTab tb = load_tab(tabs, tt.limb);
    const typename A::Mod md = A::mod(tb.q, tb.one_s);
    typename ENG::Twiddles tw;
    ENG::template load_all<true, false>(tw, tid, tt.blk, tb.inv);
    const typename A::Twid ninv = A::tw(tb.ninv), wn = A::tw(tb.wn);
    const size_t stride = (size_t)L << ENG::LOGN;
    uint64_t *p = polys + (((size_t)tt.m0 * L + tt.limb) << ENG::LOGN) + ((size_t)tt.blk << ENG::LOGB);
    uint64_t nx[E];
#pragma unroll
    for (int k = 0; k < E; ++k) nx[k] = ld64(p, 8u * (uint32_t)tid, 8u * ENG::T * k);
    for (uint32_t m = tt.m0; m < tt.m1; ++m, p += stride) {
        typename A::elem x[E];
#pragma unroll
        for (int k = 0; k < E; ++k) x[k] = A::inv_input(nx[k], md);
        if (m + 1 < tt.m1) {
#pragma unroll
            for (int k = 0; k < E; ++k) nx[k] = ld64(p + stride, 8u * (uint32_t)tid, 8u * ENG::T * k);
        }
        ENG::template inverse<false>(x, lds, tid, tw, md, ninv, wn);
#pragma unroll
        for (int k = 0; k < E; ++k) st64(p, 8u * (uint32_t)tid, 8u * ENG::T * k, to_bits<A>(x[k]));   // lazy, head finishes
    }
}

// -------------------------------------------------------------------------------------
// Sampling helpers: small polynomials are drawn block by block, staged in LDS as packed
// words (one per coefficient, natural order) and then picked up by their pass-0 owners.
// -------------------------------------------------------------------------------------
// mu (ternary) in byte 0, e0 in byte 1, e1 in byte 2 (two's complement bytes); their domains are
// dom, dom + 1, dom + 2 (DOM_ENC_U for Encrypt, DOM_CVT_U for a conversion share)
template <class ENG>
D2_DEV void stage_encrypt_samples(uint32_t *lds32, int tid, uint32_t dom, uint32_t party, uint32_t group,
                                  uint32_t ct, const RoundConst &rc)
{
    for (int j = tid; j < ENG::NB / 4; j += ENG::T) {
        int32_t mu[4], e0[4], e1[4];
        ternary4(philox4x32_10(j, ct, party, counter_tag(dom, 0, group), rc.key), mu);
        cbd2(philox4x32_10(2 * j, ct, party, counter_tag(dom + 1, 0, group), rc.key), rc.eta_mask, e0);
        cbd2(philox4x32_10(2 * j + 1, ct, party, counter_tag(dom + 1, 0, group), rc.key), rc.eta_mask, e0 + 2);
        cbd2(philox4x32_10(2 * j, ct, party, counter_tag(dom + 2, 0, group), rc.key), rc.eta_mask, e1);
        cbd2(philox4x32_10(2 * j + 1, ct, party, counter_tag(dom + 2, 0, group), rc.key), rc.eta_mask, e1 + 2);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            lds32[4 * j + i] = ((uint32_t)mu[i] & 0xffu) | (((uint32_t)e0[i] & 0xffu) << 8) |
                               (((uint32_t)e1[i] & 0xffu) << 16);
    }
}

template <class ENG>
D2_DEV void stage_cbd(uint32_t *lds32, int tid, uint32_t domain, uint32_t party, uint32_t group, uint32_t ct,
                      const RoundConst &rc)
{
    for (int j = tid; j < ENG::NB / 2; j += ENG::T) {
        int32_t e[2];
        cbd2(philox4x32_10(j, ct, party, counter_tag(domain, 0, group), rc.key), rc.eta_mask, e);
        lds32[2 * j] = (uint32_t)e[0];
        lds32[2 * j + 1] = (uint32_t)e[1];
    }
}

D2_DEV int32_t sbyte(uint32_t w, int i) { return (int32_t)(int8_t)(w >> (8 * i)); }

// -------------------------------------------------------------------------------------
// Fixed point + slots (encode) as a device step: leaves the plaintext polynomial of
// ciphertext index c in registers in pass-0 (natural) ownership, values in [0, t).
// With rc.coeff_packing the values are the coefficients themselves (an addition-only workload
// never needs the slot structure): no transform on either side.
// `lds` must not have been used by the workgroup yet (no wave may still be reading it).
// -------------------------------------------------------------------------------------
template <class ENG>
D2_DEV void encode_to_regs(uint32_t (&m)[ENG::E], uint64_t *lds, int tid, const float *grad, uint64_t first,
                           uint64_t n_values, const LimbTab &tt, const RoundConst &rc)
{
    // the plaintext modulus is below 2^30: its transform runs on 32-bit residues whatever the context's
    // own arithmetic is (same thread shape and ownership)
    typedef typename ENG::template Rebind<Arith32> TE;
    typedef Arith32 A;
    const uint64_t t = tt.q;
    const typename A::Mod md = A::mod(t, tt.one_s);
    auto fixed = [&](uint64_t gi) -> uint64_t {          // value gi as a residue mod t
        float v = gi < n_values ? grad[gi] : 0.0f;
        float r = (v != v) ? 0.0f : __builtin_rintf(v * rc.scale);
        // The clamp bound (< 2^30) need not be a float once it exceeds 2^24: bring the rounded value into
        // the int32 range first (2^30 is a float), then compare as integers.
        r = r > 0x1p30f ? 0x1p30f : r;
        r = r < -0x1p30f ? -0x1p30f : r;
        int32_t z = (int32_t)r;
        z = z > rc.clamp ? rc.clamp : z;
        z = z < -rc.clamp ? -rc.clamp : z;
        return z >= 0 ? (uint64_t)z : t - (uint64_t)(uint32_t)(-z);
    };
    if (rc.coeff_packing) {                              // coefficient packing: no transform
#pragma unroll
        for (int k = 0; k < ENG::E; ++k) m[k] = (uint32_t)fixed(first + (uint64_t)ENG::coef_pos(k, tid));
        return;
    }
    // (no barrier in front of these writes: the callers have not used this buffer before)
    for (int j = tid; j < ENG::NB; j += ENG::T) lds[ENG::phys(j)] = fixed(first + (uint64_t)j);
    __syncthreads();
    // slot j is the evaluation xhat[j], which the engine keeps at block index bitrev(j)
    typename A::elem x[ENG::E];
#pragma unroll
    for (int k = 0; k < ENG::E; ++k)
        x[k] = A::inv_input(lds[ENG::phys((int)bitrev((uint32_t)(tid * ENG::E + k), ENG::LOGB))], md);
    TE::template inverse<true>(x, lds, tid, 0, tt.inv, md, A::tw(tt.ninv), A::tw(tt.wn));
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) m[k] = (uint32_t)A::canon_inv(x[k], md);
}

// registers hold a plaintext polynomial (natural ownership, [0,t)) -> floats
template <class ENG>
D2_DEV void decode_from_regs(uint32_t (&m)[ENG::E], uint64_t *lds, int tid, float *out, uint64_t first,
                             uint64_t n_values, const LimbTab &tt, const RoundConst &rc)
{
    typedef typename ENG::template Rebind<Arith32> TE;       // as in encode_to_regs
    typedef Arith32 A;
    const uint64_t t = tt.q;
    const typename A::Mod md = A::mod(t, tt.one_s);
    if (rc.coeff_packing) {                              // coefficient packing: no transform
#pragma unroll
        for (int k = 0; k < ENG::E; ++k) {
            const uint64_t gi = first + (uint64_t)ENG::coef_pos(k, tid), z = m[k];
            if (gi < n_values) {
                const int32_t c = z > (t - 1) / 2 ? (int32_t)((int64_t)z - (int64_t)t) : (int32_t)z;
                out[gi] = (float)c * rc.inv_scale;
            }
        }
        return;
    }
    typename A::elem x[ENG::E];
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) x[k] = A::from_canon((uint64_t)m[k], md);
    TE::forward(x, lds, tid, 0, tt.fwd, md);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < ENG::E; ++k)
        lds[ENG::phys((int)bitrev((uint32_t)(tid * ENG::E + k), ENG::LOGB))] = A::canon_fwd(x[k], md);
    __syncthreads();
    for (int j = tid; j < ENG::NB; j += ENG::T) {
        uint64_t gi = first + (uint64_t)j;
        if (gi < n_values) {
            uint64_t z = lds[ENG::phys(j)];
            int32_t c = z > (t - 1) / 2 ? (int32_t)((int64_t)z - (int64_t)t) : (int32_t)z;
            out[gi] = (float)c * rc.inv_scale;
        }
    }
}

template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_encode(const float *grad, uint64_t n_values, uint64_t *pt,
                                                   const LimbTab *tabs, RoundConst rc)
{
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    uint32_t m[ENG::E];
    encode_to_regs<ENG>(m, lds, tid, grad, (uint64_t)c * ENG::NB, n_values, load_tab(tabs, rc.L), rc);
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) pt[(size_t)c * ENG::NB + ENG::coef_pos(k, tid)] = m[k];
}

template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_decode(const uint64_t *pt, uint64_t n_values, float *out,
                                                   const LimbTab *tabs, RoundConst rc)
{
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    uint32_t m[ENG::E];
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) m[k] = (uint32_t)pt[(size_t)c * ENG::NB + ENG::coef_pos(k, tid)];
    decode_from_regs<ENG>(m, lds, tid, out, (uint64_t)c * ENG::NB, n_values, load_tab(tabs, rc.L), rc);
}

// -------------------------------------------------------------------------------------
// Set-up: one party's key share.  grid = L (one workgroup per limb).
//   sk (prepared): NTT(s) and Shoup quotients;  pk0 = -(p1 s + e) in evaluation form.
// p1 is the prepared common random polynomial.
// -------------------------------------------------------------------------------------
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_keygen(uint32_t party, uint64_t *sk, uint64_t *pk0, const uint64_t *p1,
                                                   const LimbTab *tabs, RoundConst rc)
{
    typedef typename ENG::A A;
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    uint32_t *lds32 = (uint32_t *)lds;
    const int tid = threadIdx.x;
    const uint32_t limb = blockIdx.x, L = rc.L;
    const LimbTab tb = load_tab(tabs, limb);
    const uint64_t q = tb.q;
    const typename A::Mod md = A::mod(q, tb.one_s);
    const size_t LN = (size_t)L * ENG::NB, off = (size_t)limb * ENG::NB;
    typename A::elem s[ENG::E], e[ENG::E];
    // secret share: ternary, counter (block, 0, party, SK)
    for (int j = tid; j < ENG::NB / 4; j += ENG::T) {
        int32_t v[4];
        ternary4(philox4x32_10(j, 0, party, counter_tag(DOM_SK, 0, 0), rc.key), v);
#pragma unroll
        for (int i = 0; i < 4; ++i) lds32[4 * j + i] = (uint32_t)v[i];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) s[k] = A::from_small((int32_t)lds32[ENG::coef_pos(k, tid)], md);
    __syncthreads();
    stage_cbd<ENG>(lds32, tid, DOM_PK_E, party, 0, 0, rc);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) e[k] = A::from_small((int32_t)lds32[ENG::coef_pos(k, tid)], md);
    ENG::forward(s, lds, tid, 0, tb.fwd, md);
    ENG::forward(e, lds, tid, 0, tb.fwd, md);
#pragma unroll
    for (int k = 0; k < ENG::E; ++k) {
        const int pos = ENG::eval_pos(k, tid);
        const uint64_t sv = A::canon_fwd(s[k], md);
        sk[off + pos] = sv;
        sk[LN + off + pos] = shoup_quotient(sv, q);
        const typename A::elem prod = A::mul(A::from_canon(sv, md), A::tw(p1[off + pos], p1[LN + off + pos]), md);
        const uint64_t sum = A::canon_acc(A::add(prod, e[k]), md);      // p1 s + e
        pk0[off + pos] = sum == 0 ? 0 : q - sum;
    }
}

// -------------------------------------------------------------------------------------
// dst = u * key + x, canonical, for the E slots of a thread (evaluation form, one limb).  u comes
// from registers (SRC_REGS: the lazy output of a transform), from raw bits parked at `src`
// (SRC_PARKED: such an output written out earlier; `src` may be `dst` itself) or from canonical
// words at `src` (SRC_CANON: a ciphertext component); x is a transform's lazy output; the key is a
// prepared polynomial (values kp, quotients kps).
// The order of the memory instructions is written out.  A wait for vector memory counts loads and
// stores together, in issue order: a load issued after a store cannot be waited for without also
// waiting for that store to reach memory, and the compiler never moves a load in front of a store
// that might alias it.  So the slots go in batches (sixteen key values and source words at once
// exceed the register budget), and the loads of a batch are issued before the stores of the
// previous one.
// -------------------------------------------------------------------------------------
// NEG: dst = x - u * key instead.
enum { SRC_REGS = 0, SRC_PARKED = 1, SRC_CANON = 2 };
template <class ENG, int SRC, bool NEG = false>
D2_DEV void mul_add_store(uint64_t *dst, const uint64_t *kp, const uint64_t *kps, const uint64_t *src,
                          const typename ENG::A::elem (&u)[ENG::E], const typename ENG::A::elem (&x)[ENG::E], int tl,
                          const typename ENG::A::Mod &md, uint64_t q = 0 /* the modulus, for NEG */)
{
    typedef typename ENG::A A;
    constexpr int E = ENG::E, BATCH = E < 8 ? E : 8, NB = E / BATCH;
    const uint32_t lo = 8u * (uint32_t)tl;
    typename A::Twid kv[BATCH];
    uint64_t ub[BATCH];
#pragma unroll
    for (int k = 0; k < BATCH; ++k) {
        kv[k] = A::key(kp, kps, lo, 8u * ENG::T * k);
        if constexpr (SRC != SRC_REGS) ub[k] = ld64(src, lo, 8u * ENG::T * k);
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        uint64_t r[BATCH];
#pragma unroll
        for (int k = 0; k < BATCH; ++k) {
            typename A::elem uu;
            if constexpr (SRC == SRC_PARKED) uu = from_bits<A>(ub[k]);
            else if constexpr (SRC == SRC_CANON) uu = A::from_canon(ub[k], md);
            else uu = u[b * BATCH + k];
            if constexpr (NEG) {
                const uint64_t prod = A::canon_acc(A::mul(uu, kv[k], md), md);
                r[k] = A::canon_acc(A::add(x[b * BATCH + k], A::from_canon(prod ? q - prod : 0, md)), md);
            } else {
                r[k] = A::canon_acc(A::add(A::mul(uu, kv[k], md), x[b * BATCH + k]), md);
            }
        }
        if (b + 1 < NB) {
#pragma unroll
            for (int k = 0; k < BATCH; ++k) {
                kv[k] = A::key(kp, kps, lo, 8u * ENG::T * ((b + 1) * BATCH + k));
                if constexpr (SRC != SRC_REGS) ub[k] = ld64(src, lo, 8u * ENG::T * ((b + 1) * BATCH + k));
            }
        }
#pragma unroll
        for (int k = 0; k < BATCH; ++k) st64_stream(dst, lo, 8u * ENG::T * (b * BATCH + k), r[k]);
    }
}

// -------------------------------------------------------------------------------------
// BFV.Encrypt in evaluation form.  grid = (C, jobs); one workgroup per ciphertext.
//   c0 = NTT(Lambda m + e0) + NTT(mu) * p0,   c1 = NTT(e1) + NTT(mu) * p1.
// FROM_FLOAT: the plaintext is encoded on the fly from the member's gradient;
// otherwise it is read from pt [C][N].
// -------------------------------------------------------------------------------------
template <class ENG, bool FROM_FLOAT>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_encrypt(EncJobs jobs, uint32_t ct_base, uint64_t n_values,
                                                    const LimbTab *tabs, RoundConst rc)
{
    typedef typename ENG::A A;
    typedef typename A::elem elem;
    __shared__ uint64_t lds[ENG::LDS_CHAIN_WORDS];
    uint32_t turn = 0;      // the buffer used last; the transforms take the two buffers in turn
    uint32_t *lds32 = (uint32_t *)lds;
    constexpr int E = ENG::E;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x, job = blockIdx.y, L = rc.L;
    const uint32_t party = jobs.party[job], group = jobs.group[job];
    const uint64_t *pk = jobs.pk[job];
    const size_t LN = (size_t)L * ENG::NB;
    uint64_t *out = jobs.out[job] + (size_t)c * 2 * LN;

    // With two buffers the samples are staged in the second one, next to the encoding in the first:
    // one barrier then makes them visible and also ends the encoding's reads of the first buffer,
    // which the first transform of the chain takes.
    uint32_t *stage = ENG::PINGPONG ? lds32 + 2 * ENG::LDS_WORDS : lds32;
    if (ENG::PINGPONG) {
        stage_encrypt_samples<ENG>(stage, tid, DOM_ENC_U, party, group, ct_base + c, rc);
        turn = 1;
    }
    uint32_t m[E];
    if (FROM_FLOAT) {
        encode_to_regs<ENG>(m, lds, tid, (const float *)jobs.src[job], (uint64_t)c * ENG::NB, n_values, load_tab(tabs, L), rc);
    } else {
        const uint64_t *pt = (const uint64_t *)jobs.src[job] + (size_t)c * ENG::NB;
#pragma unroll
        for (int k = 0; k < E; ++k) m[k] = (uint32_t)pt[ENG::coef_pos(k, tid)];
    }
    uint32_t smp[E];
    if (!ENG::PINGPONG) {
        __syncthreads();
        stage_encrypt_samples<ENG>(stage, tid, DOM_ENC_U, party, group, ct_base + c, rc);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < E; ++k) smp[k] = stage[ENG::coef_pos(k, tid)];

    for (uint32_t limb = 0; limb < L; ++limb) {
        const LimbTab tb = load_tab(tabs, limb);
        const typename A::Mod md = A::mod(tb.q, tb.one_s);
        const typename A::Twid lam = A::tw(tb.lambda);
        const size_t off = (size_t)limb * ENG::NB;
        const uint64_t *p0 = pk + off, *p0s = pk + LN + off;
        const uint64_t *p1 = pk + 2 * LN + off, *p1s = pk + 3 * LN + off;
        const int tl = opaque(tid);
        // With 16 coefficients per thread NTT(mu) is parked (lazy, as raw bits) in the c1 slot of the
        // output, which every thread re-reads at its own positions and overwrites last: keeping
        // it in 32 registers across the next two transforms would halve the occupancy.  With 8
        // per thread it stays in registers (no extra memory traffic).
        constexpr bool STASH = E > 8;
        uint64_t *stash = out + LN + off;
        elem u[E];
        int32_t sv[E];          // the samples of this transform as plain small integers
#pragma unroll
        for (int k = 0; k < E; ++k) sv[k] = sbyte(opaque(smp[k]), 0);
        ENG::forward_chained_small(sv, u, lds, turn, tl, tb.fwd, md);
        if (STASH) {
#pragma unroll
            for (int k = 0; k < E; ++k) st64(stash, 8u * (uint32_t)tl, 8u * ENG::T * k, to_bits<A>(u[k]));
        }
        elem x[E];
#pragma unroll
        for (int k = 0; k < E; ++k)
            x[k] = A::add_small(A::mul_u32(opaque(m[k]), lam, md), sbyte(opaque(smp[k]), 1), md);
        ENG::forward_chained(x, lds, turn, opaque(tl), 0, tb.fwd, md);
        mul_add_store<ENG, STASH ? SRC_PARKED : SRC_REGS>(out + off, p0, p0s, stash, u, x, tl, md);
#pragma unroll
        for (int k = 0; k < E; ++k) sv[k] = sbyte(opaque(smp[k]), 2);
        ENG::forward_chained_small(sv, x, lds, turn, opaque(tl), tb.fwd, md);
        mul_add_store<ENG, STASH ? SRC_PARKED : SRC_REGS>(stash, p1, p1s, stash, u, x, tl, md);
    }
}

// -------------------------------------------------------------------------------------
// Decryption share h = s c1 + e in evaluation form.  grid = (C, jobs).
// -------------------------------------------------------------------------------------
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_share(ShareJobs jobs, uint32_t ct_base, const LimbTab *tabs, RoundConst rc)
{
    typedef typename ENG::A A;
    __shared__ uint64_t lds[ENG::LDS_CHAIN_WORDS];
    uint32_t turn = 0;
    uint32_t *lds32 = (uint32_t *)lds;
    constexpr int E = ENG::E;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x, job = blockIdx.y, L = rc.L;
    const size_t LN = (size_t)L * ENG::NB;
    const uint64_t *sk = jobs.sk[job];
    const uint64_t *c1 = jobs.ct[job] + ((size_t)c * 2 + 1) * LN;
    uint64_t *out = jobs.out[job] + (size_t)c * LN;
    int e[E];
    stage_cbd<ENG>(lds32, tid, DOM_DEC_E, jobs.party[job], jobs.group[job], ct_base + c, rc);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < E; ++k) e[k] = (int)lds32[ENG::coef_pos(k, tid)];
    for (uint32_t limb = 0; limb < L; ++limb) {
        const LimbTab tb = load_tab(tabs, limb);
        const typename A::Mod md = A::mod(tb.q, tb.one_s);
        const size_t off = (size_t)limb * ENG::NB;
        const int tl = opaque(tid);
        typename A::elem x[E];
        int32_t sv[E];
#pragma unroll
        for (int k = 0; k < E; ++k) sv[k] = opaque(e[k]);
        ENG::forward_chained_small(sv, x, lds, turn, tl, tb.fwd, md);
        mul_add_store<ENG, SRC_CANON>(out + off, sk + off, sk + LN + off, c1 + off, x, x, tl, md);
    }
}

// -------------------------------------------------------------------------------------
// Combine: y = c0 + sum_k h_k, back to coefficient form, then pt = round(t y / Q) mod t
// by summing t * y_i' / q_i over the limbs with y_i' = y_i (Q/q_i)^-1 mod q_i: integer
// parts exactly, fractional parts in 64-bit fixed point (each term is truncated by less
// than 2^-63, so the rounding is exact unless t y / Q lies within L * 2^-63 of a half-integer).
// SH(j) returns the share buffer of member j.
// MODE 1 (MBFV.Convert, Eq. (2)): a share is a pair (h0, h1) [C][2][L][N] and the receiver's
// single-key decryption is folded in: y = c0 + sum h0_k + (z0 + sum h1_k) sk, where z0 = c1 of
// `ct` if keep_c1 (plain BFV.Decrypt of `ct` when K = 0) and 0 otherwise (the converted
// ciphertext drops the old c1).  aux: the receiver's prepared secret key.
// MODE 2 (MBFV.Bootstrap, Eq. (3)): a share is a pair (eta0, eta1); y = c0 + sum eta0_k is rounded
// to x in R_t, and the refreshed ciphertext (Lambda x + sum eta1_k, alpha) goes to ct_out.
// aux: alpha [C][L][N] in evaluation form.
// -------------------------------------------------------------------------------------
// One limb's term of round(t y / Q) = round(sum_i t y_i' / q_i): y_i' = y_i (Q/q_i)^-1 mod q_i, then
// y_i' * theta / 2^128 = integer part, next 64 bits = fraction (theta = floor(t 2^128 / q_i)); added to the
// running integer part and 64-bit fraction of a coefficient.
D2_DEV void scale_term(uint64_t y_canon, const LimbTab &tb, uint64_t &acc_int, uint64_t &acc_frac)
{
    const uint64_t yi = mul_shoup64(y_canon, tb.gamma.w, tb.gamma.ws, tb.q);
    uint64_t hi_lo = yi * tb.theta_hi, hi_hi = __umul64hi(yi, tb.theta_hi);
    uint64_t lo_hi = __umul64hi(yi, tb.theta_lo);
    uint64_t frac = hi_lo + lo_hi;
    uint64_t ip = hi_hi + (frac < hi_lo ? 1 : 0);
    uint64_t nf = acc_frac + frac;
    acc_int += ip + (nf < frac ? 1 : 0);
    acc_frac = nf;
}
// + 1/2, floor, mod t.  The sum is below (L + 1) t < 2^35: reduced in doubles (exact on integers; the
// quotient estimate can be off by one in either direction).
D2_DEV uint32_t round_mod_t(uint64_t acc_int, uint64_t acc_frac, const RoundConst &rc)
{
    const double td = (double)(uint32_t)rc.t, tinv = 1.0 / td;
    const uint64_t v = acc_int + (acc_frac >> 63);
    const double vd = (double)(uint32_t)v + 4294967296.0 * (double)(uint32_t)(v >> 32);
    double r = __builtin_fma(-__builtin_floor(vd * tinv), td, vd);
    r = r < 0.0 ? r + td : r;
    r = r >= td ? r - td : r;
    return (uint32_t)r;
}

enum { COMBINE_COLLECTIVE = 0, COMBINE_CONVERT = 1, COMBINE_BOOTSTRAP = 2 };
template <class ENG, bool DECODE, int MODE, class SH>
D2_DEV void combine_body(uint64_t *lds, const uint64_t *ct, SH share_of, uint32_t K, const uint64_t *aux,
                         bool keep_c1, uint64_t *pt, float *out, uint64_t n_values, const LimbTab *tabs,
                         const RoundConst &rc)
{
    constexpr bool CONVERT = MODE == COMBINE_CONVERT;
    const uint64_t *skr = aux;
    typedef typename ENG::A A;
    constexpr int E = ENG::E;
    const int tid = threadIdx.x;
    // ciphertext indices (and, in the whole-round kernels, jobs) from the last to the first: what the
    // share kernel wrote last is still in the memory-side cache
    const uint32_t c = gridDim.x - 1 - blockIdx.x, L = rc.L;
    const size_t LN = (size_t)L * ENG::NB;
    const size_t share_ct = (MODE == COMBINE_COLLECTIVE ? 1 : 2) * LN;       // words of one share per ciphertext index
    const uint64_t *c0 = ct + (size_t)c * 2 * LN;
    uint64_t acc_int[E], acc_frac[E];
#pragma unroll
    for (int k = 0; k < E; ++k) { acc_int[k] = 0; acc_frac[k] = 0; }
    for (uint32_t limb = 0; limb < L; ++limb) {
        const LimbTab tb = load_tab(tabs, limb);
        const uint64_t q = tb.q;
        const typename A::Mod md = A::mod(q, tb.one_s);
        const size_t off = (size_t)limb * ENG::NB;
        const int tl = opaque(tid);
        // c0 + sum of the shares, one batch of loads per member; with 8 coefficients per thread the
        // next member's values are already in flight while this one's are added
        constexpr bool PIPE = E <= 8 && !CONVERT;
        uint64_t y[E], hv[E];
#pragma unroll
        for (int k = 0; k < E; ++k) y[k] = ld64_stream(c0 + off, 8u * (uint32_t)tl, 8u * ENG::T * k);
        if (PIPE && K > 0) {
            const uint64_t *h = share_of(0) + (size_t)c * share_ct + off;
#pragma unroll
            for (int k = 0; k < E; ++k) hv[k] = ld64_stream(h, 8u * (uint32_t)tl, 8u * ENG::T * k);
        }
        for (uint32_t j = 0; j < K; ++j) {
            if constexpr (PIPE) {
                uint64_t nv[E];
                if (j + 1 < K) {
                    const uint64_t *h = share_of(j + 1) + (size_t)c * share_ct + off;
#pragma unroll
                    for (int k = 0; k < E; ++k) nv[k] = ld64_stream(h, 8u * (uint32_t)tl, 8u * ENG::T * k);
                }
#pragma unroll
                for (int k = 0; k < E; ++k) {
                    y[k] = add_mod(y[k], hv[k], q);
                    hv[k] = nv[k];
                }
            } else {
                const uint64_t *h = share_of(j) + (size_t)c * share_ct + off;
#pragma unroll
                for (int k = 0; k < E; ++k) hv[k] = ld64_stream(h, 8u * (uint32_t)tl, 8u * ENG::T * k);
#pragma unroll
                for (int k = 0; k < E; ++k) y[k] = add_mod(y[k], hv[k], q);
            }
        }
        typename A::elem x[E];
        if constexpr (CONVERT) {
            uint64_t z[E];
#pragma unroll
            for (int k = 0; k < E; ++k) z[k] = keep_c1 ? ld64_stream(c0 + LN + off, 8u * (uint32_t)tl, 8u * ENG::T * k) : 0;
            for (uint32_t j = 0; j < K; ++j) {
                const uint64_t *h = share_of(j) + (size_t)c * share_ct + LN + off;
#pragma unroll
                for (int k = 0; k < E; ++k) hv[k] = ld64_stream(h, 8u * (uint32_t)tl, 8u * ENG::T * k);
#pragma unroll
                for (int k = 0; k < E; ++k) z[k] = add_mod(z[k], hv[k], q);
            }
            typename A::Twid kv[E];
#pragma unroll
            for (int k = 0; k < E; ++k) kv[k] = A::key(skr + off, skr + LN + off, 8u * (uint32_t)tl, 8u * ENG::T * k);
#pragma unroll
            for (int k = 0; k < E; ++k) {
                const typename A::elem prod = A::mul(A::from_canon(z[k], md), kv[k], md);
                x[k] = A::inv_input(A::canon_acc(A::add(prod, A::from_canon(y[k], md)), md), md);
            }
        } else {
#pragma unroll
            for (int k = 0; k < E; ++k) x[k] = A::inv_input(y[k], md);
        }
        ENG::template inverse<true>(x, lds, tl, 0, tb.inv, md, A::tw(tb.ninv), A::tw(tb.wn));
#pragma unroll
        for (int k = 0; k < E; ++k) scale_term(A::canon_inv(x[k], md), tb, acc_int[k], acc_frac[k]);
    }
    uint32_t m[E];
#pragma unroll
    for (int k = 0; k < E; ++k) m[k] = round_mod_t(acc_int[k], acc_frac[k], rc);
    if constexpr (MODE == COMBINE_BOOTSTRAP) {
        // x sits where a forward transform takes its input: c0' = NTT(Lambda x) + sum eta1_k, c1' = alpha
        uint64_t *ct_out = pt + (size_t)c * 2 * LN;
        const uint64_t *alpha = aux + (size_t)c * LN;
        for (uint32_t limb = 0; limb < L; ++limb) {
            const LimbTab tb = load_tab(tabs, limb);
            const uint64_t q = tb.q;
            const typename A::Mod md = A::mod(q, tb.one_s);
            const typename A::Twid lam = A::tw(tb.lambda);
            const size_t off = (size_t)limb * ENG::NB;
            const int tl = opaque(tid);
            typename A::elem x[E];
#pragma unroll
            for (int k = 0; k < E; ++k) x[k] = A::mul_u32(opaque(m[k]), lam, md);
            ENG::forward(x, lds, tl, 0, tb.fwd, md);
            uint64_t y[E], hv[E];
#pragma unroll
            for (int k = 0; k < E; ++k) y[k] = A::canon_fwd(x[k], md);
            for (uint32_t j = 0; j < K; ++j) {
                const uint64_t *h = share_of(j) + (size_t)c * share_ct + LN + off;
#pragma unroll
                for (int k = 0; k < E; ++k) hv[k] = ld64_stream(h, 8u * (uint32_t)tl, 8u * ENG::T * k);
#pragma unroll
                for (int k = 0; k < E; ++k) y[k] = add_mod(y[k], hv[k], q);
            }
#pragma unroll
            for (int k = 0; k < E; ++k) {
                const uint32_t lo = 8u * (uint32_t)tl, so = 8u * ENG::T * k;
                st64(ct_out + off, lo, so, y[k]);
                st64(ct_out + LN + off, lo, so, ld64(alpha + off, lo, so));
            }
        }
    } else if (DECODE) {
        decode_from_regs<ENG>(m, lds, tid, out, (uint64_t)c * ENG::NB, n_values, load_tab(tabs, L), rc);
    } else {
#pragma unroll
        for (int k = 0; k < E; ++k) pt[(size_t)c * ENG::NB + ENG::coef_pos(k, tid)] = m[k];
    }
}

// one aggregate, K share buffers anywhere in memory, plaintext polynomials out; grid = C
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_combine(const uint64_t *ct, PtrList shares, uint32_t K, uint64_t *pt,
                                                    const LimbTab *tabs, RoundConst rc)
{
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    combine_body<ENG, false, COMBINE_COLLECTIVE>(lds, ct, [&](uint32_t j) { return (const uint64_t *)shares.p[j]; }, K,
                                    (const uint64_t *)nullptr, false, pt, (float *)nullptr, 0, tabs, rc);
}

// whole round: grid = (C, groups); the group's shares lie `stride` words apart; decoded floats out
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_combine_decode(GroupJobs jobs, size_t stride, uint64_t n_values,
                                                           const LimbTab *tabs, RoundConst rc)
{
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const uint32_t job = gridDim.y - 1 - blockIdx.y;
    const uint64_t *first = jobs.first[job];
    combine_body<ENG, true, COMBINE_COLLECTIVE>(lds, jobs.ct[job], [&](uint32_t j) { return first + (size_t)j * stride; },
                                   jobs.K[job], (const uint64_t *)nullptr, false, (uint64_t *)nullptr,
                                   (float *)jobs.out[job], n_values, tabs, rc);
}

// -------------------------------------------------------------------------------------
// MBFV.Convert (Sec. 4.2 item 3): key switching of an aggregate to a receiver's own key.
// -------------------------------------------------------------------------------------
// Set-up: a node's own single-key pair (Sec. 3.2 items 1-2).  grid = L.
//   sk (prepared) [2][L][N] = NTT(s), quotients;  pk (prepared) [2][2][L][N] = (p0, quotients,
//   p1, quotients) with p1 = NTT(a), a uniform in R_q, p0 = -(p1 s + e).
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_receiver_keygen(uint32_t party, uint64_t *sk, uint64_t *pk,
                                                            const LimbTab *tabs, RoundConst rc)
{
    typedef typename ENG::A A;
    constexpr int E = ENG::E;
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    uint32_t *lds32 = (uint32_t *)lds;
    const int tid = threadIdx.x;
    const uint32_t limb = blockIdx.x, L = rc.L;
    const LimbTab tb = load_tab(tabs, limb);
    const uint64_t q = tb.q;
    const typename A::Mod md = A::mod(q, tb.one_s);
    const size_t LN = (size_t)L * ENG::NB, off = (size_t)limb * ENG::NB;
    typename A::elem x[E];
    // secret key: ternary, counter (block, 0, party, RSK)
    for (int j = tid; j < ENG::NB / 4; j += ENG::T) {
        int32_t v[4];
        ternary4(philox4x32_10(j, 0, party, counter_tag(DOM_RSK, 0, 0), rc.key), v);
#pragma unroll
        for (int i = 0; i < 4; ++i) lds32[4 * j + i] = (uint32_t)v[i];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < E; ++k) x[k] = A::from_small((int32_t)lds32[ENG::coef_pos(k, tid)], md);
    ENG::forward(x, lds, tid, 0, tb.fwd, md);
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int pos = ENG::eval_pos(k, tid);
        const uint64_t sv = A::canon_fwd(x[k], md);
        sk[off + pos] = sv;
        sk[LN + off + pos] = shoup_quotient(sv, q);
    }
    // p1: coefficient n is block n of (RPK_A, limb) reduced mod q
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const uint32_t n = (uint32_t)ENG::coef_pos(k, tid);
        x[k] = A::from_canon(uniform_mod(philox4x32_10(n, 0, party, counter_tag(DOM_RPK_A, limb, 0), rc.key), tb), md);
    }
    ENG::forward(x, lds, tid, 0, tb.fwd, md);
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int pos = ENG::eval_pos(k, tid);
        const uint64_t av = A::canon_fwd(x[k], md);
        pk[2 * LN + off + pos] = av;
        pk[3 * LN + off + pos] = shoup_quotient(av, q);
    }
    // error, then p0 = -(p1 s + e) from the values this thread has just stored
    __syncthreads();
    stage_cbd<ENG>(lds32, tid, DOM_RPK_E, party, 0, 0, rc);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < E; ++k) x[k] = A::from_small((int32_t)lds32[ENG::coef_pos(k, tid)], md);
    ENG::forward(x, lds, tid, 0, tb.fwd, md);
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int pos = ENG::eval_pos(k, tid);
        const typename A::elem prod = A::mul(A::from_canon(sk[off + pos], md),
                                             A::tw(pk[2 * LN + off + pos], pk[3 * LN + off + pos]), md);
        const uint64_t sum = A::canon_acc(A::add(prod, x[k]), md);      // p1 s + e
        const uint64_t p0 = sum == 0 ? 0 : q - sum;
        pk[off + pos] = p0;
        pk[LN + off + pos] = shoup_quotient(p0, q);
    }
}

// A member's conversion share towards a receiver, Eq. (1), in evaluation form.  grid = (C, jobs).
//   h0 = s_k c1 + NTT(mu) p0_i + NTT(e0),   h1 = NTT(mu) p1_i + NTT(e1)
// mu ternary, e0, e1 from chi, counters (block, ciphertext, member | receiver << 16, domain | group << 16).
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_convert_share(ConvJobs jobs, uint32_t ct_base, const LimbTab *tabs,
                                                          RoundConst rc)
{
    typedef typename ENG::A A;
    typedef typename A::elem elem;
    __shared__ uint64_t lds[ENG::LDS_CHAIN_WORDS];
    uint32_t turn = 0;      // staging uses buffer 0; the transforms then take the two buffers in turn
    uint32_t *lds32 = (uint32_t *)lds;
    constexpr int E = ENG::E;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x, job = blockIdx.y, L = rc.L;
    const size_t LN = (size_t)L * ENG::NB;
    const uint64_t *sk = jobs.sk[job], *pk = jobs.pk[job];
    const uint64_t *c1 = jobs.ct[job] + ((size_t)c * 2 + 1) * LN;
    uint64_t *out = jobs.out[job] + (size_t)c * 2 * LN;
    uint32_t smp[E];
    stage_encrypt_samples<ENG>(lds32, tid, DOM_CVT_U, jobs.who[job], jobs.group[job], ct_base + c, rc);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < E; ++k) smp[k] = lds32[ENG::coef_pos(k, tid)];

    for (uint32_t limb = 0; limb < L; ++limb) {
        const LimbTab tb = load_tab(tabs, limb);
        const typename A::Mod md = A::mod(tb.q, tb.one_s);
        const size_t off = (size_t)limb * ENG::NB;
        const int tl = opaque(tid);
        // as in Encrypt: with 16 coefficients per thread NTT(mu) is parked in the h1 slot of the output
        constexpr bool STASH = E > 8;
        uint64_t *stash = out + LN + off;
        elem u[E];
        int32_t sv[E];
#pragma unroll
        for (int k = 0; k < E; ++k) sv[k] = sbyte(opaque(smp[k]), 0);
        ENG::forward_chained_small(sv, u, lds, turn, tl, tb.fwd, md);
        if (STASH) {
#pragma unroll
            for (int k = 0; k < E; ++k) st64(stash, 8u * (uint32_t)tl, 8u * ENG::T * k, to_bits<A>(u[k]));
        }
        elem x[E];
#pragma unroll
        for (int k = 0; k < E; ++k) sv[k] = sbyte(opaque(smp[k]), 1);
        ENG::forward_chained_small(sv, x, lds, turn, opaque(tl), tb.fwd, md);
        // h0: two products per slot, each reduced on its own; first x <- s c1 + x (loads only, eight slots at a time)
        constexpr int BATCH = E < 8 ? E : 8;
#pragma unroll
        for (int k0 = 0; k0 < E; k0 += BATCH) {
            typename A::Twid kv[BATCH];
            uint64_t cv[BATCH];
#pragma unroll
            for (int k = 0; k < BATCH; ++k) {
                kv[k] = A::key(sk + off, sk + LN + off, 8u * (uint32_t)tl, 8u * ENG::T * (k0 + k));
                cv[k] = ld64(c1 + off, 8u * (uint32_t)tl, 8u * ENG::T * (k0 + k));
            }
#pragma unroll
            for (int k = 0; k < BATCH; ++k)
                x[k0 + k] = A::from_canon(A::canon_acc(A::add(A::mul(A::from_canon(cv[k], md), kv[k], md), x[k0 + k]), md), md);
        }
        mul_add_store<ENG, STASH ? SRC_PARKED : SRC_REGS>(out + off, pk + off, pk + LN + off, stash, u, x, tl, md);
#pragma unroll
        for (int k = 0; k < E; ++k) sv[k] = sbyte(opaque(smp[k]), 2);
        ENG::forward_chained_small(sv, x, lds, turn, opaque(tl), tb.fwd, md);
        mul_add_store<ENG, STASH ? SRC_PARKED : SRC_REGS>(stash, pk + 2 * LN + off, pk + 3 * LN + off, stash, u, x, tl, md);
    }
}

// The receiver's side of MBFV.Convert fused with BFV.Decrypt(sk_i, .) (Eq. (2)); grid = C.
// Plaintext polynomials out.  K = 0 and keep_c1: plain single-key decryption of `ct`.
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_convert_combine(const uint64_t *ct, PtrList shares, uint32_t K,
                                                            const uint64_t *skr, int keep_c1, uint64_t *pt,
                                                            const LimbTab *tabs, RoundConst rc)
{
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    combine_body<ENG, false, COMBINE_CONVERT>(lds, ct, [&](uint32_t j) { return (const uint64_t *)shares.p[j]; }, K, skr,
                                   keep_c1 != 0, pt, (float *)nullptr, 0, tabs, rc);
}

// whole round: grid = (C, receivers of all groups); decoded floats out
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_convert_combine_decode(RecvJobs jobs, size_t stride,
                                                                   uint64_t n_values, const LimbTab *tabs,
                                                                   RoundConst rc)
{
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const uint32_t job = gridDim.y - 1 - blockIdx.y;
    const uint64_t *first = jobs.first[job];
    combine_body<ENG, true, COMBINE_CONVERT>(lds, jobs.ct[job], [&](uint32_t j) { return first + (size_t)j * stride; },
                                  jobs.K[job], jobs.sk[job], false, (uint64_t *)nullptr, (float *)jobs.out[job],
                                  n_values, tabs, rc);
}

// -------------------------------------------------------------------------------------
// MBFV.Bootstrap (Sec. 4.2 item 4): collective refresh of a ciphertext.
// -------------------------------------------------------------------------------------
// alpha of ciphertext indices ct_base .. ct_base + C - 1 of a group, evaluation form, [C][L][N].
// grid = (C, L).  Coefficient n of limb i = block n of (BS_A, limb i, group) reduced mod q_i.
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_bootstrap_alpha(uint64_t *alpha, uint32_t group, uint32_t ct_base,
                                                            const LimbTab *tabs, RoundConst rc)
{
    typedef typename ENG::A A;
    constexpr int E = ENG::E;
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x, limb = blockIdx.y, L = rc.L;
    const LimbTab tb = load_tab(tabs, limb);
    const typename A::Mod md = A::mod(tb.q, tb.one_s);
    typename A::elem x[E];
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const uint32_t n = (uint32_t)ENG::coef_pos(k, tid);
        x[k] = A::from_canon(uniform_mod(philox4x32_10(n, ct_base + c, 0, counter_tag(DOM_BS_A, limb, group), rc.key), tb), md);
    }
    ENG::forward(x, lds, tid, 0, tb.fwd, md);
    uint64_t *o = alpha + ((size_t)c * L + limb) * ENG::NB;
#pragma unroll
    for (int k = 0; k < E; ++k) st64(o, 8u * (uint32_t)tid, 8u * ENG::T * k, A::canon_fwd(x[k], md));
}

// A member's refresh share, Eq. (3), in evaluation form.  grid = (C, jobs); jobs.pk holds alpha.
//   eta0 = s_k c1 + NTT(e0 - Lambda M),   eta1 = NTT(Lambda M + e1) - s_k alpha
// M uniform mod t (one block per coefficient), e0, e1 from chi.
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_bootstrap_share(ConvJobs jobs, uint32_t ct_base, const LimbTab *tabs,
                                                            RoundConst rc)
{
    typedef typename ENG::A A;
    typedef typename A::elem elem;
    __shared__ uint64_t lds[ENG::LDS_CHAIN_WORDS];
    uint32_t turn = 0;      // staging uses buffer 0; the transforms then take the two buffers in turn
    uint32_t *lds32 = (uint32_t *)lds;
    constexpr int E = ENG::E;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x, job = blockIdx.y, L = rc.L;
    const size_t LN = (size_t)L * ENG::NB;
    const uint32_t party = jobs.who[job], group = jobs.group[job];
    const uint64_t *sk = jobs.sk[job];
    const uint64_t *alpha = jobs.pk[job] + (size_t)c * LN;
    const uint64_t *c1 = jobs.ct[job] + ((size_t)c * 2 + 1) * LN;
    uint64_t *out = jobs.out[job] + (size_t)c * 2 * LN;
    // staging: words [0, NB) the masks, words [NB, 2 NB) e0 | e1 << 8 (two's complement bytes)
    const LimbTab tt = load_tab(tabs, L);                 // the entry of the plaintext modulus
    for (int n = tid; n < ENG::NB; n += ENG::T)
        lds32[n] = (uint32_t)uniform_mod(philox4x32_10(n, ct_base + c, party, counter_tag(DOM_BS_M, 0, group), rc.key), tt);
    for (int j = tid; j < ENG::NB / 2; j += ENG::T) {
        int32_t e0[2], e1[2];
        cbd2(philox4x32_10(j, ct_base + c, party, counter_tag(DOM_BS_E0, 0, group), rc.key), rc.eta_mask, e0);
        cbd2(philox4x32_10(j, ct_base + c, party, counter_tag(DOM_BS_E1, 0, group), rc.key), rc.eta_mask, e1);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            lds32[ENG::NB + 2 * j + i] = ((uint32_t)e0[i] & 0xffu) | (((uint32_t)e1[i] & 0xffu) << 8);
    }
    __syncthreads();
    uint32_t mv[E], ev[E];
#pragma unroll
    for (int k = 0; k < E; ++k) {
        mv[k] = lds32[ENG::coef_pos(k, tid)];
        ev[k] = lds32[ENG::NB + ENG::coef_pos(k, tid)];
    }
    for (uint32_t limb = 0; limb < L; ++limb) {
        const LimbTab tb = load_tab(tabs, limb);
        const uint64_t q = tb.q;
        const typename A::Mod md = A::mod(q, tb.one_s);
        const typename A::Twid lam = A::tw(tb.lambda);
        const size_t off = (size_t)limb * ENG::NB;
        const int tl = opaque(tid);
        uint64_t lm[E];                                     // Lambda M mod q, canonical
#pragma unroll
        for (int k = 0; k < E; ++k) lm[k] = A::canon_acc(A::mul_u32(opaque(mv[k]), lam, md), md);
        elem x[E];
#pragma unroll
        for (int k = 0; k < E; ++k)
            x[k] = A::add(A::from_canon(lm[k] ? q - lm[k] : 0, md), A::from_small(sbyte(opaque(ev[k]), 0), md));
        ENG::forward_chained(x, lds, turn, tl, 0, tb.fwd, md);
        mul_add_store<ENG, SRC_CANON>(out + off, sk + off, sk + LN + off, c1 + off, x, x, tl, md);
#pragma unroll
        for (int k = 0; k < E; ++k)
            x[k] = A::add(A::from_canon(lm[k], md), A::from_small(sbyte(opaque(ev[k]), 1), md));
        ENG::forward_chained(x, lds, turn, opaque(tl), 0, tb.fwd, md);
        // eta1 = Lambda M + e1 - s_k alpha
        mul_add_store<ENG, SRC_CANON, true>(out + LN + off, sk + off, sk + LN + off, alpha + off, x, x, tl, md, q);
    }
}

// The receiver's side of MBFV.Bootstrap; grid = C.  ct_out [C][2][L][N].
template <class ENG>
__global__ void __launch_bounds__(ENG::T, ENG::WAVES) k_bootstrap_combine(const uint64_t *ct, PtrList shares, uint32_t K,
                                                              const uint64_t *alpha, uint64_t *ct_out,
                                                              const LimbTab *tabs, RoundConst rc)
{
    __shared__ uint64_t lds[ENG::LDS_WORDS];
    combine_body<ENG, false, COMBINE_BOOTSTRAP>(lds, ct, [&](uint32_t j) { return (const uint64_t *)shares.p[j]; }, K,
                                                alpha, false, ct_out, (float *)nullptr, 0, tabs, rc);
}

}  // namespace d2
