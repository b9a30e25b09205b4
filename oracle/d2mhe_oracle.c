/*
 * CPU oracle for the multiparty-BFV gradient exchange of D2-MHE (arXiv 2207.04604).
 * TEST INFRASTRUCTURE ONLY -- see d2mhe_oracle.h.  Written for clarity, not speed.
 */
#include "d2mhe_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef unsigned __int128 u128;

/* ------------------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as       */
/* 1, 2, 3", SC'11).  Ten rounds; the key is bumped after every round.                   */
/* ------------------------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void philox_block(uint64_t seed, uint32_t block, uint32_t ct, uint32_t party,
                         uint32_t domain, uint32_t limb, uint32_t group, uint32_t w[4])
{
    uint32_t ctr[4] = { block, ct, party, (domain & 0xffu) | ((limb & 0xffu) << 8) | (group << 16) };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    orc_philox4x32_10(ctr, key, w);
}

static int popcount32(uint32_t x)
{
    int c = 0;
    while (x) { c += (int)(x & 1u); x >>= 1; }
    return c;
}

/* Ternary coefficient n: word (n mod 4) of block floor(n/4); value floor(3w / 2^32) - 1. */
void orc_sample_ternary(uint64_t seed, uint32_t domain, uint32_t party, uint32_t group,
                        uint32_t ct, size_t n, int32_t *out)
{
    for (size_t i = 0; i < n; ++i) {
        uint32_t w[4];
        philox_block(seed, (uint32_t)(i >> 2), ct, party, domain, 0, group, w);
        out[i] = (int32_t)(((uint64_t)w[i & 3] * 3u) >> 32) - 1;
    }
}

/* Centred binomial coefficient n: words (2(n mod 2), 2(n mod 2)+1) of block floor(n/2);
 * value popcount(low eta bits of the first) - popcount(low eta bits of the second).     */
void orc_sample_cbd(uint64_t seed, uint32_t domain, uint32_t party, uint32_t group,
                    uint32_t ct, uint32_t eta, size_t n, int32_t *out)
{
    uint32_t mask = eta >= 32 ? 0xffffffffu : ((1u << eta) - 1u);
    for (size_t i = 0; i < n; ++i) {
        uint32_t w[4];
        philox_block(seed, (uint32_t)(i >> 1), ct, party, domain, 0, group, w);
        size_t j = 2 * (i & 1);
        out[i] = popcount32(w[j] & mask) - popcount32(w[j + 1] & mask);
    }
}

/* Uniform coefficient n: the 128-bit little-endian value of block n, reduced mod q.     */
void orc_sample_uniform(uint64_t seed, uint32_t domain, uint32_t limb, uint32_t party,
                        uint32_t group, uint32_t ct, uint64_t q, size_t n, uint64_t *out)
{
    for (size_t i = 0; i < n; ++i) {
        uint32_t w[4];
        philox_block(seed, (uint32_t)i, ct, party, domain, limb, group, w);
        u128 u = (u128)w[0] | ((u128)w[1] << 32) | ((u128)w[2] << 64) | ((u128)w[3] << 96);
        out[i] = (uint64_t)(u % q);
    }
}

/* ------------------------------------------------------------------------------------ */
/* Number theory                                                                        */
/* ------------------------------------------------------------------------------------ */
uint64_t orc_mulmod(uint64_t a, uint64_t b, uint64_t q) { return (uint64_t)(((u128)a * b) % q); }

static uint64_t addmod(uint64_t a, uint64_t b, uint64_t q) { return (uint64_t)(((u128)a + b) % q); }
static uint64_t submod(uint64_t a, uint64_t b, uint64_t q) { return (uint64_t)(((u128)a + q - b) % q); }

uint64_t orc_powmod(uint64_t a, uint64_t e, uint64_t q)
{
    uint64_t r = 1 % q;
    a %= q;
    while (e) {
        if (e & 1) r = orc_mulmod(r, a, q);
        a = orc_mulmod(a, a, q);
        e >>= 1;
    }
    return r;
}

static uint64_t invmod_prime(uint64_t a, uint64_t q) { return orc_powmod(a, q - 2, q); }

int orc_is_prime(uint64_t n)
{
    static const uint64_t bases[12] = { 2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37 };
    if (n < 2) return 0;
    for (int i = 0; i < 12; ++i) {
        if (n == bases[i]) return 1;
        if (n % bases[i] == 0) return 0;
    }
    uint64_t d = n - 1;
    int r = 0;
    while ((d & 1) == 0) { d >>= 1; ++r; }
    for (int i = 0; i < 12; ++i) {
        uint64_t x = orc_powmod(bases[i], d, n);
        if (x == 1 || x == n - 1) continue;
        int witness = 1;
        for (int j = 1; j < r; ++j) {
            x = orc_mulmod(x, x, n);
            if (x == n - 1) { witness = 0; break; }
        }
        if (witness) return 0;
    }
    return 1;
}

int orc_find_primes(uint32_t bits, uint32_t log2_n, int count, uint64_t *out)
{
    uint64_t two_n = (uint64_t)2 << log2_n;
    uint64_t top = (uint64_t)1 << bits;
    int found = 0;
    for (uint64_t k = 1; found < count && k * two_n < top; ++k) {
        uint64_t cand = top - k * two_n + 1;
        if (orc_is_prime(cand)) out[found++] = cand;
    }
    return found;
}

uint64_t orc_find_psi(uint64_t q, uint32_t log2_n)
{
    uint64_t n = (uint64_t)1 << log2_n;
    if ((q - 1) % (2 * n) != 0) return 0;
    for (uint64_t x = 2; x < q; ++x) {
        uint64_t psi = orc_powmod(x, (q - 1) / (2 * n), q);
        if (orc_powmod(psi, n, q) == q - 1) return psi;
    }
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Ring arithmetic in Z_q[X]/(X^n+1)                                                     */
/* ------------------------------------------------------------------------------------ */

/* (a*b)[k] = sum_{i+j=k} a_i b_j - sum_{i+j=k+n} a_i b_j, because X^n = -1.             */
void orc_negacyclic_schoolbook(const uint64_t *a, const uint64_t *b, size_t n, uint64_t q,
                               uint64_t *out)
{
    for (size_t k = 0; k < n; ++k) out[k] = 0;
    for (size_t i = 0; i < n; ++i) {
        for (size_t j = 0; j < n; ++j) {
            uint64_t p = orc_mulmod(a[i], b[j], q);
            size_t k = i + j;
            if (k < n) out[k] = addmod(out[k], p, q);
            else out[k - n] = submod(out[k - n], p, q);
        }
    }
}

void orc_ntt_definition(const uint64_t *x, size_t n, uint64_t q, uint64_t psi, uint64_t *out)
{
    for (size_t j = 0; j < n; ++j) {
        uint64_t root = orc_powmod(psi, 2 * j + 1, q); /* psi^(2j+1) */
        uint64_t acc = 0, pw = 1;
        for (size_t i = 0; i < n; ++i) {
            acc = addmod(acc, orc_mulmod(x[i], pw, q), q);
            pw = orc_mulmod(pw, root, q);
        }
        out[j] = acc;
    }
}

static size_t bit_reverse(size_t v, unsigned bits)
{
    size_t r = 0;
    for (unsigned i = 0; i < bits; ++i) { r = (r << 1) | (v & 1); v >>= 1; }
    return r;
}

/* Textbook in-place cyclic transform X[j] = sum_n x[n] w^(jn): bit-reversal permutation
 * followed by log2(n) rounds of decimation-in-time butterflies.                         */
static void cyclic_ntt(uint64_t *x, size_t n, uint64_t q, uint64_t w)
{
    unsigned bits = 0;
    while (((size_t)1 << bits) < n) ++bits;
    for (size_t i = 0; i < n; ++i) {
        size_t j = bit_reverse(i, bits);
        if (i < j) { uint64_t tmp = x[i]; x[i] = x[j]; x[j] = tmp; }
    }
    for (size_t len = 2; len <= n; len <<= 1) {
        uint64_t wlen = orc_powmod(w, n / len, q);
        for (size_t start = 0; start < n; start += len) {
            uint64_t wk = 1;
            for (size_t k = 0; k < len / 2; ++k) {
                uint64_t u = x[start + k];
                uint64_t v = orc_mulmod(x[start + k + len / 2], wk, q);
                x[start + k] = addmod(u, v, q);
                x[start + k + len / 2] = submod(u, v, q);
                wk = orc_mulmod(wk, wlen, q);
            }
        }
    }
}

/* psi^((2j+1) n) = psi^n * (psi^2)^(jn): twist by psi^n, then a cyclic transform.       */
void orc_ntt_forward(uint64_t *x, size_t n, uint64_t q, uint64_t psi)
{
    uint64_t pw = 1;
    for (size_t i = 0; i < n; ++i) {
        x[i] = orc_mulmod(x[i], pw, q);
        pw = orc_mulmod(pw, psi, q);
    }
    cyclic_ntt(x, n, q, orc_mulmod(psi, psi, q));
}

void orc_ntt_inverse(uint64_t *x, size_t n, uint64_t q, uint64_t psi)
{
    uint64_t psi_inv = invmod_prime(psi, q);
    uint64_t n_inv = invmod_prime((uint64_t)n % q, q);
    cyclic_ntt(x, n, q, orc_mulmod(psi_inv, psi_inv, q));
    uint64_t pw = n_inv;
    for (size_t i = 0; i < n; ++i) {
        x[i] = orc_mulmod(x[i], pw, q);
        pw = orc_mulmod(pw, psi_inv, q);
    }
}

void orc_ring_mul(const uint64_t *a, const uint64_t *b, size_t n, uint64_t q, uint64_t psi,
                  uint64_t *out)
{
    uint64_t *fa = (uint64_t *)malloc(n * sizeof(uint64_t));
    uint64_t *fb = (uint64_t *)malloc(n * sizeof(uint64_t));
    memcpy(fa, a, n * sizeof(uint64_t));
    memcpy(fb, b, n * sizeof(uint64_t));
    orc_ntt_forward(fa, n, q, psi);
    orc_ntt_forward(fb, n, q, psi);
    for (size_t i = 0; i < n; ++i) fa[i] = orc_mulmod(fa[i], fb[i], q);
    orc_ntt_inverse(fa, n, q, psi);
    memcpy(out, fa, n * sizeof(uint64_t));
    free(fa);
    free(fb);
}

/* ------------------------------------------------------------------------------------ */
/* A small unsigned multi-word integer (little-endian 32-bit words), enough for          */
/* 2 t y + Q with Q up to 16 limbs of 61 bits.                                           */
/* ------------------------------------------------------------------------------------ */
#define BIG_WORDS 40
typedef struct { uint32_t w[BIG_WORDS]; } big_t;

static void big_set_u64(big_t *a, uint64_t v)
{
    memset(a, 0, sizeof(*a));
    a->w[0] = (uint32_t)v;
    a->w[1] = (uint32_t)(v >> 32);
}

static void big_mul_u64(big_t *a, uint64_t m) /* a *= m */
{
    uint32_t mlo = (uint32_t)m, mhi = (uint32_t)(m >> 32);
    big_t lo, hi;
    uint64_t carry = 0;
    for (int i = 0; i < BIG_WORDS; ++i) {
        uint64_t p = (uint64_t)a->w[i] * mlo + carry;
        lo.w[i] = (uint32_t)p;
        carry = p >> 32;
    }
    carry = 0;
    hi.w[0] = 0;
    for (int i = 0; i + 1 < BIG_WORDS; ++i) {
        uint64_t p = (uint64_t)a->w[i] * mhi + carry;
        hi.w[i + 1] = (uint32_t)p;
        carry = p >> 32;
    }
    carry = 0;
    for (int i = 0; i < BIG_WORDS; ++i) {
        uint64_t s = (uint64_t)lo.w[i] + hi.w[i] + carry;
        a->w[i] = (uint32_t)s;
        carry = s >> 32;
    }
}

static void big_add(big_t *a, const big_t *b) /* a += b */
{
    uint64_t carry = 0;
    for (int i = 0; i < BIG_WORDS; ++i) {
        uint64_t s = (uint64_t)a->w[i] + b->w[i] + carry;
        a->w[i] = (uint32_t)s;
        carry = s >> 32;
    }
}

static void big_sub(big_t *a, const big_t *b) /* a -= b, requires a >= b */
{
    int64_t borrow = 0;
    for (int i = 0; i < BIG_WORDS; ++i) {
        int64_t d = (int64_t)a->w[i] - (int64_t)b->w[i] - borrow;
        borrow = d < 0;
        a->w[i] = (uint32_t)(d + (borrow ? ((int64_t)1 << 32) : 0));
    }
}

static int big_cmp(const big_t *a, const big_t *b)
{
    for (int i = BIG_WORDS - 1; i >= 0; --i) {
        if (a->w[i] != b->w[i]) return a->w[i] < b->w[i] ? -1 : 1;
    }
    return 0;
}

static uint64_t big_mod_u64(const big_t *a, uint64_t m)
{
    u128 r = 0;
    for (int i = BIG_WORDS - 1; i >= 0; --i) r = ((r << 32) | a->w[i]) % m;
    return (uint64_t)r;
}

static void big_div_u64(big_t *a, uint64_t m) /* a = floor(a / m) */
{
    u128 r = 0;
    for (int i = BIG_WORDS - 1; i >= 0; --i) {
        u128 cur = (r << 32) | a->w[i];
        a->w[i] = (uint32_t)(cur / m);
        r = cur % m;
    }
}

static unsigned big_bits(const big_t *a)
{
    for (int i = BIG_WORDS - 1; i >= 0; --i) {
        if (a->w[i]) {
            unsigned b = 0;
            uint32_t v = a->w[i];
            while (v) { ++b; v >>= 1; }
            return (unsigned)i * 32u + b;
        }
    }
    return 0;
}

static void big_shl(big_t *a, unsigned s) /* a <<= s */
{
    unsigned ws = s / 32, bs = s % 32;
    big_t r;
    memset(&r, 0, sizeof(r));
    for (int i = BIG_WORDS - 1; i >= (int)ws; --i) {
        uint64_t v = (uint64_t)a->w[i - ws] << bs;
        if (bs && i - (int)ws - 1 >= 0) v |= a->w[i - ws - 1] >> (32 - bs);
        r.w[i] = (uint32_t)v;
    }
    *a = r;
}

/* floor(a / b) for a quotient known to fit 64 bits: binary long division.               */
static uint64_t big_div_small_quotient(const big_t *a, const big_t *b)
{
    big_t rem = *a;
    unsigned ba = big_bits(a), bb = big_bits(b);
    if (bb == 0 || ba < bb) return 0;
    uint64_t quo = 0;
    for (int s = (int)(ba - bb); s >= 0; --s) {
        big_t shifted = *b;
        big_shl(&shifted, (unsigned)s);
        if (big_cmp(&shifted, &rem) <= 0) {
            big_sub(&rem, &shifted);
            quo |= (uint64_t)1 << s;
        }
    }
    return quo;
}

/* ------------------------------------------------------------------------------------ */
/* Scheme context                                                                       */
/* ------------------------------------------------------------------------------------ */
struct orc_ctx {
    orc_params p;
    size_t n;
    uint64_t psi[ORC_MAX_LIMBS];
    uint64_t psi_t;
    big_t Q;                              /* prod q_i                                   */
    big_t two_Q;
    big_t Lambda;                         /* floor(Q / t)                               */
    uint64_t lambda_mod_q[ORC_MAX_LIMBS]; /* Lambda mod q_i                             */
    big_t Q_over_qi[ORC_MAX_LIMBS];       /* Q / q_i                                    */
    uint64_t Q_over_qi_inv[ORC_MAX_LIMBS]; /* (Q / q_i)^-1 mod q_i                       */
    int64_t clamp;                        /* floor(((t-1)/2) / K_max)                   */
};

orc_ctx *orc_create(const orc_params *p)
{
    if (!p || p->log2_n < 1 || p->log2_n > 20 || p->num_limbs < 1 || p->num_limbs > ORC_MAX_LIMBS)
        return NULL;
    uint64_t two_n = (uint64_t)2 << p->log2_n;
    for (uint32_t i = 0; i < p->num_limbs; ++i) {
        if (p->q[i] >> 61) return NULL;
        if (!orc_is_prime(p->q[i]) || (p->q[i] - 1) % two_n != 0) return NULL;
        for (uint32_t j = 0; j < i; ++j)
            if (p->q[i] == p->q[j]) return NULL;
        if (p->t && p->t >= p->q[i]) return NULL;
    }
    if (p->t && (!orc_is_prime(p->t) || (p->t - 1) % two_n != 0)) return NULL;
    if (p->cbd_eta < 1 || p->cbd_eta > 32) return NULL;

    orc_ctx *c = (orc_ctx *)calloc(1, sizeof(orc_ctx));
    c->p = *p;
    c->n = (size_t)1 << p->log2_n;
    for (uint32_t i = 0; i < p->num_limbs; ++i) c->psi[i] = orc_find_psi(p->q[i], p->log2_n);
    big_set_u64(&c->Q, 1);
    for (uint32_t i = 0; i < p->num_limbs; ++i) big_mul_u64(&c->Q, p->q[i]);
    c->two_Q = c->Q;
    big_add(&c->two_Q, &c->Q);
    for (uint32_t i = 0; i < p->num_limbs; ++i) {
        big_set_u64(&c->Q_over_qi[i], 1);
        for (uint32_t j = 0; j < p->num_limbs; ++j)
            if (j != i) big_mul_u64(&c->Q_over_qi[i], p->q[j]);
        c->Q_over_qi_inv[i] = invmod_prime(big_mod_u64(&c->Q_over_qi[i], p->q[i]), p->q[i]);
    }
    if (p->t) {
        c->psi_t = orc_find_psi(p->t, p->log2_n);
        c->Lambda = c->Q;
        big_div_u64(&c->Lambda, p->t);
        for (uint32_t i = 0; i < p->num_limbs; ++i)
            c->lambda_mod_q[i] = big_mod_u64(&c->Lambda, p->q[i]);
        uint32_t kmax = p->max_group ? p->max_group : 1;
        c->clamp = (int64_t)(((p->t - 1) / 2) / kmax);
    }
    return c;
}

void orc_destroy(orc_ctx *c) { free(c); }
uint64_t orc_psi(const orc_ctx *c, uint32_t limb) { return c->psi[limb]; }
uint64_t orc_psi_t(const orc_ctx *c) { return c->psi_t; }
uint64_t orc_lambda_mod_q(const orc_ctx *c, uint32_t limb) { return c->lambda_mod_q[limb]; }
uint64_t orc_q_mod_t(const orc_ctx *c) { return big_mod_u64(&c->Q, c->p.t); }
uint32_t orc_lambda_bits(const orc_ctx *c) { return big_bits(&c->Lambda); }
int64_t orc_encode_clamp(const orc_ctx *c) { return c->clamp; }

/* A small signed value v enters limb i as v (v >= 0) or q_i + v (v < 0).                */
static uint64_t lift_small(int32_t v, uint64_t q) { return v >= 0 ? (uint64_t)v : q - (uint64_t)(-(int64_t)v); }

void orc_crs(const orc_ctx *c, uint64_t *p1)
{
    for (uint32_t i = 0; i < c->p.num_limbs; ++i)
        orc_sample_uniform(c->p.seed, ORC_DOM_CRS, i, 0, 0, 0, c->p.q[i], c->n, p1 + (size_t)i * c->n);
}

void orc_keygen_share(const orc_ctx *c, uint32_t party, uint64_t *sk, uint64_t *pk0_share,
                      int32_t *sk_small, int32_t *e_small)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    int32_t *s = (int32_t *)malloc(n * sizeof(int32_t));
    int32_t *e = (int32_t *)malloc(n * sizeof(int32_t));
    uint64_t *p1 = (uint64_t *)malloc((size_t)L * n * sizeof(uint64_t));
    uint64_t *prod = (uint64_t *)malloc(n * sizeof(uint64_t));
    orc_sample_ternary(c->p.seed, ORC_DOM_SK, party, 0, 0, n, s);
    orc_sample_cbd(c->p.seed, ORC_DOM_PK_E, party, 0, 0, c->p.cbd_eta, n, e);
    orc_crs(c, p1);
    for (uint32_t i = 0; i < L; ++i) {
        uint64_t q = c->p.q[i];
        uint64_t *ski = sk + (size_t)i * n;
        for (size_t k = 0; k < n; ++k) ski[k] = lift_small(s[k], q);
        orc_ring_mul(p1 + (size_t)i * n, ski, n, q, c->psi[i], prod);
        for (size_t k = 0; k < n; ++k) {
            uint64_t v = addmod(prod[k], lift_small(e[k], q), q); /* p1 s_k + e_k */
            pk0_share[(size_t)i * n + k] = submod(0, v, q);       /* negated      */
        }
    }
    if (sk_small) memcpy(sk_small, s, n * sizeof(int32_t));
    if (e_small) memcpy(e_small, e, n * sizeof(int32_t));
    free(s); free(e); free(p1); free(prod);
}

void orc_aggregate_pk(const orc_ctx *c, const uint64_t *const *pk0_shares, uint32_t K,
                      uint64_t *pk)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    for (uint32_t i = 0; i < L; ++i) {
        uint64_t q = c->p.q[i];
        for (size_t k = 0; k < n; ++k) {
            uint64_t acc = 0;
            for (uint32_t m = 0; m < K; ++m) acc = addmod(acc, pk0_shares[m][(size_t)i * n + k], q);
            pk[(size_t)i * n + k] = acc;
        }
    }
    orc_crs(c, pk + (size_t)L * n);
}

/* Fixed point: r = rint(v 2^f) in float32 (ties to even), NaN -> 0, clamped so that a sum
 * of K_max values cannot wrap mod t; z = r mod t.  Slot j of plaintext c holds value
 * c N + j; the plaintext polynomial m has m(psi_t^(2j+1)) = z[j].                        */
int orc_encode(const orc_ctx *c, const float *grad, uint64_t n_values, uint64_t *pt, uint32_t C)
{
    size_t n = c->n;
    uint64_t t = c->p.t;
    if (!t || n_values > (uint64_t)C * n) return -1;
    float scale = ldexpf(1.0f, (int)c->p.frac_bits);
    /* the clamp is applied to the rounded value as an exact comparison (in double, which holds
     * every float and every bound below 2^53): a bound above 2^24 need not be a float32          */
    double bound = (double)c->clamp;
    for (uint32_t ci = 0; ci < C; ++ci) {
        uint64_t *z = pt + (size_t)ci * n;
        for (size_t j = 0; j < n; ++j) {
            uint64_t idx = (uint64_t)ci * n + j;
            int64_t r = 0;
            if (idx < n_values) {
                float v = grad[idx];
                double rf = isnan(v) ? 0.0 : (double)rintf(v * scale);
                if (rf > bound) rf = bound;
                if (rf < -bound) rf = -bound;
                r = (int64_t)rf;
            }
            z[j] = r >= 0 ? (uint64_t)r : t - (uint64_t)(-r);
        }
        orc_ntt_inverse(z, n, t, c->psi_t);
    }
    return 0;
}

int orc_decode(const orc_ctx *c, const uint64_t *pt, uint32_t C, uint64_t n_values, float *out)
{
    size_t n = c->n;
    uint64_t t = c->p.t;
    if (!t || n_values > (uint64_t)C * n) return -1;
    uint64_t *z = (uint64_t *)malloc(n * sizeof(uint64_t));
    for (uint32_t ci = 0; ci < C; ++ci) {
        memcpy(z, pt + (size_t)ci * n, n * sizeof(uint64_t));
        orc_ntt_forward(z, n, t, c->psi_t);
        for (size_t j = 0; j < n; ++j) {
            uint64_t idx = (uint64_t)ci * n + j;
            if (idx >= n_values) break;
            int64_t v = z[j] > (t - 1) / 2 ? (int64_t)z[j] - (int64_t)t : (int64_t)z[j];
            out[idx] = ldexpf((float)v, -(int)c->p.frac_bits);
        }
    }
    free(z);
    return 0;
}

/* The same fixed point without the slot transform: value c N + j is coefficient j.          */
int orc_encode_coefficients(const orc_ctx *c, const float *grad, uint64_t n_values, uint64_t *pt,
                            uint32_t C)
{
    size_t n = c->n;
    uint64_t t = c->p.t;
    if (!t || n_values > (uint64_t)C * n) return -1;
    float scale = ldexpf(1.0f, (int)c->p.frac_bits);
    double bound = (double)c->clamp;      /* exact comparison, as in orc_encode */
    for (uint64_t idx = 0; idx < (uint64_t)C * n; ++idx) {
        int64_t r = 0;
        if (idx < n_values) {
            float v = grad[idx];
            double rf = isnan(v) ? 0.0 : (double)rintf(v * scale);
            if (rf > bound) rf = bound;
            if (rf < -bound) rf = -bound;
            r = (int64_t)rf;
        }
        pt[idx] = r >= 0 ? (uint64_t)r : t - (uint64_t)(-r);
    }
    return 0;
}

int orc_decode_coefficients(const orc_ctx *c, const uint64_t *pt, uint32_t C, uint64_t n_values,
                            float *out)
{
    uint64_t t = c->p.t;
    if (!t || n_values > (uint64_t)C * c->n) return -1;
    for (uint64_t idx = 0; idx < n_values; ++idx) {
        int64_t v = pt[idx] > (t - 1) / 2 ? (int64_t)pt[idx] - (int64_t)t : (int64_t)pt[idx];
        out[idx] = ldexpf((float)v, -(int)c->p.frac_bits);
    }
    return 0;
}

/* BFV.Encrypt: ct = (Lambda x + mu p0 + e0, mu p1 + e1), mu ternary, e0, e1 from chi.    */
void orc_encrypt(const orc_ctx *c, const uint64_t *pk, const uint64_t *pt, uint32_t C,
                 uint32_t party, uint32_t group, uint32_t ct_base, uint64_t *ct)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    int32_t *mu = (int32_t *)malloc(n * sizeof(int32_t));
    int32_t *e0 = (int32_t *)malloc(n * sizeof(int32_t));
    int32_t *e1 = (int32_t *)malloc(n * sizeof(int32_t));
    uint64_t *mu_q = (uint64_t *)malloc(n * sizeof(uint64_t));
    uint64_t *prod = (uint64_t *)malloc(n * sizeof(uint64_t));
    for (uint32_t ci = 0; ci < C; ++ci) {
        uint32_t index = ct_base + ci;
        orc_sample_ternary(c->p.seed, ORC_DOM_ENC_U, party, group, index, n, mu);
        orc_sample_cbd(c->p.seed, ORC_DOM_ENC_E0, party, group, index, c->p.cbd_eta, n, e0);
        orc_sample_cbd(c->p.seed, ORC_DOM_ENC_E1, party, group, index, c->p.cbd_eta, n, e1);
        const uint64_t *m = pt + (size_t)ci * n;
        uint64_t *c0 = ct + (size_t)ci * 2 * L * n;
        uint64_t *c1 = c0 + (size_t)L * n;
        for (uint32_t i = 0; i < L; ++i) {
            uint64_t q = c->p.q[i];
            const uint64_t *p0 = pk + (size_t)i * n;
            const uint64_t *p1 = pk + (size_t)(L + i) * n;
            for (size_t k = 0; k < n; ++k) mu_q[k] = lift_small(mu[k], q);
            orc_ring_mul(mu_q, p0, n, q, c->psi[i], prod);
            for (size_t k = 0; k < n; ++k) {
                uint64_t lm = orc_mulmod(c->lambda_mod_q[i], m[k] % q, q);
                c0[(size_t)i * n + k] = addmod(addmod(lm, prod[k], q), lift_small(e0[k], q), q);
            }
            orc_ring_mul(mu_q, p1, n, q, c->psi[i], prod);
            for (size_t k = 0; k < n; ++k)
                c1[(size_t)i * n + k] = addmod(prod[k], lift_small(e1[k], q), q);
        }
    }
    free(mu); free(e0); free(e1); free(mu_q); free(prod);
}

void orc_add(const orc_ctx *c, uint64_t *acc, const uint64_t *in, uint32_t C)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    for (uint32_t ci = 0; ci < C; ++ci)
        for (uint32_t comp = 0; comp < 2; ++comp)
            for (uint32_t i = 0; i < L; ++i) {
                size_t off = (((size_t)ci * 2 + comp) * L + i) * n;
                for (size_t k = 0; k < n; ++k) acc[off + k] = addmod(acc[off + k], in[off + k], c->p.q[i]);
            }
}

/* Share of the collective decryption: h_k = s_k c1 + e_k.                               */
void orc_partial_decrypt(const orc_ctx *c, const uint64_t *sk, const uint64_t *ct, uint32_t C,
                         uint32_t party, uint32_t group, uint32_t ct_base, uint64_t *share)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    int32_t *e = (int32_t *)malloc(n * sizeof(int32_t));
    uint64_t *prod = (uint64_t *)malloc(n * sizeof(uint64_t));
    for (uint32_t ci = 0; ci < C; ++ci) {
        orc_sample_cbd(c->p.seed, ORC_DOM_DEC_E, party, group, ct_base + ci, c->p.cbd_eta, n, e);
        const uint64_t *c1 = ct + ((size_t)ci * 2 + 1) * L * n;
        for (uint32_t i = 0; i < L; ++i) {
            uint64_t q = c->p.q[i];
            orc_ring_mul(sk + (size_t)i * n, c1 + (size_t)i * n, n, q, c->psi[i], prod);
            for (size_t k = 0; k < n; ++k)
                share[((size_t)ci * L + i) * n + k] = addmod(prod[k], lift_small(e[k], q), q);
        }
    }
    free(e); free(prod);
}

/* round(t y / Q) mod t for y given by its residues: lift y to [0,Q) by the Chinese
 * remainder theorem, then floor((2 t y + Q) / (2 Q)) with multi-word integers.          */
static uint64_t scale_round(const orc_ctx *c, const uint64_t *res)
{
    uint32_t L = c->p.num_limbs;
    big_t y;
    big_set_u64(&y, 0);
    for (uint32_t i = 0; i < L; ++i) {
        big_t term = c->Q_over_qi[i];
        big_mul_u64(&term, orc_mulmod(res[i], c->Q_over_qi_inv[i], c->p.q[i]));
        big_add(&y, &term);
    }
    while (big_cmp(&y, &c->Q) >= 0) big_sub(&y, &c->Q);
    big_mul_u64(&y, 2 * c->p.t);
    big_add(&y, &c->Q);
    return big_div_small_quotient(&y, &c->two_Q) % c->p.t;
}

void orc_combine(const orc_ctx *c, const uint64_t *ct, const uint64_t *const *shares,
                 uint32_t K, uint32_t C, uint64_t *pt)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    for (uint32_t ci = 0; ci < C; ++ci) {
        const uint64_t *c0 = ct + (size_t)ci * 2 * L * n;
        for (size_t k = 0; k < n; ++k) {
            uint64_t res[ORC_MAX_LIMBS];
            for (uint32_t i = 0; i < L; ++i) {
                uint64_t acc = c0[(size_t)i * n + k];
                for (uint32_t m = 0; m < K; ++m)
                    acc = addmod(acc, shares[m][((size_t)ci * L + i) * n + k], c->p.q[i]);
                res[i] = acc;
            }
            pt[(size_t)ci * n + k] = scale_round(c, res);
        }
    }
}

/* BFV.Decrypt: x = [round(t/q [c0 + c1 s]_q)]_t.                                         */
void orc_decrypt_with_secret(const orc_ctx *c, const uint64_t *s, const uint64_t *ct,
                             uint32_t C, uint64_t *pt)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    uint64_t *y = (uint64_t *)malloc((size_t)L * n * sizeof(uint64_t));
    for (uint32_t ci = 0; ci < C; ++ci) {
        const uint64_t *c0 = ct + (size_t)ci * 2 * L * n;
        const uint64_t *c1 = c0 + (size_t)L * n;
        for (uint32_t i = 0; i < L; ++i) {
            uint64_t q = c->p.q[i];
            orc_ring_mul(c1 + (size_t)i * n, s + (size_t)i * n, n, q, c->psi[i], y + (size_t)i * n);
            for (size_t k = 0; k < n; ++k)
                y[(size_t)i * n + k] = addmod(y[(size_t)i * n + k], c0[(size_t)i * n + k], q);
        }
        for (size_t k = 0; k < n; ++k) {
            uint64_t res[ORC_MAX_LIMBS];
            for (uint32_t i = 0; i < L; ++i) res[i] = y[(size_t)i * n + k];
            pt[(size_t)ci * n + k] = scale_round(c, res);
        }
    }
    free(y);
}

/* ---- MBFV.Convert (Sec. 4.2 item 3, Eq. (1)-(2)) ---- */

/* BFV.SecKeyGen and BFV.PubKeyGen of one node (Sec. 3.2 items 1-2).                      */
void orc_receiver_keygen(const orc_ctx *c, uint32_t party, uint64_t *sk, uint64_t *pk,
                         int32_t *sk_small, int32_t *e_small)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    int32_t *s = (int32_t *)malloc(n * sizeof(int32_t));
    int32_t *e = (int32_t *)malloc(n * sizeof(int32_t));
    uint64_t *prod = (uint64_t *)malloc(n * sizeof(uint64_t));
    orc_sample_ternary(c->p.seed, ORC_DOM_RSK, party, 0, 0, n, s);
    orc_sample_cbd(c->p.seed, ORC_DOM_RPK_E, party, 0, 0, c->p.cbd_eta, n, e);
    for (uint32_t i = 0; i < L; ++i) {
        uint64_t q = c->p.q[i];
        uint64_t *ski = sk + (size_t)i * n;
        uint64_t *p0 = pk + (size_t)i * n;
        uint64_t *p1 = pk + (size_t)(L + i) * n;
        orc_sample_uniform(c->p.seed, ORC_DOM_RPK_A, i, party, 0, 0, q, n, p1);
        for (size_t k = 0; k < n; ++k) ski[k] = lift_small(s[k], q);
        orc_ring_mul(p1, ski, n, q, c->psi[i], prod);
        for (size_t k = 0; k < n; ++k)
            p0[k] = submod(0, addmod(prod[k], lift_small(e[k], q), q), q); /* -(p1 sk + e) */
    }
    if (sk_small) memcpy(sk_small, s, n * sizeof(int32_t));
    if (e_small) memcpy(e_small, e, n * sizeof(int32_t));
    free(s); free(e); free(prod);
}

void orc_convert_share(const orc_ctx *c, const uint64_t *sk_share, const uint64_t *pk_recv,
                       const uint64_t *ct, uint32_t C, uint32_t party, uint32_t receiver,
                       uint32_t group, uint32_t ct_base, uint64_t *share)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    uint32_t who = party | (receiver << 16);
    int32_t *mu = (int32_t *)malloc(n * sizeof(int32_t));
    int32_t *e0 = (int32_t *)malloc(n * sizeof(int32_t));
    int32_t *e1 = (int32_t *)malloc(n * sizeof(int32_t));
    uint64_t *mu_q = (uint64_t *)malloc(n * sizeof(uint64_t));
    uint64_t *sc1 = (uint64_t *)malloc(n * sizeof(uint64_t));
    uint64_t *prod = (uint64_t *)malloc(n * sizeof(uint64_t));
    for (uint32_t ci = 0; ci < C; ++ci) {
        uint32_t index = ct_base + ci;
        orc_sample_ternary(c->p.seed, ORC_DOM_CVT_U, who, group, index, n, mu);
        orc_sample_cbd(c->p.seed, ORC_DOM_CVT_E0, who, group, index, c->p.cbd_eta, n, e0);
        orc_sample_cbd(c->p.seed, ORC_DOM_CVT_E1, who, group, index, c->p.cbd_eta, n, e1);
        const uint64_t *c1 = ct + ((size_t)ci * 2 + 1) * L * n;
        uint64_t *h0 = share + (size_t)ci * 2 * L * n;
        uint64_t *h1 = h0 + (size_t)L * n;
        for (uint32_t i = 0; i < L; ++i) {
            uint64_t q = c->p.q[i];
            const uint64_t *p0 = pk_recv + (size_t)i * n;
            const uint64_t *p1 = pk_recv + (size_t)(L + i) * n;
            for (size_t k = 0; k < n; ++k) mu_q[k] = lift_small(mu[k], q);
            orc_ring_mul(sk_share + (size_t)i * n, c1 + (size_t)i * n, n, q, c->psi[i], sc1);
            orc_ring_mul(mu_q, p0, n, q, c->psi[i], prod);
            for (size_t k = 0; k < n; ++k)
                h0[(size_t)i * n + k] = addmod(addmod(sc1[k], prod[k], q), lift_small(e0[k], q), q);
            orc_ring_mul(mu_q, p1, n, q, c->psi[i], prod);
            for (size_t k = 0; k < n; ++k)
                h1[(size_t)i * n + k] = addmod(prod[k], lift_small(e1[k], q), q);
        }
    }
    free(mu); free(e0); free(e1); free(mu_q); free(sc1); free(prod);
}

void orc_convert_combine(const orc_ctx *c, const uint64_t *ct, const uint64_t *const *shares,
                         uint32_t K, uint32_t C, uint64_t *ct_out)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    for (uint32_t ci = 0; ci < C; ++ci)
        for (uint32_t i = 0; i < L; ++i) {
            uint64_t q = c->p.q[i];
            size_t o0 = ((size_t)ci * 2 * L + i) * n, o1 = o0 + (size_t)L * n;
            for (size_t k = 0; k < n; ++k) {
                uint64_t a0 = ct[o0 + k], a1 = 0; /* the old c1 is dropped */
                for (uint32_t m = 0; m < K; ++m) {
                    a0 = addmod(a0, shares[m][o0 + k], q);
                    a1 = addmod(a1, shares[m][o1 + k], q);
                }
                ct_out[o0 + k] = a0;
                ct_out[o1 + k] = a1;
            }
        }
}

/* ---- MBFV.Bootstrap (Sec. 4.2 item 4, Eq. (3)) ---- */

void orc_bootstrap_alpha(const orc_ctx *c, uint32_t group, uint32_t ct, uint64_t *alpha)
{
    for (uint32_t i = 0; i < c->p.num_limbs; ++i)
        orc_sample_uniform(c->p.seed, ORC_DOM_BS_A, i, 0, group, ct, c->p.q[i], c->n, alpha + (size_t)i * c->n);
}

void orc_bootstrap_share(const orc_ctx *c, const uint64_t *sk_share, const uint64_t *ct, uint32_t C,
                         uint32_t party, uint32_t group, uint32_t ct_base, uint64_t *share)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    uint64_t *M = (uint64_t *)malloc(n * sizeof(uint64_t));
    int32_t *e0 = (int32_t *)malloc(n * sizeof(int32_t));
    int32_t *e1 = (int32_t *)malloc(n * sizeof(int32_t));
    uint64_t *alpha = (uint64_t *)malloc((size_t)L * n * sizeof(uint64_t));
    uint64_t *sc1 = (uint64_t *)malloc(n * sizeof(uint64_t));
    uint64_t *sa = (uint64_t *)malloc(n * sizeof(uint64_t));
    for (uint32_t ci = 0; ci < C; ++ci) {
        uint32_t index = ct_base + ci;
        orc_sample_uniform(c->p.seed, ORC_DOM_BS_M, 0, party, group, index, c->p.t, n, M);
        orc_sample_cbd(c->p.seed, ORC_DOM_BS_E0, party, group, index, c->p.cbd_eta, n, e0);
        orc_sample_cbd(c->p.seed, ORC_DOM_BS_E1, party, group, index, c->p.cbd_eta, n, e1);
        orc_bootstrap_alpha(c, group, index, alpha);
        const uint64_t *c1 = ct + ((size_t)ci * 2 + 1) * L * n;
        uint64_t *eta0 = share + (size_t)ci * 2 * L * n;
        uint64_t *eta1 = eta0 + (size_t)L * n;
        for (uint32_t i = 0; i < L; ++i) {
            uint64_t q = c->p.q[i];
            const uint64_t *ski = sk_share + (size_t)i * n;
            orc_ring_mul(ski, c1 + (size_t)i * n, n, q, c->psi[i], sc1);
            orc_ring_mul(ski, alpha + (size_t)i * n, n, q, c->psi[i], sa);
            for (size_t k = 0; k < n; ++k) {
                uint64_t lm = orc_mulmod(c->lambda_mod_q[i], M[k] % q, q); /* Lambda M_k */
                eta0[(size_t)i * n + k] = addmod(submod(sc1[k], lm, q), lift_small(e0[k], q), q);
                eta1[(size_t)i * n + k] = addmod(submod(lm, sa[k], q), lift_small(e1[k], q), q);
            }
        }
    }
    free(M); free(e0); free(e1); free(alpha); free(sc1); free(sa);
}

void orc_bootstrap_combine(const orc_ctx *c, const uint64_t *ct, const uint64_t *const *shares,
                           uint32_t K, uint32_t C, uint32_t group, uint32_t ct_base, uint64_t *ct_out)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    for (uint32_t ci = 0; ci < C; ++ci) {
        size_t base = (size_t)ci * 2 * L * n;
        for (size_t k = 0; k < n; ++k) {
            uint64_t res[ORC_MAX_LIMBS];
            for (uint32_t i = 0; i < L; ++i) {
                uint64_t acc = ct[base + (size_t)i * n + k];              /* c0 + eta0 */
                for (uint32_t m = 0; m < K; ++m) acc = addmod(acc, shares[m][base + (size_t)i * n + k], c->p.q[i]);
                res[i] = acc;
            }
            uint64_t x = scale_round(c, res);                              /* in [0,t) */
            for (uint32_t i = 0; i < L; ++i) {
                uint64_t q = c->p.q[i];
                uint64_t acc = orc_mulmod(c->lambda_mod_q[i], x % q, q);  /* Lambda x + eta1 */
                for (uint32_t m = 0; m < K; ++m)
                    acc = addmod(acc, shares[m][base + (size_t)(L + i) * n + k], q);
                ct_out[base + (size_t)i * n + k] = acc;
            }
        }
        orc_bootstrap_alpha(c, group, ct_base + ci, ct_out + base + (size_t)L * n);
    }
}

/* Alg. 2 lines 9-10: W_{k+1/2,i} = (1/K) sum_j W_{k,j} over the closed neighbourhood, then
 * W_{k+1,i} = W_{k+1/2,i} - gamma g_i.  volatile keeps every intermediate in float32.       */
void orc_average_update(const float *sum, uint32_t K, const float *grad, float gamma, uint64_t n,
                        float *w)
{
    volatile float inv_k = 1.0f / (float)K;
    for (uint64_t j = 0; j < n; ++j) {
        volatile float avg = sum[j] * inv_k;
        if (grad) {
            volatile float step = gamma * grad[j];
            w[j] = avg - step;
        } else {
            w[j] = avg;
        }
    }
}

void orc_bench_polys(const orc_ctx *c, uint32_t B, uint64_t *out)
{
    for (uint32_t b = 0; b < B; ++b)
        for (uint32_t i = 0; i < c->p.num_limbs; ++i)
            orc_sample_uniform(c->p.seed, ORC_DOM_BENCH, i, 0, 0, b, c->p.q[i], c->n,
                               out + ((size_t)b * c->p.num_limbs + i) * c->n);
}

void orc_ntt_forward_batch(const orc_ctx *c, uint64_t *polys, uint32_t B)
{
    uint32_t L = c->p.num_limbs;
    long total = (long)B * L;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic)
#endif
    for (long idx = 0; idx < total; ++idx)
        orc_ntt_forward(polys + (size_t)idx * c->n, c->n, c->p.q[idx % L], c->psi[idx % L]);
}

void orc_ntt_inverse_batch(const orc_ctx *c, uint64_t *polys, uint32_t B)
{
    uint32_t L = c->p.num_limbs;
    long total = (long)B * L;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic)
#endif
    for (long idx = 0; idx < total; ++idx)
        orc_ntt_inverse(polys + (size_t)idx * c->n, c->n, c->p.q[idx % L], c->psi[idx % L]);
}

/* One exchange round for one group, ciphertext indices [ct_begin, ct_end): every member
 * encodes and encrypts, the ciphertexts are summed, every member contributes a share,
 * the shares are combined and the result is decoded (Alg. 2, lines 6-9).                */
int orc_round_group(const orc_ctx *c, const uint64_t *pk, const uint64_t *const *sks,
                    const float *const *grads, const uint32_t *members, uint32_t K,
                    uint32_t group, uint64_t n_values, uint32_t ct_begin, uint32_t ct_end,
                    float *out_sum)
{
    size_t n = c->n;
    uint32_t L = c->p.num_limbs;
    size_t ct_words = (size_t)2 * L * n;
    int threads = 1;
#ifdef _OPENMP
    threads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic)
#endif
    for (long ci = (long)ct_begin; ci < (long)ct_end; ++ci) {
        uint64_t first = (uint64_t)ci * n;
        uint64_t count = first >= n_values ? 0 : (n_values - first < n ? n_values - first : n);
        uint64_t *pt = (uint64_t *)malloc(n * sizeof(uint64_t));
        uint64_t *ct = (uint64_t *)malloc(ct_words * sizeof(uint64_t));
        uint64_t *agg = (uint64_t *)calloc(ct_words, sizeof(uint64_t));
        uint64_t *shares = (uint64_t *)malloc((size_t)K * L * n * sizeof(uint64_t));
        const uint64_t **share_ptrs = (const uint64_t **)malloc(K * sizeof(uint64_t *));
        for (uint32_t m = 0; m < K; ++m) {
            orc_encode(c, grads[m] + first, count, pt, 1);
            orc_encrypt(c, pk, pt, 1, members[m], group, (uint32_t)ci, ct);
            orc_add(c, agg, ct, 1);
        }
        for (uint32_t m = 0; m < K; ++m) {
            share_ptrs[m] = shares + (size_t)m * L * n;
            orc_partial_decrypt(c, sks[m], agg, 1, members[m], group, (uint32_t)ci,
                                shares + (size_t)m * L * n);
        }
        orc_combine(c, agg, share_ptrs, K, 1, pt);
        orc_decode(c, pt, 1, count, out_sum + first);
        free(pt); free(ct); free(agg); free(shares); free(share_ptrs);
    }
    return threads;
}
