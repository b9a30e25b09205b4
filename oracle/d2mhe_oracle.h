/*
 * CPU oracle for the multiparty-BFV gradient exchange of D2-MHE (arXiv 2207.04604).
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, obviously-correct statement of what
 * the hot path computes.  It shares no code, table, constant generator or helper with the
 * HIP library and must never be called by it.  Only the test-suite, the smoke check and
 * the CPU-baseline leg of the benchmark may link or load it.
 *
 * Every modular product is `unsigned __int128` followed by `%`; ring products are the
 * schoolbook negacyclic convolution or a textbook (twist + cyclic Cooley-Tukey) transform
 * that the tests pin against the schoolbook product; the decryption rounding is done with
 * a small multi-word integer type, exactly as the formula in Sec. 3.2 (item 5) states it.
 *
 * Notation (Sec. 3.2): R_q = Z_q[X]/(X^N+1), q = prod q_i (RNS limbs), plaintext ring R_t,
 * Lambda = floor(q/t).  P parties; a "group" is a closed neighbourhood {i} u N_i (Sec. 4).
 *
 * Layouts: a polynomial in RNS form is uint64[L][N], limb-major, canonical residues in
 * [0,q_i), coefficient domain, natural order.  A ciphertext is uint64[2][L][N] = (c0,c1).
 */
#ifndef D2MHE_ORACLE_H
#define D2MHE_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_MAX_LIMBS 16

/* Philox domains: the byte placed in the low 8 bits of counter word 3. */
enum {
    ORC_DOM_SK = 0x01,     /* ternary secret-key share                 */
    ORC_DOM_PK_E = 0x02,   /* error of the public-key share            */
    ORC_DOM_CRS = 0x03,    /* common random polynomial p1 (per limb)   */
    ORC_DOM_ENC_U = 0x04,  /* ternary mu of Encrypt                    */
    ORC_DOM_ENC_E0 = 0x05, /* error e0 of Encrypt                      */
    ORC_DOM_ENC_E1 = 0x06, /* error e1 of Encrypt                      */
    ORC_DOM_DEC_E = 0x07,  /* smudging error of a decryption share     */
    ORC_DOM_BENCH = 0x08,  /* uniform benchmark polynomials (per limb) */
    /* MBFV.Convert (Sec. 4.2 item 3) */
    ORC_DOM_RSK = 0x10,    /* ternary single-key secret of a receiver  */
    ORC_DOM_RPK_A = 0x11,  /* uniform p1 of a receiver's public key (per limb) */
    ORC_DOM_RPK_E = 0x12,  /* error of a receiver's public key         */
    ORC_DOM_CVT_U = 0x13,  /* mu_k of a conversion share               */
    ORC_DOM_CVT_E0 = 0x14, /* e0_k of a conversion share               */
    ORC_DOM_CVT_E1 = 0x15, /* e1_k of a conversion share               */
    /* MBFV.Bootstrap (Sec. 4.2 item 4) */
    ORC_DOM_BS_M = 0x16,   /* mask M_k, uniform in R_t                 */
    ORC_DOM_BS_E0 = 0x17,  /* e0_k of a bootstrap share                */
    ORC_DOM_BS_E1 = 0x18,  /* e1_k of a bootstrap share                */
    ORC_DOM_BS_A = 0x19    /* common random polynomial alpha (per limb) */
};

typedef struct {
    uint32_t log2_n;            /* ring degree N = 2^log2_n                              */
    uint32_t num_limbs;         /* L                                                     */
    uint64_t q[ORC_MAX_LIMBS];  /* RNS primes, q_i = 1 mod 2N                            */
    uint64_t t;                 /* plaintext modulus, prime, t = 1 mod 2N (0: no slots)  */
    uint32_t cbd_eta;           /* eta of the centred binomial error distribution        */
    uint32_t frac_bits;         /* f: fixed-point fraction bits                          */
    uint32_t max_group;         /* K_max: largest closed neighbourhood (encode clamp)    */
    uint64_t seed;              /* Philox key                                            */
} orc_params;

typedef struct orc_ctx orc_ctx;

/* ---- counter-based generator (Philox4x32-10, Salmon et al., SC'11) ---- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Samplers for coefficient 0..n-1 of one polynomial.  Counter = (block, ct, party,
 * domain | limb<<8 | group<<16), key = (seed low, seed high).                           */
void orc_sample_ternary(uint64_t seed, uint32_t domain, uint32_t party, uint32_t group,
                        uint32_t ct, size_t n, int32_t *out);
void orc_sample_cbd(uint64_t seed, uint32_t domain, uint32_t party, uint32_t group,
                    uint32_t ct, uint32_t eta, size_t n, int32_t *out);
void orc_sample_uniform(uint64_t seed, uint32_t domain, uint32_t limb, uint32_t party,
                        uint32_t group, uint32_t ct, uint64_t q, size_t n, uint64_t *out);

/* ---- number theory ---- */
uint64_t orc_mulmod(uint64_t a, uint64_t b, uint64_t q);
uint64_t orc_powmod(uint64_t a, uint64_t e, uint64_t q);
int orc_is_prime(uint64_t n); /* deterministic Miller-Rabin, bases 2..37 */
/* The `count` largest primes of the form 2^bits - k*2N + 1, k = 1,2,...  Returns count. */
int orc_find_primes(uint32_t bits, uint32_t log2_n, int count, uint64_t *out);
/* psi = x^((q-1)/2N) for the smallest integer x >= 2 with psi^N = -1 (mod q).           */
uint64_t orc_find_psi(uint64_t q, uint32_t log2_n);

/* ---- ring arithmetic in Z_q[X]/(X^n+1), one limb ---- */
void orc_negacyclic_schoolbook(const uint64_t *a, const uint64_t *b, size_t n, uint64_t q,
                               uint64_t *out);
/* xhat[j] = sum_n x[n] psi^((2j+1) n), written out term by term: O(n^2).                */
void orc_ntt_definition(const uint64_t *x, size_t n, uint64_t q, uint64_t psi, uint64_t *out);
/* The same map and its inverse in O(n log n); natural order in and out, in place.       */
void orc_ntt_forward(uint64_t *x, size_t n, uint64_t q, uint64_t psi);
void orc_ntt_inverse(uint64_t *x, size_t n, uint64_t q, uint64_t psi);
void orc_ring_mul(const uint64_t *a, const uint64_t *b, size_t n, uint64_t q, uint64_t psi,
                  uint64_t *out);

/* ---- scheme ---- */
orc_ctx *orc_create(const orc_params *p); /* NULL on invalid parameters */
void orc_destroy(orc_ctx *c);
uint64_t orc_psi(const orc_ctx *c, uint32_t limb);
uint64_t orc_psi_t(const orc_ctx *c);
uint64_t orc_lambda_mod_q(const orc_ctx *c, uint32_t limb); /* floor(Q/t) mod q_i       */
uint64_t orc_q_mod_t(const orc_ctx *c);                     /* Q mod t                   */
uint32_t orc_lambda_bits(const orc_ctx *c);                 /* bit length of floor(Q/t)  */
int64_t orc_encode_clamp(const orc_ctx *c);

/* Common random polynomial p1 [L][N] (MBFV.PubKeyGen: "agreed in advance").             */
void orc_crs(const orc_ctx *c, uint64_t *p1);
/* MBFV.SecKeyGen + one party's part of MBFV.PubKeyGen:
 * s_k ternary, e_k error, p0_k = -(p1 s_k + e_k).  sk [L][N], pk0_share [L][N].
 * sk_small/e_small (nullable) receive the signed coefficients [N].                      */
void orc_keygen_share(const orc_ctx *c, uint32_t party, uint64_t *sk, uint64_t *pk0_share,
                      int32_t *sk_small, int32_t *e_small);
/* pk = ([sum_k p0_k]_q, p1), pk [2][L][N].                                              */
void orc_aggregate_pk(const orc_ctx *c, const uint64_t *const *pk0_shares, uint32_t K,
                      uint64_t *pk);
/* float gradient -> fixed point -> slots -> plaintext polynomials pt [C][N] in [0,t).   */
int orc_encode(const orc_ctx *c, const float *grad, uint64_t n_values, uint64_t *pt,
               uint32_t C);
/* Coefficient packing: the same fixed point, but value c N + j is coefficient j of plaintext c
 * (no slot structure; enough for a workload that only adds).  pt [C][N].                  */
int orc_encode_coefficients(const orc_ctx *c, const float *grad, uint64_t n_values, uint64_t *pt,
                            uint32_t C);
int orc_decode_coefficients(const orc_ctx *c, const uint64_t *pt, uint32_t C, uint64_t n_values,
                            float *out);
/* BFV.Encrypt under pk for ciphertext indices ct_base..ct_base+C-1: ct [C][2][L][N].    */
void orc_encrypt(const orc_ctx *c, const uint64_t *pk, const uint64_t *pt, uint32_t C,
                 uint32_t party, uint32_t group, uint32_t ct_base, uint64_t *ct);
/* BFV.Add: acc += in, component- and coefficient-wise.                                  */
void orc_add(const orc_ctx *c, uint64_t *acc, const uint64_t *in, uint32_t C);
/* Decryption share h_k = s_k c1 + e_k (Eq. (1) without the target-key terms).           */
void orc_partial_decrypt(const orc_ctx *c, const uint64_t *sk, const uint64_t *ct, uint32_t C,
                         uint32_t party, uint32_t group, uint32_t ct_base, uint64_t *share);
/* y = c0 + sum_k h_k; pt = [round(t*y/Q)]_t with y lifted to [0,Q).  pt [C][N].          */
void orc_combine(const orc_ctx *c, const uint64_t *ct, const uint64_t *const *shares,
                 uint32_t K, uint32_t C, uint64_t *pt);
/* plaintext polynomials -> slots -> centred -> float.                                   */
int orc_decode(const orc_ctx *c, const uint64_t *pt, uint32_t C, uint64_t n_values,
               float *out);
/* Single-key BFV.Decrypt with an explicit secret s [L][N]: the receiver's last step after
 * MBFV.Convert, and a cross-check of the collective decryption in the pins.             */
void orc_decrypt_with_secret(const orc_ctx *c, const uint64_t *s, const uint64_t *ct,
                             uint32_t C, uint64_t *pt);

/* ---- MBFV.Convert: key switching to a receiver's own key (Sec. 4.2 item 3) ---- */
/* Receiver i's single-key BFV pair (Sec. 3.2 items 1-2): sk_i ternary, p1_i uniform in R_q,
 * p0_i = -(p1_i sk_i + e).  sk [L][N], pk [2][L][N] = (p0_i, p1_i); counter party word = i.
 * sk_small/e_small (nullable) receive the signed coefficients [N].                      */
void orc_receiver_keygen(const orc_ctx *c, uint32_t party, uint64_t *sk, uint64_t *pk,
                         int32_t *sk_small, int32_t *e_small);
/* Member k's share towards receiver i, Eq. (1):
 *   (h0, h1) = (s_k c1 + mu_k p0_i + e0_k, mu_k p1_i + e1_k),   share [C][2][L][N].
 * mu_k is ternary (the same distribution as in Encrypt), e0_k, e1_k from chi; their counter
 * party word is k | i << 16, group and ciphertext index as in Encrypt.                   */
void orc_convert_share(const orc_ctx *c, const uint64_t *sk_share, const uint64_t *pk_recv,
                       const uint64_t *ct, uint32_t C, uint32_t party, uint32_t receiver,
                       uint32_t group, uint32_t ct_base, uint64_t *share);
/* The receiver's new ciphertext E' = (c0 + sum_k h0_k, sum_k h1_k), ct_out [C][2][L][N];
 * BFV.Decrypt(sk_i, E') is orc_decrypt_with_secret (Eq. (2)).                            */
void orc_convert_combine(const orc_ctx *c, const uint64_t *ct, const uint64_t *const *shares,
                         uint32_t K, uint32_t C, uint64_t *ct_out);

/* ---- MBFV.Bootstrap: collective refresh of a ciphertext (Sec. 4.2 item 4, Eq. (3)) ---- */
/* The common random polynomial alpha of the refresh of ciphertext index ct of a group:
 * uniform in R_q, alpha [L][N]; counter (block, ct, 0, BS_A | limb << 8 | group << 16).    */
void orc_bootstrap_alpha(const orc_ctx *c, uint32_t group, uint32_t ct, uint64_t *alpha);
/* Member k's share, Eq. (3):
 *   (eta0, eta1) = (s_k c1 - Lambda M_k + e0_k, -s_k alpha + Lambda M_k + e1_k),  share [C][2][L][N],
 * M_k uniform in R_t (coefficient n = the 128-bit block n reduced mod t, representative in
 * [0,t)), e0_k, e1_k from chi; counters (block, ct_base + c, k, domain | group << 16).      */
void orc_bootstrap_share(const orc_ctx *c, const uint64_t *sk_share, const uint64_t *ct, uint32_t C,
                         uint32_t party, uint32_t group, uint32_t ct_base, uint64_t *share);
/* The refreshed ciphertext ct' = ([round(t/q [c0 + eta0]_q)]_t Lambda + eta1, alpha) with
 * eta_d = sum_k eta_{d,k}; the rounded plaintext enters with its representative in [0,t).
 * ct_out [C][2][L][N].                                                                    */
void orc_bootstrap_combine(const orc_ctx *c, const uint64_t *ct, const uint64_t *const *shares,
                           uint32_t K, uint32_t C, uint32_t group, uint32_t ct_base, uint64_t *ct_out);

/* ---- the float step of one training iteration (Alg. 2 lines 9-10) ---- */
/* w[j] = sum[j] * (1/K) - gamma * grad[j], every operation rounded to float32 on its own:
 * the neighbourhood average from the decoded sum, then the local gradient step.
 * grad may be NULL when gamma = 0.                                                        */
void orc_average_update(const float *sum, uint32_t K, const float *grad, float gamma, uint64_t n,
                        float *w);

/* Uniform benchmark polynomials: out [B][L][N], polynomial b of the batch, limb i.      */
void orc_bench_polys(const orc_ctx *c, uint32_t B, uint64_t *out);
/* Batched transform of polys [B][L][N] in place (natural order).                        */
void orc_ntt_forward_batch(const orc_ctx *c, uint64_t *polys, uint32_t B);
void orc_ntt_inverse_batch(const orc_ctx *c, uint64_t *polys, uint32_t B);

/* One whole round for one group (timing driver; OpenMP over ciphertext index when built
 * with -fopenmp).  grads: K pointers to n_values floats; members: K party ids;
 * sks: K pointers [L][N]; pk [2][L][N]; out_sum: n_values floats.  Returns threads used. */
int orc_round_group(const orc_ctx *c, const uint64_t *pk, const uint64_t *const *sks,
                    const float *const *grads, const uint32_t *members, uint32_t K,
                    uint32_t group, uint64_t n_values, uint32_t ct_begin, uint32_t ct_end,
                    float *out_sum);

#ifdef __cplusplus
}
#endif
#endif
