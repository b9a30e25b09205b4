/*
 * d2mhe -- MI355X (gfx950) hot path of the private gradient exchange of D2-MHE
 * (arXiv 2207.04604): multiparty BFV over R_q = Z_q[X]/(X^N+1) in RNS form.
 *
 * C ABI.  Every data buffer is CALLER-OWNED DEVICE MEMORY unless a parameter is marked
 * "host"; the library never allocates or frees device memory.  Its tables live in a
 * caller-provided device workspace.  All device pointers must be 16-byte aligned.
 * Calls enqueue work on the given hipStream_t (passed as void*, NULL = default stream)
 * and do not synchronise, except create / destroy.  No exception or abort crosses the
 * ABI; every call returns a status (0 = OK, negative = error, see d2mhe_strerror).
 * A context is immutable after create: concurrent calls on different streams with
 * disjoint output buffers are legal.
 *
 * Notation (Sec. 3.2, Sec. 4.2 of the paper): N ring degree, L RNS limbs q_0..q_{L-1},
 * Q = prod q_i, t plaintext modulus, Lambda = floor(Q/t), K members of a closed
 * neighbourhood {i} u N_i ("group"), C ciphertexts per gradient vector.
 *
 * DEVIATION FROM A COEFFICIENT-FORM BOUNDARY.  Ciphertexts, decryption shares, key shares and public
 * keys cross this boundary in EVALUATION FORM (the image of the negacyclic transform below), not as
 * coefficient vectors of R_q: the formulas of Sec. 3.2 / Sec. 4.2 are ring identities, the transform
 * is a ring isomorphism R_q -> Z_q^N, so the objects are the same protocol messages, and Encrypt
 * then costs three forward transforms per limb and no inverse, a share one, Decrypt one inverse.
 * Plaintexts and floats are in coefficient / natural form.  d2mhe_ntt_inverse turns any of these
 * objects into the coefficient form of the paper, d2mhe_ntt_index_map publishes the storage order.
 *
 * Data forms
 *   coefficient form : uint64 [..][N], natural order, canonical residues.
 *   evaluation form  : uint64 [..][N]; position p holds xhat[perm[p]], where
 *                      xhat[j] = sum_n x[n] psi_i^((2j+1) n) mod q_i, psi_i = x^((q_i-1)/2N)
 *                      for the smallest x >= 2 with psi_i^N = -1, and perm is returned
 *                      by d2mhe_ntt_index_map.  Canonical residues in [0, q_i).
 *   d2mhe_ntt_forward / d2mhe_ntt_inverse convert between the two.
 *
 *   plaintext        pt    [C][N]        coefficient form, values in [0, t)
 *   ciphertext       ct    [C][2][L][N]  evaluation form, (c0, c1), limb-major
 *   decryption share share [C][L][N]     evaluation form
 *   pk0 share        [L][N]              evaluation form
 *   prepared key     [2][L][N] words per polynomial: the evaluation-form values [L][N]
 *                    followed by their Shoup quotients floor(v * 2^64 / q_i) [L][N].
 *                    sk_share = one prepared polynomial (2*L*N words);
 *                    pk = two prepared polynomials p0, p1 (4*L*N words).
 *
 * Randomness: Philox4x32-10 keyed by `seed`; counter = (block, ciphertext index, party,
 * domain | limb << 8 | group << 16).  Ternary coefficient n = word n&3 of block n>>2,
 * value floor(3w/2^32)-1; centred-binomial coefficient n = words 2(n&1), 2(n&1)+1 of block
 * n>>1, popcount(low eta bits) difference; uniform coefficient n = 128-bit block n mod q_i.
 * Domains: 1 secret share, 2 public-key error, 3 common random polynomial (per limb),
 * 4/5/6 mu/e0/e1 of Encrypt, 7 decryption-share error, 8 benchmark polynomials;
 * 0x10/0x11/0x12 a receiver's own secret key / uniform p1 (per limb) / key error,
 * 0x13/0x14/0x15 mu/e0/e1 of a conversion share (party word = member | receiver << 16);
 * 0x16 the mask M_k of a refresh share (block n mod t), 0x17/0x18 its e0/e1,
 * 0x19 the common polynomial alpha of a refresh (per limb, party word 0).
 */
#ifndef D2MHE_H
#define D2MHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct d2mhe_ctx d2mhe_ctx; /* opaque, host memory owned by the library */
typedef int32_t d2mhe_status;

enum {
    D2MHE_OK = 0,
    D2MHE_ERR_BAD_PARAMS = -1,    /* N, L, q_i, t, eta outside what is documented below   */
    D2MHE_ERR_NULL = -2,          /* a required pointer is NULL                            */
    D2MHE_ERR_ALIGN = -3,         /* a device pointer is not 16-byte aligned               */
    D2MHE_ERR_RANGE = -4,         /* an index or count is out of range                     */
    D2MHE_ERR_WORKSPACE = -5,     /* workspace / scratch too small                         */
    D2MHE_ERR_HIP = -6,           /* a HIP runtime call failed (d2mhe_last_hip_error)      */
    D2MHE_ERR_UNIMPLEMENTED = -7  /* valid request that this build does not cover          */
};

typedef struct {
    uint32_t log2_n;      /* 10..16                                                         */
    uint32_t num_limbs;   /* L, 1..16                                                       */
    const uint64_t *q;    /* host: L distinct primes < 2^61, q_i = 1 (mod 2N)               */
    uint64_t t;           /* prime, t = 1 (mod 2N), t < 2^30, t < min q_i;
                             0 = transform-only context (no encode/encrypt/decrypt)         */
    uint32_t cbd_eta;     /* 1..32: error = popcount(eta bits) - popcount(eta bits)          */
    uint32_t frac_bits;   /* f: fixed-point fraction bits, 0..30                            */
    uint32_t max_group;   /* K_max >= 1: encode clamps to +-floor(((t-1)/2)/K_max)          */
    uint64_t seed;        /* Philox key                                                     */
} d2mhe_params;

/* ---- context ------------------------------------------------------------------------- */
/* Bytes of device workspace that d2mhe_create needs for these parameters (0 if invalid). */
size_t d2mhe_workspace_bytes(const d2mhe_params *params);
/* Validates the parameters, builds twiddle / constant tables on the host, copies them into
 * `dev_workspace` (synchronously) and derives the common random polynomial p1 of
 * MBFV.PubKeyGen (Sec. 4.2 item 2).  The workspace must outlive the context.             */
d2mhe_status d2mhe_create(const d2mhe_params *params, void *dev_workspace, size_t bytes,
                          void *stream, d2mhe_ctx **out);
void d2mhe_destroy(d2mhe_ctx *ctx);
const char *d2mhe_strerror(d2mhe_status status);
int d2mhe_last_hip_error(const d2mhe_ctx *ctx);
/* host: perm[p] = index j of the evaluation xhat[j] stored at position p (N entries).    */
d2mhe_status d2mhe_ntt_index_map(const d2mhe_ctx *ctx, uint32_t *perm_host);
/* host: psi_i of limb i (i == L: the slot root psi_t), for inspection.                   */
uint64_t d2mhe_root(const d2mhe_ctx *ctx, uint32_t limb);

/* ---- negacyclic transforms ------------------------------------------------------------------ */
/* Sec. 3.2 defines the ciphertext ring R_q = Z_q[X]/(X^N + 1) (N a power of two) and every scheme
 * function as sums and products in it.  A product in R_q is the coefficient-wise product of the
 * evaluations at the N odd powers of a primitive 2N-th root psi_i, per RNS limb q_i:
 * forward  xhat[j] = sum_n x[n] psi_i^((2j+1) n) mod q_i,  inverse its inverse (including N^-1).
 * polys [B][L][N] device memory, in place: polynomial (b, i) is transformed modulo q_i;
 * coefficient form (natural order) <-> evaluation form (order of d2mhe_ntt_index_map), canonical
 * residues in and out.  Ring degrees above 2^14 run as two kernels per direction.  B = 0: no-op.
 * Errors: NULL ctx/polys, misaligned polys, B * L >= 2^31 (D2MHE_ERR_RANGE).                 */
d2mhe_status d2mhe_ntt_forward(d2mhe_ctx *ctx, uint64_t *polys, uint32_t B, void *stream);
d2mhe_status d2mhe_ntt_inverse(d2mhe_ctx *ctx, uint64_t *polys, uint32_t B, void *stream);
/* Uniform benchmark polynomials (Philox domain 8), coefficient form, out [B][L][N].      */
d2mhe_status d2mhe_bench_polys(d2mhe_ctx *ctx, uint64_t *out, uint32_t B, void *stream);

/* ---- set-up: MBFV.SecKeyGen and MBFV.PubKeyGen (Sec. 4.2 items 1, 2) ---------------------- */
/* Party k: s_k ternary, e_k error; sk_share = prepared s_k (2*L*N words);
 * pk0_share = -(p1 s_k + e_k) [L][N].                                                     */
d2mhe_status d2mhe_keygen_share(d2mhe_ctx *ctx, uint32_t party, uint64_t *sk_share,
                                uint64_t *pk0_share, void *stream);
/* pk = ([sum_k p0_k]_q, p1) as two prepared polynomials (4*L*N words).
 * pk0_shares: HOST array of K device pointers.                                            */
d2mhe_status d2mhe_aggregate_pk(d2mhe_ctx *ctx, const uint64_t *const *pk0_shares, uint32_t K,
                                uint64_t *pk, void *stream);

/* ---- per round (Alg. 2 lines 6-9) ---------------------------------------------------------- */
/* Encoding of a float vector into plaintext polynomials.  Sec. 6 (implementation paragraph)
 * packs many values into one plaintext's SIMD slots and converts floats to fixed point with an
 * error below 2^-d; it gives no map, so this is the library's reading: r = rint(v 2^f) in float32
 * (ties to even), NaN -> 0, clamped (exactly, as an integer) to +-floor(((t-1)/2)/K_max) so that a
 * sum of K_max terms cannot wrap modulo t (+-inf saturate), z = r mod t in [0, t); value c*N + j is
 * slot j of plaintext c, i.e. the plaintext polynomial m_c in R_t (Sec. 3.2) has
 * m_c(psi_t^(2j+1)) = z[c*N + j] (inverse negacyclic transform modulo t, psi_t by the same rule as
 * psi_i); all N slots are used.  grad: n_values floats (device); pt [C][N] coefficient form in
 * [0, t); needs n_values <= C*N (else D2MHE_ERR_RANGE), slots past n_values are zero.          */
d2mhe_status d2mhe_encode(d2mhe_ctx *ctx, const float *grad, uint64_t n_values, uint64_t *pt,
                          uint32_t C, void *stream);
/* BFV.Encrypt (Sec. 3.2 item 3) under the collective key: ct_c = (Lambda m_c + mu p0 + e0,
 * mu p1 + e1) for c = 0..C-1, randomness indexed by (party, group, ct_base + c).          */
d2mhe_status d2mhe_encrypt(d2mhe_ctx *ctx, const uint64_t *pk, const uint64_t *pt, uint32_t C,
                           uint32_t party, uint32_t group, uint32_t ct_base, uint64_t *ct,
                           void *stream);
/* BFV.Add (Sec. 3.2 item 4; Alg. 2 line 8 sums the neighbours' ciphertexts with it):
 * ct_acc <- (ct_acc.c0 + ct_in.c0, ct_acc.c1 + ct_in.c1) mod q_i, coefficient-wise, for C
 * ciphertexts [C][2][L][N] (the sum is the same in either data form; both operands must be in
 * the same one).  ct_acc may equal ct_in.  Errors: NULL, misaligned.                            */
d2mhe_status d2mhe_add(d2mhe_ctx *ctx, uint64_t *ct_acc, const uint64_t *ct_in, uint32_t C,
                       void *stream);
/* Share of the collective decryption, Eq. (1) without the target-key terms:
 * h_k = s_k c1 + e_k, randomness indexed by (party, group, ct_base + c).                  */
d2mhe_status d2mhe_partial_decrypt(d2mhe_ctx *ctx, const uint64_t *sk_share, const uint64_t *ct,
                                   uint32_t C, uint32_t party, uint32_t group, uint32_t ct_base,
                                   uint64_t *share, void *stream);
/* y = c0 + sum_k h_k, pt = [round(t y / Q)]_t (BFV.Decrypt, Sec. 3.2 item 5).  shares: HOST
 * array of K device pointers, each [C][L][N].  The rounding is exact whenever t*y/Q is
 * farther than L*2^-62 from a half-integer (always, unless decryption noise overflowed).   */
d2mhe_status d2mhe_combine(d2mhe_ctx *ctx, const uint64_t *ct, const uint64_t *const *shares,
                           uint32_t K, uint32_t C, uint64_t *pt, void *stream);
/* Inverse of d2mhe_encode (same passage of Sec. 6): slots z[j] = m_c(psi_t^(2j+1)) by the forward
 * transform modulo t, centred representative (z > (t-1)/2 -> z - t), out = float32(z) * 2^-f (both
 * steps exact, hence a decoded sum equals the fixed-point sum bit for bit).  pt [C][N] in [0, t);
 * out: n_values floats (device), n_values <= C*N.                                              */
d2mhe_status d2mhe_decode(d2mhe_ctx *ctx, const uint64_t *pt, uint32_t C, uint64_t n_values,
                          float *out, void *stream);

/* Coefficient packing, the cheaper encoding for a workload that only adds: value c*N+j is
 * coefficient j of plaintext c (same fixed point, clamp and tail rule), so neither side needs
 * the transform modulo t.  Sums of ciphertexts decode to the same sums as with slots; the two
 * encodings must not be mixed within one sum.                                             */
d2mhe_status d2mhe_encode_coefficients(d2mhe_ctx *ctx, const float *grad, uint64_t n_values,
                                       uint64_t *pt, uint32_t C, void *stream);
d2mhe_status d2mhe_decode_coefficients(d2mhe_ctx *ctx, const uint64_t *pt, uint32_t C,
                                       uint64_t n_values, float *out, void *stream);

/* ---- fused round (same results as the calls above) ---------------------------------------------- */
/* One exchange round of Alg. 2 (lines 6-9) for every group at once.  Group g has members
 * members[group_offsets[g] .. group_offsets[g+1]) (party ids); a (party, group) pair is a
 * "job".  All arrays of this struct are HOST memory; the pointers they hold are device
 * pointers.                                                                                */
typedef struct {
    uint32_t num_groups;             /* G >= 1                                              */
    const uint32_t *group_offsets;   /* [G+1], group_offsets[0] = 0, strictly increasing    */
    const uint32_t *members;         /* [group_offsets[G]] party ids <= 65535, no party twice
                                        within one group                                     */
    const uint32_t *group_ids;       /* [G] ids used in the Philox counter, pairwise distinct,
                                        each <= 65535; NULL = 0..G-1                         */
    const uint64_t *const *pks;      /* [G] prepared public key of each group               */
    uint32_t num_parties;            /* P: size of the two tables below                     */
    const uint64_t *const *sk_shares;/* [P] prepared secret share by party id               */
    const float *const *grads;       /* [P] gradient by party id, n_values floats each      */
    float *const *out_sums;          /* [G] result per group, n_values floats each          */
    uint64_t n_values;
    uint32_t packing;                /* 0: value j of a ciphertext is slot j (default);
                                        1: it is coefficient j (see d2mhe_encode_coefficients)  */
    uint32_t ct_base;                /* first ciphertext index of this round: the randomness of
                                        ciphertext c is indexed by ct_base + c; a training loop
                                        passes iteration * C so that no index is used twice  */
} d2mhe_round_desc;

/* Scratch bytes for a round with num_jobs (party, group) pairs in num_groups groups.      */
size_t d2mhe_round_scratch_bytes(const d2mhe_ctx *ctx, uint32_t num_jobs, uint32_t num_groups,
                                 uint64_t n_values);
/* Every member of every group encodes + encrypts its gradient under the group's key
 * (ciphertext index c = 0..C-1), the ciphertexts of a group are summed, every member
 * produces a decryption share of its group's aggregate, and the shares are combined and
 * decoded into out_sums[g] (the sum of the members' fixed-point gradients).
 * After the call the scratch holds, in this order, the fresh ciphertexts [J][C][2][L][N]
 * (job order), the aggregates [G][C][2][L][N] and the shares [J][C][L][N].
 * phase_events: NULL, or a HOST array of 5 hipEvent_t recorded on `stream` before the
 * first kernel and after the encrypt, sum, share and combine phases; entries may be NULL
 * (that event is skipped).                                                                  */
d2mhe_status d2mhe_round(d2mhe_ctx *ctx, const d2mhe_round_desc *desc, void *scratch,
                         size_t scratch_bytes, void *const *phase_events, void *stream);
/* The same for a single group: sk_shares, grads: HOST arrays of K device pointers in member
 * order; members: HOST array of K party ids; scratch as for num_jobs = K, num_groups = 1.   */
d2mhe_status d2mhe_round_group(d2mhe_ctx *ctx, const uint64_t *pk,
                               const uint64_t *const *sk_shares, const float *const *grads,
                               const uint32_t *members, uint32_t K, uint32_t group,
                               uint64_t n_values, float *out_sum, void *scratch,
                               size_t scratch_bytes, void *stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): d2mhe_round_group with the
 * scratch in an array of D2MHE_STATIC_SCRATCH_BYTES that the library itself holds on every GPU it
 * runs on, until the process ends.  The call allocates nothing, on the device or on the host, and
 * gives the same out_sum as d2mhe_round_group.  A round that needs more scratch than the array holds
 * (d2mhe_round_scratch_bytes(ctx, K, 1, n_values) > D2MHE_STATIC_SCRATCH_BYTES) is refused with
 * D2MHE_ERR_WORKSPACE before anything is launched.  All calls on one GPU share that GPU's array (it
 * keeps the last call's ciphertexts, aggregate and shares; every word a call reads it has written
 * itself, so nothing needs clearing): calls that overlap in time on one GPU race, on any streams.
 * The array's device address is looked up in d2mhe_create (and on a first call on another device). */
#define D2MHE_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
d2mhe_status d2mhe_round_group_static(d2mhe_ctx *ctx, const uint64_t *pk,
                                      const uint64_t *const *sk_shares, const float *const *grads,
                                      const uint32_t *members, uint32_t K, uint32_t group,
                                      uint64_t n_values, float *out_sum, void *stream);

/* ---- the float step of one training iteration (Alg. 2 lines 9-10) ---------------------------- */
/* w[j] = sum[j] * (1/K) - gamma * grad[j] in float32, each operation rounded on its own:
 * the average over a closed neighbourhood of K nodes from the decoded sum (the weights 1/K of the
 * mixing matrix are not elements of Z_t, so they are applied after decryption), then the local
 * gradient step.  Device pointers; grad may be NULL when gamma is 0; w may alias sum.
 * A multi-iteration run alternates d2mhe_round (or d2mhe_round_convert) with this call.      */
d2mhe_status d2mhe_average_update(const float *sum, uint32_t K, const float *grad, float gamma,
                                  uint64_t n, float *w, void *stream);

/* ---- MBFV.Convert: key switching to a receiver's own key (Sec. 4.2 item 3) ------------------- */
/* In the paper's protocol node i does not take part in a collective decryption of the
 * aggregate; the members of its closed neighbourhood switch the aggregate to node i's own
 * public key pk_i, and node i decrypts alone (Eq. (1), (2)).
 *
 * A node's own single-key pair (BFV.SecKeyGen / BFV.PubKeyGen, Sec. 3.2 items 1-2):
 * sk ternary, p1 uniform in R_q, p0 = -(p1 sk + e).  sk: prepared polynomial (2*L*N words);
 * pk: two prepared polynomials (p0, p1), 4*L*N words.  Randomness indexed by the party id. */
d2mhe_status d2mhe_receiver_keygen(d2mhe_ctx *ctx, uint32_t party, uint64_t *sk, uint64_t *pk,
                                   void *stream);
/* Member `party`'s share towards `receiver`, Eq. (1):
 *   (h0, h1) = (s_k c1 + mu_k p0_i + e0_k, mu_k p1_i + e1_k),   share [C][2][L][N],
 * mu_k ternary (the distribution of mu in BFV.Encrypt), e0_k, e1_k from chi; randomness indexed
 * by (party | receiver << 16, group, ct_base + c).  pk_recv: the receiver's prepared key.  */
d2mhe_status d2mhe_convert_share(d2mhe_ctx *ctx, const uint64_t *sk_share, const uint64_t *pk_recv,
                                 const uint64_t *ct, uint32_t C, uint32_t party, uint32_t receiver,
                                 uint32_t group, uint32_t ct_base, uint64_t *share, void *stream);
/* The converted ciphertext E' = (c0 + sum_k h0_k, sum_k h1_k), ct_out [C][2][L][N] (may not
 * alias ct).  shares: HOST array of K device pointers.                                      */
d2mhe_status d2mhe_convert_combine(d2mhe_ctx *ctx, const uint64_t *ct, const uint64_t *const *shares,
                                   uint32_t K, uint32_t C, uint64_t *ct_out, void *stream);
/* BFV.Decrypt with a single prepared secret key (Sec. 3.2 item 5): pt = [round(t (c0 + c1 sk) / Q)]_t,
 * pt [C][N]; rounding as in d2mhe_combine.                                                  */
d2mhe_status d2mhe_decrypt(d2mhe_ctx *ctx, const uint64_t *sk, const uint64_t *ct, uint32_t C,
                           uint64_t *pt, void *stream);

/* Receivers of a fused round: group g is converted to each of
 * receivers[recv_offsets[g] .. recv_offsets[g+1]) (party ids; at least one per group).  HOST
 * arrays of device pointers, as in d2mhe_round_desc.                                        */
typedef struct {
    const uint32_t *recv_offsets;    /* [G+1], recv_offsets[0] = 0, strictly increasing      */
    const uint32_t *receivers;       /* [recv_offsets[G]] party ids                          */
    const uint64_t *const *recv_pks; /* [P] prepared single-key public key by party id       */
    const uint64_t *const *recv_sks; /* [P] prepared single-key secret key by party id       */
    float *const *out_recv;          /* [recv_offsets[G]] result per (group, receiver)       */
} d2mhe_convert_desc;

/* Scratch bytes of d2mhe_round_convert; num_shares = sum over groups of members * receivers. */
size_t d2mhe_round_convert_scratch_bytes(const d2mhe_ctx *ctx, uint32_t num_jobs, uint32_t num_groups,
                                         uint32_t num_shares, uint64_t n_values);
/* d2mhe_round with the paper's decryption path: after the sum, every member of group g makes
 * one conversion share per receiver of g, and every receiver combines its shares with the
 * aggregate and decrypts with its own key into out_recv (desc->out_sums is not used).  The
 * scratch then holds the fresh ciphertexts [J][C][2][L][N], the aggregates [G][C][2][L][N] and
 * the conversion shares [num_shares][C][2][L][N], ordered by (group, receiver, member).
 * phase_events as in d2mhe_round.                                                           */
d2mhe_status d2mhe_round_convert(d2mhe_ctx *ctx, const d2mhe_round_desc *desc,
                                 const d2mhe_convert_desc *conv, void *scratch, size_t scratch_bytes,
                                 void *const *phase_events, void *stream);

/* ---- MBFV.Bootstrap: collective refresh of a ciphertext (Sec. 4.2 item 4, Eq. (3)) ------------- */
/* The members of a group turn a ciphertext ct = (c0, c1) under their collective key into a
 * fresh-like one (noise sum_k e1_k) of the same plaintext, without anybody learning it:
 * every member masks its decryption share with a random M_k in R_t.
 *
 * The common random polynomial alpha of ciphertext indices ct_base .. ct_base + C - 1 of a group,
 * uniform in R_q, evaluation form, alpha [C][L][N].                                         */
d2mhe_status d2mhe_bootstrap_alpha(d2mhe_ctx *ctx, uint32_t group, uint32_t ct_base, uint32_t C,
                                   uint64_t *alpha, void *stream);
/* Member `party`'s share, Eq. (3):
 *   (eta0, eta1) = (s_k c1 - Lambda M_k + e0_k, -s_k alpha + Lambda M_k + e1_k),  share [C][2][L][N],
 * M_k uniform in R_t, e0_k, e1_k from chi, randomness indexed by (party, group, ct_base + c).   */
d2mhe_status d2mhe_bootstrap_share(d2mhe_ctx *ctx, const uint64_t *sk_share, const uint64_t *ct,
                                   const uint64_t *alpha, uint32_t C, uint32_t party, uint32_t group,
                                   uint32_t ct_base, uint64_t *share, void *stream);
/* ct' = ([round(t/Q [c0 + sum_k eta0_k]_Q)]_t Lambda + sum_k eta1_k, alpha), ct_out [C][2][L][N]
 * (may not alias ct).  shares: HOST array of K device pointers.  Rounding as in d2mhe_combine. */
d2mhe_status d2mhe_bootstrap_combine(d2mhe_ctx *ctx, const uint64_t *ct, const uint64_t *alpha,
                                     const uint64_t *const *shares, uint32_t K, uint32_t C,
                                     uint64_t *ct_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif
