// C-ABI entry points of the d2mhe library (see include/d2mhe.h): parameter validation,
// host-side table construction and kernel launches.  No device memory is allocated here.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "ctx.hpp"
#include "stream_kernels.hpp"

using namespace d2;

namespace {

typedef unsigned __int128 u128;

// ---- host number theory (set-up only) -------------------------------------------------
uint64_t h_mul(uint64_t a, uint64_t b, uint64_t m) { return (uint64_t)((u128)a * b % m); }

uint64_t h_pow(uint64_t base, uint64_t exp, uint64_t m)
{
    uint64_t acc = 1 % m;
    for (base %= m; exp; exp >>= 1, base = h_mul(base, base, m))
        if (exp & 1) acc = h_mul(acc, base, m);
    return acc;
}

uint64_t h_inv(uint64_t a, uint64_t prime) { return h_pow(a, prime - 2, prime); }

// Miller-Rabin with the first twelve primes as witnesses: deterministic below 2^64.
bool h_is_prime(uint64_t n)
{
    const uint64_t wit[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return false;
    for (uint64_t p : wit) {
        if (n == p) return true;
        if (n % p == 0) return false;
    }
    int twos = 0;
    uint64_t odd = n - 1;
    while (!(odd & 1)) { odd >>= 1; ++twos; }
    for (uint64_t a : wit) {
        uint64_t y = h_pow(a, odd, n);
        if (y == 1 || y == n - 1) continue;
        bool composite = true;
        for (int i = 1; i < twos && composite; ++i) {
            y = h_mul(y, y, n);
            if (y == n - 1) composite = false;
        }
        if (composite) return false;
    }
    return true;
}

// psi = x^((m-1)/2N) for the smallest x >= 2 such that psi has order exactly 2N.
uint64_t h_root(uint64_t m, uint32_t log2n)
{
    const uint64_t n = 1ull << log2n, e = (m - 1) / (2 * n);
    for (uint64_t x = 2; x < m; ++x) {
        uint64_t psi = h_pow(x, e, m);
        if (h_pow(psi, n, m) == m - 1) return psi;
    }
    return 0;
}

uint64_t h_shoup(uint64_t w, uint64_t m) { return (uint64_t)(((u128)w << 64) / m); }

Tw h_tw(uint64_t w, uint64_t m)
{
    Tw t;
    t.w = w;
    t.ws = h_shoup(w, m);
    return t;
}

uint32_t h_bitrev(uint32_t v, int bits)
{
    uint32_t r = 0;
    for (int i = 0; i < bits; ++i) r |= ((v >> i) & 1u) << (bits - 1 - i);
    return r;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- engine shape per ring degree ----------------------------------------------------------
typedef const EngineOps *(*OpsGetter)();
const OpsGetter OPS_TABLE[4][7] = {
    {ops_f_10, ops_f_11, ops_f_12, ops_f_13, ops_f_14, ops_f_15, ops_f_16},
    {ops_s_10, ops_s_11, ops_s_12, ops_s_13, ops_s_14, ops_s_15, ops_s_16},
    {ops_b_10, ops_b_11, ops_b_12, ops_b_13, ops_b_14, ops_b_15, ops_b_16},
    {ops_w_10, ops_w_11, ops_w_12, ops_w_13, ops_w_14, ops_w_15, ops_w_16},
};
constexpr int ARITH_32 = 3;

const EngineOps *engine_ops(const d2mhe_ctx *ctx) { return OPS_TABLE[ctx->arith][ctx->log2n - 10](); }

// Arithmetic back-end from the largest modulus: 32-bit residues below 2^30, doubles below 2^44,
// 63-bit Shoup with an approximate quotient below 2^55, exact Harvey butterflies otherwise.
// Transforms modulo the plaintext modulus (< 2^30) always use the 32-bit back-end.
int arith_for(const d2mhe_params *p)
{
    uint64_t qmax = 0;
    for (uint32_t i = 0; i < p->num_limbs; ++i) qmax = p->q[i] > qmax ? p->q[i] : qmax;
    if (qmax < (1ull << 30)) return ARITH_32;
    if (qmax < (1ull << 44)) return 0;
    if (qmax < (1ull << 55)) return 1;
    return 2;
}

// table entry in the format of the back-end
Tw h_entry(int arith, uint64_t w, uint64_t m)
{
    Tw t;
    if (arith == 0) {
        const double d = (double)w;          // exact: w < 2^44
        std::memcpy(&t.w, &d, sizeof(d));
        t.ws = 0;
    } else if (arith == ARITH_32) {
        t.w = w | ((w << 32) / m) << 32;     // value and floor(w 2^32 / m) in one 8-byte word
        t.ws = 0;
    } else {
        t.w = w;
        t.ws = (uint64_t)(((unsigned __int128)w << 63) / m);
    }
    return t;
}

struct Layout {
    size_t tabs_off, tw_off, p1_off, total;
};

Layout layout_of(uint32_t log2n, uint32_t L, bool has_t)
{
    const size_t N = (size_t)1 << log2n;
    const uint32_t moduli = L + (has_t ? 1 : 0);
    Layout lo;
    lo.tabs_off = 0;
    lo.tw_off = align_up(sizeof(LimbTab) * (MAX_LIMBS + 1), 256);
    lo.p1_off = lo.tw_off + (size_t)moduli * 2 * N * sizeof(Tw);
    lo.total = lo.p1_off + (has_t ? (size_t)2 * L * N * sizeof(uint64_t) : 0);
    return lo;
}

bool params_ok(const d2mhe_params *p)
{
    if (!p || !p->q) return false;
    if (p->log2_n < 10 || p->log2_n > 16) return false;
    if (p->num_limbs < 1 || p->num_limbs > (uint32_t)MAX_LIMBS) return false;
    const uint64_t two_n = 2ull << p->log2_n;
    for (uint32_t i = 0; i < p->num_limbs; ++i) {
        const uint64_t q = p->q[i];
        if (q >> 61) return false;
        if (q % two_n != 1 || !h_is_prime(q)) return false;
        for (uint32_t j = 0; j < i; ++j)
            if (p->q[j] == q) return false;
    }
    if (p->t) {
        if (p->t >> 30) return false;
        if (p->t % two_n != 1 || !h_is_prime(p->t)) return false;
        for (uint32_t i = 0; i < p->num_limbs; ++i)
            if (p->t >= p->q[i]) return false;
        if (p->cbd_eta < 1 || p->cbd_eta > 32) return false;
        if (p->frac_bits > 30 || p->max_group < 1) return false;
    }
    return true;
}

}  // namespace

namespace {

bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

d2mhe_status launch_ntt(d2mhe_ctx *ctx, uint64_t *polys, uint32_t B, bool forward, hipStream_t st)
{
    return engine_ops(ctx)->ntt(ctx, polys, B, forward, st);
}

}  // namespace

// ---- scratch memory of d2mhe_round_group_static ------------------------------------------------
// A device array of the library's own, for callers that may not allocate.  In host code the name
// of a __device__ array is only a stand-in for the symbol, never a device address: its address on
// the current device comes from hipGetSymbolAddress, once per device (every device holds its own
// copy of the array), and only that pointer is ever handed to a kernel or a runtime call.
namespace {

static __device__ __align__(256) uint64_t static_scratch[D2MHE_STATIC_SCRATCH_BYTES / sizeof(uint64_t)];

constexpr int MAX_DEVICES = 64;
std::mutex g_static_lock;
uint64_t *g_static_ptr[MAX_DEVICES];      // address of static_scratch on device i, null until looked up

// Address of the array on the current device (looked up on first use; no allocation).
d2mhe_status static_scratch_ptr(d2mhe_ctx *ctx, uint64_t **out)
{
    int dev = -1;
    D2_HIP(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return D2MHE_ERR_RANGE;
    std::lock_guard<std::mutex> hold(g_static_lock);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        D2_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch)));
        if (!p) return D2MHE_ERR_HIP;
        g_static_ptr[dev] = (uint64_t *)p;
    }
    *out = g_static_ptr[dev];
    return D2MHE_OK;
}

}  // namespace

extern "C" {

const char *d2mhe_strerror(d2mhe_status s)
{
    switch (s) {
    case D2MHE_OK: return "ok";
    case D2MHE_ERR_BAD_PARAMS: return "invalid parameters";
    case D2MHE_ERR_NULL: return "null pointer";
    case D2MHE_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case D2MHE_ERR_RANGE: return "index or count out of range";
    case D2MHE_ERR_WORKSPACE: return "workspace or scratch too small";
    case D2MHE_ERR_HIP: return "HIP runtime error";
    case D2MHE_ERR_UNIMPLEMENTED: return "not implemented for these parameters";
    default: return "unknown status";
    }
}

size_t d2mhe_workspace_bytes(const d2mhe_params *p)
{
    if (!params_ok(p)) return 0;
    return layout_of(p->log2_n, p->num_limbs, p->t != 0).total;
}

d2mhe_status d2mhe_create(const d2mhe_params *p, void *dev_workspace, size_t bytes, void *stream,
                          d2mhe_ctx **out)
{
    if (!p || !out) return D2MHE_ERR_NULL;
    *out = nullptr;
    if (!p->q) return D2MHE_ERR_NULL;
    if (!params_ok(p)) return D2MHE_ERR_BAD_PARAMS;
    if (!dev_workspace) return D2MHE_ERR_NULL;
    if (misaligned(dev_workspace)) return D2MHE_ERR_ALIGN;
    const uint32_t L = p->num_limbs, log2n = p->log2_n;
    const size_t N = (size_t)1 << log2n;
    const bool has_t = p->t != 0;
    const Layout lo = layout_of(log2n, L, has_t);
    if (bytes < lo.total) return D2MHE_ERR_WORKSPACE;

    d2mhe_ctx *ctx = new (std::nothrow) d2mhe_ctx();
    if (!ctx) return D2MHE_ERR_HIP;
    ctx->log2n = log2n;
    ctx->L = L;
    ctx->N = N;
    ctx->t = p->t;
    ctx->max_group = p->max_group;
    ctx->arith = arith_for(p);
    ctx->last_hip = 0;
    // Long transforms run as launch pairs over at most 65535 polynomials (grid.y limit).  Smaller
    // chunks (to keep a chunk in the memory-side cache between the two kernels) were measured
    // and bring nothing on MI355X: the strided kernel already runs at copy speed.
    ctx->ntt_chunk_polys = 65535;
    char *ws = (char *)dev_workspace;
    ctx->d_tabs = (const LimbTab *)(ws + lo.tabs_off);
    ctx->d_p1 = has_t ? (uint64_t *)(ws + lo.p1_off) : nullptr;

    const uint32_t moduli = L + (has_t ? 1 : 0);
    std::vector<LimbTab> tabs(MAX_LIMBS + 1);
    std::memset(tabs.data(), 0, sizeof(LimbTab) * tabs.size());
    std::vector<Tw> tw((size_t)moduli * 2 * N);
    std::vector<uint64_t> pw(N);
    uint64_t q_mod_t = 1;
    for (uint32_t i = 0; has_t && i < L; ++i) q_mod_t = h_mul(q_mod_t, p->q[i] % p->t, p->t);
    for (uint32_t i = 0; i < moduli; ++i) {
        // slot L of the table array is the plaintext modulus
        const uint64_t m = i < L ? p->q[i] : p->t;
        const int ar = i < L ? ctx->arith : ARITH_32;      // table format of this modulus
        const uint64_t psi = h_root(m, log2n);
        if (i < L) ctx->q[i] = m;
        ctx->psi[i < L ? i : L] = psi;
        Tw *fwd = tw.data() + (size_t)i * 2 * N, *inv = fwd + N;
        pw[0] = 1;
        for (size_t k = 1; k < N; ++k) pw[k] = h_mul(pw[k - 1], psi, m);
        for (size_t k = 0; k < N; ++k) fwd[k] = h_entry(ar, pw[h_bitrev((uint32_t)k, (int)log2n)], m);
        const uint64_t psi_inv = h_inv(psi, m);
        for (size_t k = 1; k < N; ++k) pw[k] = h_mul(pw[k - 1], psi_inv, m);
        for (size_t k = 0; k < N; ++k) inv[k] = h_entry(ar, pw[h_bitrev((uint32_t)k, (int)log2n)], m);
        LimbTab &tb = tabs[i < L ? i : L];
        tb.q = m;
        if (ar == 0) {
            const double qinv = 1.0 / (double)m;
            std::memcpy(&tb.one_s, &qinv, sizeof(qinv));
        } else if (ar == ARITH_32) {
            tb.one_s = ((uint64_t)1 << 32) / m;
        } else {
            tb.one_s = (uint64_t)(((u128)1 << 63) / m);
        }
        tb.pow32 = h_tw((((uint64_t)1) << 32) % m, m);
        tb.inv64 = (uint64_t)((((u128)1) << 64) / m);
        const uint64_t ninv = h_inv((uint64_t)N % m, m);
        tb.ninv = h_entry(ar, ninv, m);
        tb.wn = h_entry(ar, h_mul(pw[h_bitrev(1u, (int)log2n)], ninv, m), m);   // inverse twiddle 1 times N^-1
        tb.fwd = (const Tw *)(ws + lo.tw_off) + (size_t)i * 2 * N;
        tb.inv = tb.fwd + N;
        if (i < L && has_t) {
            // floor(Q/t) = (Q - (Q mod t)) / t  and  Q = 0 (mod q_i)  =>  floor(Q/t) = -(Q mod t) t^-1 (mod q_i)
            const uint64_t lam = h_mul((m - q_mod_t % m) % m, h_inv(p->t % m, m), m);
            tb.lambda = h_entry(ar, lam, m);
            uint64_t others = 1;
            for (uint32_t j = 0; j < L; ++j)
                if (j != i) others = h_mul(others, p->q[j] % m, m);
            tb.gamma = h_tw(h_inv(others, m), m);      // always the integer pair
            const u128 num = (u128)p->t << 64;
            tb.theta_hi = (uint64_t)(num / m);
            tb.theta_lo = (uint64_t)(((num % m) << 64) / m);
        }
    }
    if (has_t && L < (uint32_t)MAX_LIMBS) { /* slot L already filled above */ }

    std::memset(&ctx->rc, 0, sizeof(ctx->rc));
    ctx->rc.t = p->t;
    ctx->rc.L = L;
    ctx->rc.key.k0 = (uint32_t)(p->seed & 0xffffffffu);
    ctx->rc.key.k1 = (uint32_t)(p->seed >> 32);
    if (has_t) {
        ctx->rc.eta_mask = p->cbd_eta >= 32 ? 0xffffffffu : ((1u << p->cbd_eta) - 1u);
        ctx->rc.clamp = (int32_t)(((p->t - 1) / 2) / p->max_group);
        ctx->rc.scale = (float)(1u << p->frac_bits);
        ctx->rc.inv_scale = 1.0f / (float)(1u << p->frac_bits);
    }

    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipMemcpy(ws + lo.tabs_off, tabs.data(), sizeof(LimbTab) * tabs.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(ws + lo.tw_off, tw.data(), tw.size() * sizeof(Tw), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        delete ctx;
        return D2MHE_ERR_HIP;
    }
    if (has_t) {
        // common random polynomial p1: uniform per limb, to evaluation form, with Shoup quotients
        const size_t total = (size_t)L * N;
        hipLaunchKernelGGL(k_uniform, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, ctx->d_p1,
                           ctx->d_tabs, L, log2n, (uint32_t)DOM_CRS, ctx->rc.key, total);
        d2mhe_status s = launch_ntt(ctx, ctx->d_p1, 1, true, st);
        if (s == D2MHE_OK) {
            PtrList src;
            src.p[0] = ctx->d_p1;
            hipLaunchKernelGGL(k_prepare, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, ctx->d_p1, src,
                               1u, ctx->d_tabs, log2n, total);
            if (hipGetLastError() != hipSuccess) s = D2MHE_ERR_HIP;
        }
        if (s == D2MHE_OK && hipStreamSynchronize(st) != hipSuccess) s = D2MHE_ERR_HIP;
        if (s != D2MHE_OK) {
            delete ctx;
            return s;
        }
    }
    // d2mhe_round_group_static's scratch array: look its address up now, with this device current
    uint64_t *own_scratch = nullptr;
    const d2mhe_status ss = static_scratch_ptr(ctx, &own_scratch);
    if (ss != D2MHE_OK) {
        delete ctx;
        return ss;
    }
    *out = ctx;
    return D2MHE_OK;
}

void d2mhe_destroy(d2mhe_ctx *ctx) { delete ctx; }

int d2mhe_last_hip_error(const d2mhe_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

uint64_t d2mhe_root(const d2mhe_ctx *ctx, uint32_t limb)
{
    if (!ctx || limb > ctx->L || (limb == ctx->L && !ctx->t)) return 0;
    return ctx->psi[limb];
}

d2mhe_status d2mhe_ntt_index_map(const d2mhe_ctx *ctx, uint32_t *perm)
{
    if (!ctx || !perm) return D2MHE_ERR_NULL;
    const EngineOps *ops = engine_ops(ctx);
    const int elog = ops->elog, logb = ops->logb;
    const uint32_t T = 1u << (logb - elog), NB = 1u << logb;
    for (uint32_t pos = 0; pos < ctx->N; ++pos) {
        const uint32_t blk = pos >> logb, lp = pos & (NB - 1);
        const uint32_t idx = (blk << logb) | ((lp % T) << elog) | (lp / T);
        perm[pos] = h_bitrev(idx, (int)ctx->log2n);
    }
    return D2MHE_OK;
}

d2mhe_status d2mhe_ntt_forward(d2mhe_ctx *ctx, uint64_t *polys, uint32_t B, void *stream)
{
    if (!ctx || !polys) return D2MHE_ERR_NULL;
    if (misaligned(polys)) return D2MHE_ERR_ALIGN;
    if (B == 0) return D2MHE_OK;
    if ((uint64_t)B * ctx->L > 0x7fffffffull) return D2MHE_ERR_RANGE;
    return launch_ntt(ctx, polys, B, true, (hipStream_t)stream);
}

d2mhe_status d2mhe_ntt_inverse(d2mhe_ctx *ctx, uint64_t *polys, uint32_t B, void *stream)
{
    if (!ctx || !polys) return D2MHE_ERR_NULL;
    if (misaligned(polys)) return D2MHE_ERR_ALIGN;
    if (B == 0) return D2MHE_OK;
    if ((uint64_t)B * ctx->L > 0x7fffffffull) return D2MHE_ERR_RANGE;
    return launch_ntt(ctx, polys, B, false, (hipStream_t)stream);
}

d2mhe_status d2mhe_bench_polys(d2mhe_ctx *ctx, uint64_t *out, uint32_t B, void *stream)
{
    if (!ctx || !out) return D2MHE_ERR_NULL;
    if (misaligned(out)) return D2MHE_ERR_ALIGN;
    if (B == 0) return D2MHE_OK;
    const size_t total = (size_t)B * ctx->L * ctx->N;
    hipLaunchKernelGGL(k_uniform, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, out,
                       ctx->d_tabs, ctx->L, ctx->log2n, (uint32_t)DOM_BENCH, ctx->rc.key, total);
    D2_LAUNCHED(ctx);
    return D2MHE_OK;
}

#define D2_NEED_SCHEME(ctx)                                          \
    do {                                                             \
        if (!(ctx)) return D2MHE_ERR_NULL;                           \
        if (!(ctx)->t) return D2MHE_ERR_BAD_PARAMS;                  \
        if ((ctx)->log2n > 14) return D2MHE_ERR_UNIMPLEMENTED;       \
    } while (0)

d2mhe_status d2mhe_keygen_share(d2mhe_ctx *ctx, uint32_t party, uint64_t *sk_share, uint64_t *pk0_share,
                                void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!sk_share || !pk0_share) return D2MHE_ERR_NULL;
    if (misaligned(sk_share) || misaligned(pk0_share)) return D2MHE_ERR_ALIGN;
    if (party > 0xffffu) return D2MHE_ERR_RANGE;
    return engine_ops(ctx)->keygen(ctx, party, sk_share, pk0_share, (hipStream_t)stream);
}

d2mhe_status d2mhe_aggregate_pk(d2mhe_ctx *ctx, const uint64_t *const *pk0_shares, uint32_t K, uint64_t *pk,
                                void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!pk0_shares || !pk) return D2MHE_ERR_NULL;
    if (K == 0 || K > (uint32_t)MAX_GROUP || K > ctx->max_group) return D2MHE_ERR_RANGE;
    if (misaligned(pk)) return D2MHE_ERR_ALIGN;
    PtrList src;
    for (uint32_t k = 0; k < K; ++k) {
        if (!pk0_shares[k]) return D2MHE_ERR_NULL;
        if (misaligned(pk0_shares[k])) return D2MHE_ERR_ALIGN;
        src.p[k] = pk0_shares[k];
    }
    const size_t total = (size_t)ctx->L * ctx->N;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(k_prepare, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, pk, src, K, ctx->d_tabs,
                       ctx->log2n, total);
    D2_LAUNCHED(ctx);
    D2_HIP(ctx, hipMemcpyAsync(pk + 2 * total, ctx->d_p1, 2 * total * sizeof(uint64_t), hipMemcpyDeviceToDevice, st));
    return D2MHE_OK;
}

d2mhe_status d2mhe_encode(d2mhe_ctx *ctx, const float *grad, uint64_t n_values, uint64_t *pt, uint32_t C,
                          void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!pt || (!grad && n_values)) return D2MHE_ERR_NULL;
    if (misaligned(pt) || misaligned(grad)) return D2MHE_ERR_ALIGN;
    if (n_values > (uint64_t)C * ctx->N) return D2MHE_ERR_RANGE;
    if (C == 0) return D2MHE_OK;
    return engine_ops(ctx)->encode(ctx, grad, n_values, pt, C, (hipStream_t)stream);
}

d2mhe_status d2mhe_decode(d2mhe_ctx *ctx, const uint64_t *pt, uint32_t C, uint64_t n_values, float *out,
                          void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!pt || (!out && n_values)) return D2MHE_ERR_NULL;
    if (misaligned(pt) || misaligned(out)) return D2MHE_ERR_ALIGN;
    if (n_values > (uint64_t)C * ctx->N) return D2MHE_ERR_RANGE;
    if (C == 0) return D2MHE_OK;
    return engine_ops(ctx)->decode(ctx, pt, C, n_values, out, (hipStream_t)stream);
}

// Coefficient packing (value j of a ciphertext is coefficient j): the same launchers with the
// packing flag set in a private copy of the context.
d2mhe_status d2mhe_encode_coefficients(d2mhe_ctx *ctx, const float *grad, uint64_t n_values, uint64_t *pt,
                                       uint32_t C, void *stream)
{
    D2_NEED_SCHEME(ctx);
    d2mhe_ctx local = *ctx;
    local.rc.coeff_packing = 1;
    const d2mhe_status s = d2mhe_encode(&local, grad, n_values, pt, C, stream);
    ctx->last_hip = local.last_hip;
    return s;
}

d2mhe_status d2mhe_decode_coefficients(d2mhe_ctx *ctx, const uint64_t *pt, uint32_t C, uint64_t n_values,
                                       float *out, void *stream)
{
    D2_NEED_SCHEME(ctx);
    d2mhe_ctx local = *ctx;
    local.rc.coeff_packing = 1;
    const d2mhe_status s = d2mhe_decode(&local, pt, C, n_values, out, stream);
    ctx->last_hip = local.last_hip;
    return s;
}

d2mhe_status d2mhe_encrypt(d2mhe_ctx *ctx, const uint64_t *pk, const uint64_t *pt, uint32_t C, uint32_t party,
                           uint32_t group, uint32_t ct_base, uint64_t *ct, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!pk || !pt || !ct) return D2MHE_ERR_NULL;
    if (misaligned(pk) || misaligned(pt) || misaligned(ct)) return D2MHE_ERR_ALIGN;
    if (party > 0xffffu || group > 0xffffu || (uint64_t)ct_base + C > 0xffffffffull) return D2MHE_ERR_RANGE;
    if (C == 0) return D2MHE_OK;
    EncJobs jobs;
    jobs.src[0] = pt;
    jobs.pk[0] = pk;
    jobs.out[0] = ct;
    jobs.party[0] = party;
    jobs.group[0] = group;
    return engine_ops(ctx)->encrypt(ctx, false, jobs, 1, ct_base, 0, C, (hipStream_t)stream);
}

d2mhe_status d2mhe_add(d2mhe_ctx *ctx, uint64_t *ct_acc, const uint64_t *ct_in, uint32_t C, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!ct_acc || !ct_in) return D2MHE_ERR_NULL;
    if (misaligned(ct_acc) || misaligned(ct_in)) return D2MHE_ERR_ALIGN;
    if (C == 0) return D2MHE_OK;
    PtrList src;
    src.p[0] = ct_acc;
    src.p[1] = ct_in;
    const size_t total = (size_t)C * 2 * ctx->L * ctx->N;
    hipLaunchKernelGGL(k_sum, dim3((unsigned)((total / 2 + 255) / 256)), dim3(256), 0, (hipStream_t)stream, ct_acc,
                       src, 2u, ctx->d_tabs, ctx->L, ctx->log2n, total);
    D2_LAUNCHED(ctx);
    return D2MHE_OK;
}

d2mhe_status d2mhe_partial_decrypt(d2mhe_ctx *ctx, const uint64_t *sk_share, const uint64_t *ct, uint32_t C,
                                   uint32_t party, uint32_t group, uint32_t ct_base, uint64_t *share, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!sk_share || !ct || !share) return D2MHE_ERR_NULL;
    if (misaligned(sk_share) || misaligned(ct) || misaligned(share)) return D2MHE_ERR_ALIGN;
    if (party > 0xffffu || group > 0xffffu || (uint64_t)ct_base + C > 0xffffffffull) return D2MHE_ERR_RANGE;
    if (C == 0) return D2MHE_OK;
    ShareJobs jobs;
    jobs.sk[0] = sk_share;
    jobs.ct[0] = ct;
    jobs.out[0] = share;
    jobs.party[0] = party;
    jobs.group[0] = group;
    return engine_ops(ctx)->share(ctx, jobs, 1, ct_base, C, (hipStream_t)stream);
}

d2mhe_status d2mhe_combine(d2mhe_ctx *ctx, const uint64_t *ct, const uint64_t *const *shares, uint32_t K, uint32_t C,
                           uint64_t *pt, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!ct || !shares || !pt) return D2MHE_ERR_NULL;
    if (K == 0 || K > (uint32_t)MAX_GROUP || K > ctx->max_group) return D2MHE_ERR_RANGE;
    if (misaligned(ct) || misaligned(pt)) return D2MHE_ERR_ALIGN;
    PtrList sh;
    for (uint32_t k = 0; k < K; ++k) {
        if (!shares[k]) return D2MHE_ERR_NULL;
        if (misaligned(shares[k])) return D2MHE_ERR_ALIGN;
        sh.p[k] = shares[k];
    }
    if (C == 0) return D2MHE_OK;
    return engine_ops(ctx)->combine(ctx, ct, sh, K, C, pt, (hipStream_t)stream);
}

// ---- MBFV.Convert ------------------------------------------------------------------------------

d2mhe_status d2mhe_receiver_keygen(d2mhe_ctx *ctx, uint32_t party, uint64_t *sk, uint64_t *pk, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!sk || !pk) return D2MHE_ERR_NULL;
    if (misaligned(sk) || misaligned(pk)) return D2MHE_ERR_ALIGN;
    if (party > 0xffffu) return D2MHE_ERR_RANGE;
    return engine_ops(ctx)->receiver_keygen(ctx, party, sk, pk, (hipStream_t)stream);
}

d2mhe_status d2mhe_convert_share(d2mhe_ctx *ctx, const uint64_t *sk_share, const uint64_t *pk_recv,
                                 const uint64_t *ct, uint32_t C, uint32_t party, uint32_t receiver, uint32_t group,
                                 uint32_t ct_base, uint64_t *share, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!sk_share || !pk_recv || !ct || !share) return D2MHE_ERR_NULL;
    if (misaligned(sk_share) || misaligned(pk_recv) || misaligned(ct) || misaligned(share)) return D2MHE_ERR_ALIGN;
    if (party > 0xffffu || receiver > 0xffffu || group > 0xffffu || (uint64_t)ct_base + C > 0xffffffffull)
        return D2MHE_ERR_RANGE;
    if (C == 0) return D2MHE_OK;
    ConvJobs jobs;
    jobs.sk[0] = sk_share;
    jobs.pk[0] = pk_recv;
    jobs.ct[0] = ct;
    jobs.out[0] = share;
    jobs.who[0] = party | (receiver << 16);
    jobs.group[0] = group;
    return engine_ops(ctx)->convert_share(ctx, jobs, 1, ct_base, C, (hipStream_t)stream);
}

d2mhe_status d2mhe_convert_combine(d2mhe_ctx *ctx, const uint64_t *ct, const uint64_t *const *shares, uint32_t K,
                                   uint32_t C, uint64_t *ct_out, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!ct || !shares || !ct_out) return D2MHE_ERR_NULL;
    if (K == 0 || K > (uint32_t)MAX_GROUP || K > ctx->max_group) return D2MHE_ERR_RANGE;
    if (misaligned(ct) || misaligned(ct_out)) return D2MHE_ERR_ALIGN;
    PtrList sh;
    for (uint32_t k = 0; k < K; ++k) {
        if (!shares[k]) return D2MHE_ERR_NULL;
        if (misaligned(shares[k])) return D2MHE_ERR_ALIGN;
        sh.p[k] = shares[k];
    }
    if (C == 0) return D2MHE_OK;
    const size_t LN = (size_t)ctx->L * ctx->N, total = (size_t)C * 2 * LN;
    hipLaunchKernelGGL(k_convert_sum, dim3((unsigned)((total / 2 + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       ct_out, ct, sh, K, ctx->d_tabs, ctx->L, ctx->log2n, LN, total);
    D2_LAUNCHED(ctx);
    return D2MHE_OK;
}

d2mhe_status d2mhe_decrypt(d2mhe_ctx *ctx, const uint64_t *sk, const uint64_t *ct, uint32_t C, uint64_t *pt,
                           void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!sk || !ct || !pt) return D2MHE_ERR_NULL;
    if (misaligned(sk) || misaligned(ct) || misaligned(pt)) return D2MHE_ERR_ALIGN;
    if (C == 0) return D2MHE_OK;
    PtrList none;
    none.p[0] = nullptr;
    return engine_ops(ctx)->convert_combine(ctx, ct, none, 0, sk, true, C, pt, (hipStream_t)stream);
}

// ---- MBFV.Bootstrap ----------------------------------------------------------------------------

d2mhe_status d2mhe_bootstrap_alpha(d2mhe_ctx *ctx, uint32_t group, uint32_t ct_base, uint32_t C, uint64_t *alpha,
                                   void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!alpha) return D2MHE_ERR_NULL;
    if (misaligned(alpha)) return D2MHE_ERR_ALIGN;
    if (group > 0xffffu || (uint64_t)ct_base + C > 0xffffffffull || C > 0xffffu * 0x10000ull) return D2MHE_ERR_RANGE;
    if (C == 0) return D2MHE_OK;
    return engine_ops(ctx)->bootstrap_alpha(ctx, group, ct_base, C, alpha, (hipStream_t)stream);
}

d2mhe_status d2mhe_bootstrap_share(d2mhe_ctx *ctx, const uint64_t *sk_share, const uint64_t *ct,
                                   const uint64_t *alpha, uint32_t C, uint32_t party, uint32_t group,
                                   uint32_t ct_base, uint64_t *share, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!sk_share || !ct || !alpha || !share) return D2MHE_ERR_NULL;
    if (misaligned(sk_share) || misaligned(ct) || misaligned(alpha) || misaligned(share)) return D2MHE_ERR_ALIGN;
    if (party > 0xffffu || group > 0xffffu || (uint64_t)ct_base + C > 0xffffffffull) return D2MHE_ERR_RANGE;
    if (C == 0) return D2MHE_OK;
    ConvJobs jobs;
    jobs.sk[0] = sk_share;
    jobs.pk[0] = alpha;
    jobs.ct[0] = ct;
    jobs.out[0] = share;
    jobs.who[0] = party;
    jobs.group[0] = group;
    return engine_ops(ctx)->bootstrap_share(ctx, jobs, 1, ct_base, C, (hipStream_t)stream);
}

d2mhe_status d2mhe_bootstrap_combine(d2mhe_ctx *ctx, const uint64_t *ct, const uint64_t *alpha,
                                     const uint64_t *const *shares, uint32_t K, uint32_t C, uint64_t *ct_out,
                                     void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!ct || !alpha || !shares || !ct_out) return D2MHE_ERR_NULL;
    if (K == 0 || K > (uint32_t)MAX_GROUP || K > ctx->max_group) return D2MHE_ERR_RANGE;
    if (misaligned(ct) || misaligned(alpha) || misaligned(ct_out)) return D2MHE_ERR_ALIGN;
    PtrList sh;
    for (uint32_t k = 0; k < K; ++k) {
        if (!shares[k]) return D2MHE_ERR_NULL;
        if (misaligned(shares[k])) return D2MHE_ERR_ALIGN;
        sh.p[k] = shares[k];
    }
    if (C == 0) return D2MHE_OK;
    return engine_ops(ctx)->bootstrap_combine(ctx, ct, sh, K, alpha, C, ct_out, (hipStream_t)stream);
}

// ---- the float step of one training iteration (Alg. 2 lines 9-10) -----------------------------

d2mhe_status d2mhe_average_update(const float *sum, uint32_t K, const float *grad, float gamma, uint64_t n,
                                  float *w, void *stream)
{
    if (!sum || !w || (!grad && gamma != 0.0f)) return D2MHE_ERR_NULL;
    if (K == 0) return D2MHE_ERR_RANGE;
    if (n == 0) return D2MHE_OK;
    if (n > 0xffffffffull * 256ull) return D2MHE_ERR_RANGE;
    hipLaunchKernelGGL(k_average_update, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, sum,
                       1.0f / (float)K, grad, gamma, n, w);
    if (hipGetLastError() != hipSuccess) return D2MHE_ERR_HIP;
    return D2MHE_OK;
}

namespace {

// a party listed twice among the (at most MAX_GROUP) members of a group
bool has_duplicates(const uint32_t *members, uint32_t K)
{
    for (uint32_t a = 1; a < K; ++a)
        for (uint32_t b = 0; b < a; ++b)
            if (members[a] == members[b]) return true;
    return false;
}

// words of scratch for J (party, group) jobs, G groups, C ciphertext indices; S conversion shares
// (0: collective decryption, one single-polynomial share per job)
size_t round_words(const d2mhe_ctx *ctx, uint64_t J, uint64_t G, uint64_t S, uint64_t C)
{
    const size_t LN = (size_t)ctx->L * ctx->N;
    const size_t shares = S ? (size_t)S * 2 * LN : (size_t)J * LN;
    return (size_t)C * ((size_t)J * 2 * LN + (size_t)G * 2 * LN + shares);
}

// One exchange round; conv == nullptr: collective decryption of every aggregate, otherwise key
// switching to every receiver (MBFV.Convert) and single-key decryption.
d2mhe_status run_round(d2mhe_ctx *ctx, const d2mhe_round_desc *d, const d2mhe_convert_desc *conv, void *scratch,
                       size_t scratch_bytes, void *const *phase_events, void *stream)
{
    if (!d || !scratch) return D2MHE_ERR_NULL;
    if (!d->group_offsets || !d->members || !d->pks || !d->sk_shares || !d->grads) return D2MHE_ERR_NULL;
    if (!conv && !d->out_sums) return D2MHE_ERR_NULL;
    if (conv && (!conv->recv_offsets || !conv->receivers || !conv->recv_pks || !conv->recv_sks || !conv->out_recv))
        return D2MHE_ERR_NULL;
    const uint32_t G = d->num_groups;
    if (G == 0 || G > 0xffffu) return D2MHE_ERR_RANGE;
    if (d->group_offsets[0] != 0) return D2MHE_ERR_RANGE;
    const uint32_t J = d->group_offsets[G];
    for (uint32_t g = 0; g < G; ++g) {
        if (d->group_offsets[g + 1] <= d->group_offsets[g]) return D2MHE_ERR_RANGE;
        const uint32_t K = d->group_offsets[g + 1] - d->group_offsets[g];
        if (K > (uint32_t)MAX_GROUP || K > ctx->max_group) return D2MHE_ERR_RANGE;
        if (!d->pks[g]) return D2MHE_ERR_NULL;
        if (misaligned(d->pks[g])) return D2MHE_ERR_ALIGN;
        if (!conv) {
            if (!d->out_sums[g]) return D2MHE_ERR_NULL;
            if (misaligned(d->out_sums[g])) return D2MHE_ERR_ALIGN;
        }
    }
    // The Philox counters hold 16 bits of group id and of party id, and a (party, group id) pair names one
    // stream of randomness: ids beyond 16 bits, two groups with one id or a member listed twice in a group
    // would make two encryptions share their mu, e0, e1.
    if (d->group_ids) {
        std::vector<uint32_t> ids(d->group_ids, d->group_ids + G);
        std::sort(ids.begin(), ids.end());
        if (ids.back() > 0xffffu) return D2MHE_ERR_RANGE;
        if (std::adjacent_find(ids.begin(), ids.end()) != ids.end()) return D2MHE_ERR_RANGE;
    }
    for (uint32_t g = 0; g < G; ++g)
        if (has_duplicates(d->members + d->group_offsets[g], d->group_offsets[g + 1] - d->group_offsets[g]))
            return D2MHE_ERR_RANGE;
    for (uint32_t j = 0; j < J; ++j) {
        const uint32_t party = d->members[j];
        if (party >= d->num_parties || party > 0xffffu) return D2MHE_ERR_RANGE;
        if (!d->sk_shares[party] || !d->grads[party]) return D2MHE_ERR_NULL;
        if (misaligned(d->sk_shares[party]) || misaligned(d->grads[party])) return D2MHE_ERR_ALIGN;
    }
    uint64_t S = 0;          // conversion shares
    uint32_t R = 0;          // (group, receiver) pairs
    if (conv) {
        if (conv->recv_offsets[0] != 0) return D2MHE_ERR_RANGE;
        for (uint32_t g = 0; g < G; ++g) {
            if (conv->recv_offsets[g + 1] <= conv->recv_offsets[g]) return D2MHE_ERR_RANGE;
            S += (uint64_t)(conv->recv_offsets[g + 1] - conv->recv_offsets[g]) *
                 (d->group_offsets[g + 1] - d->group_offsets[g]);
        }
        R = conv->recv_offsets[G];
        if (S > 0xffffffffull) return D2MHE_ERR_RANGE;
        for (uint32_t r = 0; r < R; ++r) {
            const uint32_t party = conv->receivers[r];
            if (party >= d->num_parties || party > 0xffffu) return D2MHE_ERR_RANGE;
            if (!conv->recv_pks[party] || !conv->recv_sks[party] || !conv->out_recv[r]) return D2MHE_ERR_NULL;
            if (misaligned(conv->recv_pks[party]) || misaligned(conv->recv_sks[party]) || misaligned(conv->out_recv[r]))
                return D2MHE_ERR_ALIGN;
        }
    }
    if (misaligned(scratch)) return D2MHE_ERR_ALIGN;
    if (d->n_values == 0) return D2MHE_OK;
    const uint64_t C64 = (d->n_values + ctx->N - 1) / ctx->N;
    if (C64 > 0x7fffffffull || (uint64_t)d->ct_base + C64 > 0xffffffffull) return D2MHE_ERR_RANGE;
    const uint32_t C = (uint32_t)C64;
    if (scratch_bytes < round_words(ctx, J, G, S, C) * sizeof(uint64_t)) return D2MHE_ERR_WORKSPACE;

    const size_t LN = (size_t)ctx->L * ctx->N;
    const size_t ct_words = (size_t)C * 2 * LN, sh_words = (size_t)C * LN;
    uint64_t *cts = (uint64_t *)scratch;
    uint64_t *agg = cts + (size_t)J * ct_words;
    uint64_t *shares = agg + (size_t)G * ct_words;
    hipStream_t st = (hipStream_t)stream;
    const EngineOps *ops = engine_ops(ctx);
    hipEvent_t *ev = (hipEvent_t *)phase_events;
    if (ev && ev[0]) D2_HIP(ctx, hipEventRecord(ev[0], st));

    // phase 1: every member of every group encodes and encrypts its gradient
    std::vector<uint32_t> group_of(J);
    for (uint32_t g = 0; g < G; ++g)
        for (uint32_t j = d->group_offsets[g]; j < d->group_offsets[g + 1]; ++j) group_of[j] = g;
    for (uint32_t j0 = 0; j0 < J; j0 += JOB_CHUNK) {
        const uint32_t n = J - j0 < (uint32_t)JOB_CHUNK ? J - j0 : (uint32_t)JOB_CHUNK;
        EncJobs jobs;
        for (uint32_t i = 0; i < n; ++i) {
            const uint32_t j = j0 + i, g = group_of[j];
            jobs.src[i] = d->grads[d->members[j]];
            jobs.pk[i] = d->pks[g];
            jobs.out[i] = cts + (size_t)j * ct_words;
            jobs.party[i] = d->members[j];
            jobs.group[i] = d->group_ids ? d->group_ids[g] : g;
        }
        d2mhe_status s = ops->encrypt(ctx, true, jobs, n, d->ct_base, d->n_values, C, st);
        if (s != D2MHE_OK) return s;
    }
    if (ev && ev[1]) D2_HIP(ctx, hipEventRecord(ev[1], st));

    // phase 2: homomorphic sum per group
    for (uint32_t g0 = 0; g0 < G; g0 += JOB_CHUNK) {
        const uint32_t n = G - g0 < (uint32_t)JOB_CHUNK ? G - g0 : (uint32_t)JOB_CHUNK;
        GroupJobs jobs;
        for (uint32_t i = 0; i < n; ++i) {
            const uint32_t g = g0 + i;
            jobs.first[i] = cts + (size_t)d->group_offsets[g] * ct_words;
            jobs.ct[i] = nullptr;
            jobs.out[i] = agg + (size_t)g * ct_words;
            jobs.K[i] = d->group_offsets[g + 1] - d->group_offsets[g];
        }
        hipLaunchKernelGGL(k_sum_groups, dim3((unsigned)((ct_words / 2 + 255) / 256), n), dim3(256), 0, st, jobs,
                           ct_words, ctx->d_tabs, ctx->L, ctx->log2n, ct_words);
        D2_LAUNCHED(ctx);
    }
    if (ev && ev[2]) D2_HIP(ctx, hipEventRecord(ev[2], st));

    if (!conv) {
        // phase 3: every member's decryption share of its group's aggregate
        for (uint32_t j0 = 0; j0 < J; j0 += JOB_CHUNK) {
            const uint32_t n = J - j0 < (uint32_t)JOB_CHUNK ? J - j0 : (uint32_t)JOB_CHUNK;
            ShareJobs jobs;
            for (uint32_t i = 0; i < n; ++i) {
                const uint32_t j = j0 + i, g = group_of[j];
                jobs.sk[i] = d->sk_shares[d->members[j]];
                jobs.ct[i] = agg + (size_t)g * ct_words;
                jobs.out[i] = shares + (size_t)j * sh_words;
                jobs.party[i] = d->members[j];
                jobs.group[i] = d->group_ids ? d->group_ids[g] : g;
            }
            d2mhe_status s = ops->share(ctx, jobs, n, d->ct_base, C, st);
            if (s != D2MHE_OK) return s;
        }
        if (ev && ev[3]) D2_HIP(ctx, hipEventRecord(ev[3], st));

        // phase 4: combine the shares, round, decode
        for (uint32_t g0 = 0; g0 < G; g0 += JOB_CHUNK) {
            const uint32_t n = G - g0 < (uint32_t)JOB_CHUNK ? G - g0 : (uint32_t)JOB_CHUNK;
            GroupJobs jobs;
            for (uint32_t i = 0; i < n; ++i) {
                const uint32_t g = g0 + i;
                jobs.first[i] = shares + (size_t)d->group_offsets[g] * sh_words;
                jobs.ct[i] = agg + (size_t)g * ct_words;
                jobs.out[i] = d->out_sums[g];
                jobs.K[i] = d->group_offsets[g + 1] - d->group_offsets[g];
            }
            d2mhe_status s = ops->combine_decode(ctx, jobs, n, sh_words, C, d->n_values, st);
            if (s != D2MHE_OK) return s;
        }
        if (ev && ev[4]) D2_HIP(ctx, hipEventRecord(ev[4], st));
        return D2MHE_OK;
    }

    // phase 3 (Convert): one share per (group, receiver, member), in that order
    struct ShareRef {
        uint32_t g, r, j;      // group, index into receivers, index into members
    };
    std::vector<ShareRef> refs;
    refs.reserve((size_t)S);
    std::vector<size_t> first_share(R);     // position of the first share of a (group, receiver) pair
    for (uint32_t g = 0; g < G; ++g)
        for (uint32_t r = conv->recv_offsets[g]; r < conv->recv_offsets[g + 1]; ++r) {
            first_share[r] = refs.size();
            for (uint32_t j = d->group_offsets[g]; j < d->group_offsets[g + 1]; ++j) refs.push_back(ShareRef{g, r, j});
        }
    for (size_t s0 = 0; s0 < refs.size(); s0 += CONV_CHUNK) {
        const uint32_t n = (uint32_t)(refs.size() - s0 < (size_t)CONV_CHUNK ? refs.size() - s0 : (size_t)CONV_CHUNK);
        ConvJobs jobs;
        for (uint32_t i = 0; i < n; ++i) {
            const ShareRef &f = refs[s0 + i];
            const uint32_t member = d->members[f.j], receiver = conv->receivers[f.r];
            jobs.sk[i] = d->sk_shares[member];
            jobs.pk[i] = conv->recv_pks[receiver];
            jobs.ct[i] = agg + (size_t)f.g * ct_words;
            jobs.out[i] = shares + (s0 + i) * ct_words;
            jobs.who[i] = member | (receiver << 16);
            jobs.group[i] = d->group_ids ? d->group_ids[f.g] : f.g;
        }
        d2mhe_status s = ops->convert_share(ctx, jobs, n, d->ct_base, C, st);
        if (s != D2MHE_OK) return s;
    }
    if (ev && ev[3]) D2_HIP(ctx, hipEventRecord(ev[3], st));

    // phase 4 (Convert): every receiver forms its ciphertext, decrypts with its own key, decodes
    for (uint32_t r0 = 0; r0 < R; r0 += CONV_CHUNK) {
        const uint32_t n = R - r0 < (uint32_t)CONV_CHUNK ? R - r0 : (uint32_t)CONV_CHUNK;
        RecvJobs jobs;
        uint32_t g = 0;
        for (uint32_t i = 0; i < n; ++i) {
            const uint32_t r = r0 + i;
            while (conv->recv_offsets[g + 1] <= r) ++g;
            jobs.first[i] = shares + first_share[r] * ct_words;
            jobs.ct[i] = agg + (size_t)g * ct_words;
            jobs.sk[i] = conv->recv_sks[conv->receivers[r]];
            jobs.out[i] = conv->out_recv[r];
            jobs.K[i] = d->group_offsets[g + 1] - d->group_offsets[g];
        }
        d2mhe_status s = ops->convert_combine_decode(ctx, jobs, n, ct_words, C, d->n_values, st);
        if (s != D2MHE_OK) return s;
    }
    if (ev && ev[4]) D2_HIP(ctx, hipEventRecord(ev[4], st));
    return D2MHE_OK;
}

}  // namespace

size_t d2mhe_round_scratch_bytes(const d2mhe_ctx *ctx, uint32_t num_jobs, uint32_t num_groups, uint64_t n_values)
{
    if (!ctx || !ctx->t || num_jobs == 0 || num_groups == 0) return 0;
    const uint64_t C = (n_values + ctx->N - 1) / ctx->N;
    return round_words(ctx, num_jobs, num_groups, 0, C) * sizeof(uint64_t);
}

size_t d2mhe_round_convert_scratch_bytes(const d2mhe_ctx *ctx, uint32_t num_jobs, uint32_t num_groups,
                                         uint32_t num_shares, uint64_t n_values)
{
    if (!ctx || !ctx->t || num_jobs == 0 || num_groups == 0 || num_shares == 0) return 0;
    const uint64_t C = (n_values + ctx->N - 1) / ctx->N;
    return round_words(ctx, num_jobs, num_groups, num_shares, C) * sizeof(uint64_t);
}

// The packing of the round travels in a private copy of the context (the launchers read the
// per-context constants from it).
d2mhe_status run_round_packed(d2mhe_ctx *ctx, const d2mhe_round_desc *d, const d2mhe_convert_desc *conv,
                              void *scratch, size_t scratch_bytes, void *const *phase_events, void *stream)
{
    if (!d) return D2MHE_ERR_NULL;
    if (d->packing > 1) return D2MHE_ERR_RANGE;
    d2mhe_ctx local = *ctx;
    local.rc.coeff_packing = d->packing;
    const d2mhe_status s = run_round(&local, d, conv, scratch, scratch_bytes, phase_events, stream);
    ctx->last_hip = local.last_hip;
    return s;
}

d2mhe_status d2mhe_round(d2mhe_ctx *ctx, const d2mhe_round_desc *d, void *scratch, size_t scratch_bytes,
                         void *const *phase_events, void *stream)
{
    D2_NEED_SCHEME(ctx);
    return run_round_packed(ctx, d, nullptr, scratch, scratch_bytes, phase_events, stream);
}

d2mhe_status d2mhe_round_convert(d2mhe_ctx *ctx, const d2mhe_round_desc *d, const d2mhe_convert_desc *conv,
                                 void *scratch, size_t scratch_bytes, void *const *phase_events, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!conv) return D2MHE_ERR_NULL;
    return run_round_packed(ctx, d, conv, scratch, scratch_bytes, phase_events, stream);
}

d2mhe_status d2mhe_round_group(d2mhe_ctx *ctx, const uint64_t *pk, const uint64_t *const *sk_shares,
                               const float *const *grads, const uint32_t *members, uint32_t K, uint32_t group,
                               uint64_t n_values, float *out_sum, void *scratch, size_t scratch_bytes, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!pk || !sk_shares || !grads || !members || !out_sum || !scratch) return D2MHE_ERR_NULL;
    if (K == 0 || K > (uint32_t)MAX_GROUP || K > ctx->max_group || group > 0xffffu) return D2MHE_ERR_RANGE;
    // a one-group round
    uint32_t offsets[2] = {0, K};
    for (uint32_t k = 0; k < K; ++k)
        if (members[k] > 0xffffu) return D2MHE_ERR_RANGE;
    if (has_duplicates(members, K)) return D2MHE_ERR_RANGE;
    // pointer tables indexed by party id: build sparse views of size max id + 1
    uint32_t max_id = 0;
    for (uint32_t k = 0; k < K; ++k) max_id = members[k] > max_id ? members[k] : max_id;
    std::vector<const uint64_t *> sk_by_party(max_id + 1, nullptr);
    std::vector<const float *> grad_by_party(max_id + 1, nullptr);
    for (uint32_t k = 0; k < K; ++k) {
        sk_by_party[members[k]] = sk_shares[k];
        grad_by_party[members[k]] = grads[k];
    }
    d2mhe_round_desc d;
    d.num_groups = 1;
    d.group_offsets = offsets;
    d.members = members;
    d.group_ids = &group;
    d.pks = &pk;
    d.num_parties = max_id + 1;
    d.sk_shares = sk_by_party.data();
    d.grads = grad_by_party.data();
    d.out_sums = &out_sum;
    d.n_values = n_values;
    d.ct_base = 0;
    d.packing = 0;
    return d2mhe_round(ctx, &d, scratch, scratch_bytes, nullptr, stream);
}

// d2mhe_round_group for callers that may not allocate: the same four launches on the library's own
// scratch array.  Nothing here touches the heap or the device allocator: the job tables are on the
// stack (K <= 64 fits one launch per phase) and travel in the kernel arguments.
d2mhe_status d2mhe_round_group_static(d2mhe_ctx *ctx, const uint64_t *pk, const uint64_t *const *sk_shares,
                                      const float *const *grads, const uint32_t *members, uint32_t K,
                                      uint32_t group, uint64_t n_values, float *out_sum, void *stream)
{
    D2_NEED_SCHEME(ctx);
    if (!pk || !sk_shares || !grads || !members || !out_sum) return D2MHE_ERR_NULL;
    if (K == 0 || K > (uint32_t)MAX_GROUP || K > ctx->max_group || group > 0xffffu) return D2MHE_ERR_RANGE;
    static_assert(MAX_GROUP <= JOB_CHUNK, "a group must fit one launch");
    if (misaligned(pk) || misaligned(out_sum)) return D2MHE_ERR_ALIGN;
    for (uint32_t k = 0; k < K; ++k) {
        if (members[k] > 0xffffu) return D2MHE_ERR_RANGE;
        if (!sk_shares[k] || !grads[k]) return D2MHE_ERR_NULL;
        if (misaligned(sk_shares[k]) || misaligned(grads[k])) return D2MHE_ERR_ALIGN;
    }
    if (has_duplicates(members, K)) return D2MHE_ERR_RANGE;
    if (n_values == 0) return D2MHE_OK;
    const uint64_t C64 = (n_values + ctx->N - 1) / ctx->N;
    if (C64 > 0x7fffffffull) return D2MHE_ERR_RANGE;
    const uint32_t C = (uint32_t)C64;
    // the limit: the scratch of this round must fit the array
    const size_t LN = (size_t)ctx->L * ctx->N;
    if (C64 > D2MHE_STATIC_SCRATCH_BYTES / sizeof(uint64_t) / ((size_t)(3 * K + 2) * LN)) return D2MHE_ERR_WORKSPACE;
    uint64_t *base = nullptr;
    const d2mhe_status ps = static_scratch_ptr(ctx, &base);       // the device address, never the array's name
    if (ps != D2MHE_OK) return ps;

    const size_t ct_words = (size_t)C * 2 * LN, sh_words = (size_t)C * LN;
    uint64_t *cts = base, *agg = cts + (size_t)K * ct_words, *shares = agg + ct_words;
    hipStream_t st = (hipStream_t)stream;
    const EngineOps *ops = engine_ops(ctx);
    d2mhe_ctx local = *ctx;                  // slot packing, whatever a concurrent call sets in its own copy
    local.rc.coeff_packing = 0;

    EncJobs enc;
    ShareJobs shr;
    for (uint32_t k = 0; k < K; ++k) {
        enc.src[k] = grads[k];
        enc.pk[k] = pk;
        enc.out[k] = cts + (size_t)k * ct_words;
        enc.party[k] = shr.party[k] = members[k];
        enc.group[k] = shr.group[k] = group;
        shr.sk[k] = sk_shares[k];
        shr.ct[k] = agg;
        shr.out[k] = shares + (size_t)k * sh_words;
    }
    d2mhe_status s = ops->encrypt(&local, true, enc, K, 0, n_values, C, st);
    if (s == D2MHE_OK) {
        GroupJobs sum;
        sum.first[0] = cts;
        sum.ct[0] = nullptr;
        sum.out[0] = agg;
        sum.K[0] = K;
        hipLaunchKernelGGL(k_sum_groups, dim3((unsigned)((ct_words / 2 + 255) / 256), 1), dim3(256), 0, st, sum,
                           ct_words, ctx->d_tabs, ctx->L, ctx->log2n, ct_words);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            local.last_hip = (int)e;
            s = D2MHE_ERR_HIP;
        }
    }
    if (s == D2MHE_OK) s = ops->share(&local, shr, K, 0, C, st);
    if (s == D2MHE_OK) {
        GroupJobs cmb;
        cmb.first[0] = shares;
        cmb.ct[0] = agg;
        cmb.out[0] = out_sum;
        cmb.K[0] = K;
        s = ops->combine_decode(&local, cmb, 1, sh_words, C, n_values, st);
    }
    ctx->last_hip = local.last_hip;
    return s;
}

}  // extern "C"
