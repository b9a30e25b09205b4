// Host build of the library's modular-arithmetic policies (paper_2207_04604_amd/csrc/arith.hpp, the
// plain-C side of every block) checked against 128-bit integer arithmetic: every operation must give
// the residue it documents, inside the range it documents, for inputs anywhere in the range it
// accepts -- including the ends of those ranges, word boundaries and the largest moduli a policy
// takes, which random ciphertext data practically never reaches.  Compiled and run by
// tests/test_host_logic.py; prints one line per policy and exits non-zero on the first violation.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define D2_DEV inline
static inline double __longlong_as_double(long long v) { double d; std::memcpy(&d, &v, 8); return d; }
static inline long long __double_as_longlong(double d) { long long v; std::memcpy(&v, &d, 8); return v; }
static inline uint32_t __umulhi(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * b) >> 32); }
static inline uint64_t __umul64hi(uint64_t a, uint64_t b) { return (uint64_t)(((unsigned __int128)a * b) >> 64); }

#include "../paper_2207_04604_amd/csrc/arith.hpp"

typedef unsigned __int128 u128;
typedef __int128 i128;
using namespace d2;

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd()
{   // splitmix64
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint64_t below(uint64_t n) { return n ? (uint64_t)(((u128)rnd() * n) >> 64) : 0; }

static int failures = 0;
#define CHECK(cond, ...)                                         \
    do {                                                         \
        if (!(cond)) {                                           \
            std::printf("FAILED %s:%d  ", __FILE__, __LINE__);   \
            std::printf(__VA_ARGS__);                            \
            std::printf("\n");                                   \
            if (++failures > 10) std::exit(1);                   \
        }                                                        \
    } while (0)

// values of [0, bound) worth trying: both ends, multiples of q, word boundaries, random ones
static std::vector<uint64_t> probes(uint64_t bound, uint64_t q, int n_random)
{
    std::vector<uint64_t> v;
    const uint64_t fixed[] = {0, 1, 2, q - 1, q, q + 1, 2 * q - 1, 2 * q, 2 * q + 1, 4 * q - 1, 4 * q, 0xffffffffull,
                              0x100000000ull, 0x100000001ull, 0x7fffffffull, 0x80000000ull, bound - 1, bound - 2,
                              bound / 2, bound / 2 + 1, bound - 0x100000000ull, (bound - 1) & ~0xffffffffull,
                              ((bound - 1) & ~0xffffffffull) - 1};
    for (uint64_t f : fixed)
        if (f < bound) v.push_back(f);
    for (int i = 0; i < n_random; ++i) v.push_back(below(bound));
    for (int i = 0; i < n_random / 4; ++i) v.push_back(bound - 1 - below(bound < 1000 ? bound : 1000));
    return v;
}
static std::vector<uint64_t> multiplicands(uint64_t q, int n_random)
{
    std::vector<uint64_t> v = {0, 1, 2, q - 1, q - 2, q / 2, q / 2 + 1, 0xffffffffull % q, 0x100000000ull % q};
    for (int i = 0; i < n_random; ++i) v.push_back(below(q));
    return v;
}
static uint64_t mod_of(i128 v, uint64_t q)
{
    i128 r = v % (i128)q;
    return (uint64_t)(r < 0 ? r + q : r);
}

// ------------------------------------------------------------------ the two 64-bit integer policies
// in_fwd: exclusive bound on the inputs of a forward butterfly; grow: what a forward stage may add to it;
// prod: exclusive bound of a lazy product; in_inv: bound of the inverse butterflies' values; in_mul: of mul's y
template <class A>
static void check_u64(const char *name, uint64_t q, uint64_t in_mul, uint64_t in_fwd, uint64_t prod_q, uint64_t in_inv_q,
                      bool fwd_grows, uint64_t wide, uint64_t acc_q)
{
    const uint64_t one_s = (uint64_t)(((u128)1 << 63) / q);
    const typename A::Mod md = A::mod(q, one_s);
    const auto ws = multiplicands(q, 40);
    for (uint64_t w : ws) {
        const typename A::Twid tw = A::tw(w, (uint64_t)(((u128)w << 64) / q));      // from the 64-bit quotient
        Tw entry{w, (uint64_t)(((u128)w << 63) / q)};
        const typename A::Twid tw2 = A::tw(entry);
        CHECK(tw.w == tw2.w && tw.ws == tw2.ws, "%s twiddle forms differ w=%llu", name, (unsigned long long)w);
        for (uint64_t y : probes(in_mul, q, 300)) {
            const uint64_t r = A::mul(y, tw, md);
            CHECK(r < prod_q * q && r % q == (uint64_t)(((u128)w * y) % q), "%s mul q=%llu w=%llu y=%llu -> %llu", name,
                  (unsigned long long)q, (unsigned long long)w, (unsigned long long)y, (unsigned long long)r);
        }
        for (uint64_t y : probes(1ull << 32, q, 300)) {                    // a 32-bit operand (plaintext coefficient)
            const uint64_t r = A::mul_u32((uint32_t)y, tw, md);
            CHECK(r < prod_q * q && r % q == (uint64_t)(((u128)w * y) % q), "%s mul_u32 q=%llu w=%llu y=%llu -> %llu", name,
                  (unsigned long long)q, (unsigned long long)w, (unsigned long long)y, (unsigned long long)r);
        }
        // forward butterfly
        for (uint64_t x0 : probes(in_fwd, q, 40))
            for (uint64_t y0 : probes(in_fwd, q, 12)) {
                uint64_t x = x0, y = y0;
                A::ct(x, y, tw, md);
                const uint64_t t = (uint64_t)(((u128)w * y0) % q);
                bool ok = x % q == (x0 % q + t) % q && y % q == (x0 % q + q - t) % q;
                if (fwd_grows) ok = ok && x < x0 + prod_q * q && y <= x0 + prod_q * q && x >= x0;
                else ok = ok && x < in_fwd && y < in_fwd;
                CHECK(ok, "%s ct q=%llu w=%llu x=%llu y=%llu -> %llu %llu", name, (unsigned long long)q,
                      (unsigned long long)w, (unsigned long long)x0, (unsigned long long)y0, (unsigned long long)x,
                      (unsigned long long)y);
            }
        // first stage on small samples
        for (int xv = -32; xv <= 32; xv += (xv == -32 || xv == 31) ? 1 : 7)
            for (int yv = -32; yv <= 32; ++yv) {
                uint64_t x, y;
                A::ct_small(xv, yv, x, y, tw, md);
                const uint64_t ex = mod_of((i128)xv + (i128)w * yv, q), ey = mod_of((i128)xv - (i128)w * yv, q);
                const uint64_t lim = fwd_grows ? 64 * q + 33 : in_fwd;
                CHECK(x % q == ex && y % q == ey && x < lim && y < lim, "%s ct_small q=%llu w=%llu %d %d", name,
                      (unsigned long long)q, (unsigned long long)w, xv, yv);
            }
        // inverse butterflies
        for (uint64_t x0 : probes(in_inv_q * q, q, 40))
            for (uint64_t y0 : probes(in_inv_q * q, q, 12)) {
                uint64_t x = x0, y = y0;
                A::gs(x, y, tw, md);
                const uint64_t d = (x0 % q + q - y0 % q) % q;
                CHECK(x < in_inv_q * q && y < in_inv_q * q && x % q == (x0 % q + y0 % q) % q &&
                          y % q == (uint64_t)(((u128)w * d) % q),
                      "%s gs q=%llu w=%llu x=%llu y=%llu", name, (unsigned long long)q, (unsigned long long)w,
                      (unsigned long long)x0, (unsigned long long)y0);
                x = x0, y = y0;
                A::gs_last(x, y, tw, tw, md);
                CHECK(x < in_inv_q * q && y < in_inv_q * q &&
                          x % q == (uint64_t)(((u128)w * ((x0 % q + y0 % q) % q)) % q) &&
                          y % q == (uint64_t)(((u128)w * d) % q),
                      "%s gs_last q=%llu w=%llu x=%llu y=%llu", name, (unsigned long long)q, (unsigned long long)w,
                      (unsigned long long)x0, (unsigned long long)y0);
            }
    }
    for (uint64_t x : probes(wide, q, 200000)) CHECK(A::canon_wide(x, md) == x % q, "%s canon_wide %llu", name, (unsigned long long)x);
    for (uint64_t x : probes(4 * q, q, 20000)) CHECK(A::canon_lazy(x, md) == x % q, "%s canon_lazy %llu", name, (unsigned long long)x);
    for (uint64_t x : probes(acc_q, q, 20000)) CHECK(A::canon_acc(x, md) == x % q, "%s canon_acc %llu", name, (unsigned long long)x);
    for (uint64_t x : probes(in_inv_q * q, q, 20000)) CHECK(A::canon_inv(x, md) == x % q, "%s canon_inv %llu", name, (unsigned long long)x);
    for (uint64_t x : probes(fwd_grows ? wide : in_fwd, q, 20000)) CHECK(A::canon_fwd(x, md) == x % q, "%s canon_fwd %llu", name, (unsigned long long)x);
    for (int v = -40; v <= 40; ++v) CHECK(A::from_small(v, md) == mod_of(v, q), "%s from_small %d", name, v);
    for (int v = -32; v <= 32; ++v)
        for (uint64_t x : probes(prod_q * q, q, 50)) {
            const uint64_t r = A::add_small(x, v, md);
            CHECK(r % q == mod_of((i128)x + v, q) && r < (prod_q + 1) * q + 33, "%s add_small %llu %d", name, (unsigned long long)x, v);
        }
}

// ------------------------------------------------------------------ 32-bit residues
static void check_32(uint64_t q64)
{
    typedef Arith32 A;
    const uint32_t q = (uint32_t)q64;
    const A::Mod md = A::mod(q64);
    CHECK(md.one_s == (uint32_t)(((uint64_t)1 << 32) / q) && A::mod(q64, md.one_s).nq == 0u - q, "Arith32 mod");
    auto p32 = [&](uint64_t bound, int n) {
        std::vector<uint32_t> v;
        for (uint64_t x : probes(bound, q, n)) v.push_back((uint32_t)x);
        return v;
    };
    for (uint64_t w64 : multiplicands(q, 60)) {
        const uint32_t w = (uint32_t)w64;
        const A::Twid tw = A::tw(w, (uint64_t)(((u128)w << 64) / q));
        const A::Twid tw2 = A::tw(Tw{w | ((((uint64_t)w << 32) / q) << 32), 0});
        CHECK(tw.w == tw2.w && tw.ws == tw2.ws, "Arith32 twiddle forms differ w=%u", w);
        for (uint32_t y : p32((uint64_t)1 << 32, 2000)) {
            const uint32_t r = A::mul(y, tw, md);
            CHECK(r < 2 * (uint64_t)q && r % q == (uint32_t)(((uint64_t)w * y) % q), "Arith32 mul q=%u w=%u y=%u -> %u", q, w, y, r);
        }
        for (uint32_t y : p32((uint64_t)1 << 32, 300)) {
            const uint32_t r = A::mul_u32(y, tw, md);
            CHECK(r < 2 * (uint64_t)q && r % q == (uint32_t)(((uint64_t)w * y) % q), "Arith32 mul_u32 q=%u w=%u y=%u", q, w, y);
        }
        for (uint32_t x0 : p32(4 * q64, 60))
            for (uint32_t y0 : p32(4 * q64, 20)) {
                uint32_t x = x0, y = y0;
                A::ct(x, y, tw, md);
                const uint32_t t = (uint32_t)(((uint64_t)w * y0) % q);
                CHECK(x < 4 * q64 && y < 4 * q64 && x % q == (x0 % q + t) % q && y % q == (x0 % q + q - t) % q,
                      "Arith32 ct q=%u w=%u x=%u y=%u", q, w, x0, y0);
                uint32_t e = x;
                A::fwd_end(e, md);
                CHECK(e < 2 * q64 && e % q == x % q, "Arith32 fwd_end %u", x);
            }
        for (int xv = -32; xv <= 32; xv += 8)
            for (int yv = -32; yv <= 32; ++yv) {
                uint32_t x, y;
                A::ct_small(xv, yv, x, y, tw, md);
                CHECK(x < 4 * q64 && y < 4 * q64 && x % q == mod_of((i128)xv + (i128)w * yv, q) &&
                          y % q == mod_of((i128)xv - (i128)w * yv, q), "Arith32 ct_small q=%u w=%u %d %d", q, w, xv, yv);
            }
        for (uint32_t x0 : p32(2 * q64, 60))
            for (uint32_t y0 : p32(2 * q64, 20)) {
                uint32_t x = x0, y = y0;
                A::gs(x, y, tw, md);
                const uint32_t d = (x0 % q + q - y0 % q) % q;
                CHECK(x < 2 * q64 && y < 2 * q64 && x % q == (x0 % q + y0 % q) % q && y % q == (uint32_t)(((uint64_t)w * d) % q),
                      "Arith32 gs q=%u w=%u x=%u y=%u", q, w, x0, y0);
                x = x0, y = y0;
                A::gs_last(x, y, tw, tw, md);
                CHECK(x < 2 * q64 && y < 2 * q64 && x % q == (uint32_t)(((uint64_t)w * ((x0 % q + y0 % q) % q)) % q) &&
                          y % q == (uint32_t)(((uint64_t)w * d) % q), "Arith32 gs_last q=%u w=%u x=%u y=%u", q, w, x0, y0);
            }
    }
    for (uint32_t x : p32((uint64_t)1 << 32, 400000)) CHECK(A::canon_wide(x, md) == x % q, "Arith32 canon_wide %u", x);
    for (uint32_t x : p32(4 * q64, 40000)) {
        CHECK(A::canon_lazy(x, md) == x % q && A::canon_fwd(x, md) == x % q && A::canon_acc(x, md) == x % q, "Arith32 canon_lazy %u", x);
    }
    for (uint32_t x : p32(2 * q64, 40000)) CHECK(A::canon_inv(x, md) == x % q, "Arith32 canon_inv %u", x);
    for (int v = -40; v <= 40; ++v) CHECK(A::from_small(v, md) == mod_of(v, q), "Arith32 from_small %d", v);
    for (int v = -32; v <= 32; ++v)
        for (uint32_t x : p32(2 * q64, 50)) {
            const uint32_t r = A::add_small(x, v, md);
            CHECK(r % q == mod_of((i128)x + v, q) && r < 3 * q64, "Arith32 add_small %u %d", x, v);
        }
}

// ------------------------------------------------------------------ residues in doubles
static double dnear(i128 v) { return (double)(long long)v; }       // |v| < 2^53 here: exact
static void check_f(uint64_t q)
{
    typedef ArithF A;
    const A::Mod md = A::mod(q);
    const double qd = (double)q;
    for (uint64_t v : probes((uint64_t)1 << 52, q, 2000)) CHECK(A::d2u(A::u2d(v)) == v && A::u2d(v) == (double)v, "ArithF u2d %llu", (unsigned long long)v);
    // signed values whose magnitude stays below `bound`
    auto signed_probes = [&](uint64_t bound, int n) {
        std::vector<double> v;
        for (uint64_t x : probes(bound, q, n)) { v.push_back((double)x); v.push_back(-(double)x); }
        return v;
    };
    const uint64_t lim40 = 64 * q + 1;                              // canon_wide takes |x| <= 64 q
    // magnitude bound of a product w*y: q/2 + 1.5 |w y| 2^-52 (+1 for the roundings of the bound itself)
    auto prod_bound = [&](uint64_t w, double y) { return qd / 2 + 1.5 * (double)w * std::fabs(y) * 0x1p-52 + 1.0; };
    for (uint64_t w64 : multiplicands(q, 60)) {
        const A::Twid tw = A::tw(w64, 0);
        // mul: |w y| < 2^96; the lazily reduced values of a transform stay below 40 q < 2^50
        for (double y : signed_probes(lim40, 600)) {
            const double r = A::mul(y, tw, md);
            const i128 exact = (i128)w64 * (i128)(long long)y;
            CHECK(r == std::floor(r) && std::fabs(r) <= prod_bound(w64, y) && mod_of((i128)(long long)r, q) == mod_of(exact, q),
                  "ArithF mul q=%llu w=%llu y=%.0f -> %.0f", (unsigned long long)q, (unsigned long long)w64, y, r);
        }
        for (uint64_t y : probes(1ull << 30, q, 300)) {                    // plaintext coefficients are below 2^30
            const double r = A::mul_u32((uint32_t)y, tw, md);
            CHECK(std::fabs(r) <= prod_bound(w64, (double)y) && mod_of((i128)(long long)r, q) == (uint64_t)(((u128)w64 * y) % q),
                  "ArithF mul_u32 q=%llu w=%llu y=%llu", (unsigned long long)q, (unsigned long long)w64, (unsigned long long)y);
        }
        for (double x0 : signed_probes(63 * q, 40))
            for (double y0 : signed_probes(lim40, 12)) {
                double x = x0, y = y0;
                A::ct(x, y, tw, md);
                const i128 t = (i128)w64 * (i128)(long long)y0;
                CHECK(std::fabs(x) <= std::fabs(x0) + prod_bound(w64, y0) && std::fabs(y) <= std::fabs(x0) + prod_bound(w64, y0) &&
                          mod_of((i128)(long long)x, q) == mod_of((i128)(long long)x0 + t, q) &&
                          mod_of((i128)(long long)y, q) == mod_of((i128)(long long)x0 - t, q),
                      "ArithF ct q=%llu w=%llu x=%.0f y=%.0f", (unsigned long long)q, (unsigned long long)w64, x0, y0);
            }
        for (int xv = -32; xv <= 32; xv += 8)
            for (int yv = -32; yv <= 32; ++yv) {
                double x, y;
                A::ct_small(xv, yv, x, y, tw, md);
                CHECK(x == dnear((i128)xv + (i128)w64 * yv) && y == dnear((i128)xv - (i128)w64 * yv), "ArithF ct_small %d %d", xv, yv);
            }
        for (double x0 : signed_probes(q, 40))
            for (double y0 : signed_probes(q, 12)) {
                double x = x0, y = y0;
                A::gs(x, y, tw, md);
                const i128 d = (i128)(long long)x0 - (i128)(long long)y0;
                CHECK(x == x0 + y0 && std::fabs(y) <= prod_bound(w64, x0 - y0) && mod_of((i128)(long long)y, q) == mod_of((i128)w64 * d, q),
                      "ArithF gs q=%llu w=%llu x=%.0f y=%.0f", (unsigned long long)q, (unsigned long long)w64, x0, y0);
            }
    }
    for (double x : signed_probes(lim40, 200000)) {
        const uint64_t want = mod_of((i128)(long long)x, q);
        CHECK(A::canon_wide(x, md) == want, "ArithF canon_wide q=%llu x=%.0f -> %llu", (unsigned long long)q, x,
              (unsigned long long)A::canon_wide(x, md));
        const double r = A::reduce(x, md);
        CHECK(std::fabs(r) <= qd / 2 + std::fabs(x) * 0x1p-51 + 1 && mod_of((i128)(long long)r, q) == want, "ArithF reduce x=%.0f", x);
    }
}

int main()
{
    // csub and the canonical helpers
    for (int i = 0; i < 200000; ++i) {
        const uint64_t m = (rnd() >> (rnd() % 40)) | 1, x = below(m > (1ull << 62) ? m : 2 * m);
        CHECK(csub(x, m) == (x >= m ? x - m : x), "csub %llu %llu", (unsigned long long)x, (unsigned long long)m);
        const uint64_t q = (rnd() >> (3 + rnd() % 40)) | 1, a = below(q), b = below(q), y = rnd();
        CHECK(add_mod(a, b, q) == (uint64_t)(((u128)a + b) % q), "add_mod");
        CHECK(mul_shoup64(y, a, (uint64_t)(((u128)a << 64) / q), q) == (uint64_t)(((u128)a * y) % q), "mul_shoup64");
        CHECK(shoup_quotient(a, q) == (uint64_t)(((u128)a << 64) / q), "shoup_quotient");
    }
    std::printf("helpers ok\n");

    // ArithS: moduli below 2^55 (the largest one it may be given, the benchmark's 54-bit primes, small ones).
    // Forward values are never corrected: inputs up to 2^62 - 4q, a stage adds less than 4q.  Inverse values
    // and lazy products in [0, 4q).
    for (uint64_t q : {(1ull << 55) - 1, 18014398508400641ull, 18014398507794433ull, (1ull << 44) + 1, 12289ull, 65537ull})
        check_u64<ArithS>("ArithS", q, 1ull << 62, (1ull << 62) - 4 * q, 4, 4, true, 1ull << 62, 1ull << 62);
    std::printf("ArithS ok\n");
    // ArithB: moduli below 2^61; forward values in [0, 4q), inverse values and lazy products in [0, 2q);
    // mul takes any y below 2^63; canon_acc takes a forward value plus a lazy product.
    for (uint64_t q : {(1ull << 61) - 1, 1152921504606584833ull, 1152921504570802177ull, (1ull << 55) + 3, 12289ull})
        check_u64<ArithB>("ArithB", q, 1ull << 63, 4 * q, 2, 2, false, 1ull << 63, 6 * q);
    std::printf("ArithB ok\n");
    for (uint64_t q : {(1ull << 30) - 1, 1073707009ull, 12289ull, 65537ull, 786433ull, 3ull << 28})
        check_32(q);
    std::printf("Arith32 ok\n");
    for (uint64_t q : {(1ull << 44) - 1, 68719403009ull, 68719206401ull, 17592186028033ull, 12289ull, 1073707009ull})
        check_f(q);
    std::printf("ArithF ok\n");
    if (failures) return 1;
    std::printf("all arithmetic policies hold their contracts\n");
    return 0;
}
