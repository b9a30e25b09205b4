// Device build of the library's modular-arithmetic policies (paper_2207_04604_amd/csrc/arith.hpp, the
// inline-assembly side of every block) checked on the GPU against 128-bit integer arithmetic on the
// host: the same contracts as tests/arith_host_check.cpp (which covers the plain-C side), on inputs at
// the ends of every documented range, at word boundaries and for the largest moduli each policy takes.
// Built by __graft_entry__.build() (or by the test itself if missing) and run by
// tests/test_gpu_shape_sweep.py; prints one line per policy and exits non-zero on a violation.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_2207_04604_amd/csrc/arith.hpp"

typedef unsigned __int128 u128;
typedef __int128 i128;
using namespace d2;

#define HIP_OK(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(2);                                                              \
        }                                                                              \
    } while (0)

static uint64_t rng_state = 0x243F6A8885A308D3ull;
static uint64_t rnd()
{
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint64_t below(uint64_t n) { return (uint64_t)(((u128)rnd() * n) >> 64); }

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

// One work item = one (x, y, w) triple; the kernel evaluates every operation of the policy on it.
struct Item {
    uint64_t x, y, w, ws64;     // ws64 = floor(w 2^64 / q)
    int32_t sx, sy;             // small signed inputs of the first-stage short cut
};
struct Out {
    uint64_t mul, mul32, ct_x, ct_y, cs_x, cs_y, gs_x, gs_y, gl_x, gl_y, wide, lazy, acc, inv, fwd, addsm;
};

template <class A>
__global__ void k_eval(const Item *in, Out *out, int n, uint64_t q, uint64_t aux)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const Item it = in[i];
    const typename A::Mod md = A::mod(q, aux);
    const typename A::Twid tw = A::tw(it.w, it.ws64);
    Out o;
    typedef typename A::elem elem;
    auto E = [&](uint64_t v) { return from_bits<A>(v); };          // raw bits -> element (doubles travel as bits)
    auto B = [&](elem v) { return to_bits<A>(v); };
    o.mul = B(A::mul(E(it.y), tw, md));
    o.mul32 = B(A::mul_u32((uint32_t)(it.sx & 0x3fffffff) | (uint32_t)(it.y & 0x3fffffffu), tw, md));
    elem a = E(it.x), b = E(it.y);
    A::ct(a, b, tw, md);
    o.ct_x = B(a); o.ct_y = B(b);
    A::ct_small(it.sx, it.sy, a, b, tw, md);
    o.cs_x = B(a); o.cs_y = B(b);
    o.gs_x = o.gs_y = o.gl_x = o.gl_y = o.wide = o.lazy = o.acc = o.inv = o.fwd = o.addsm = 0;
    out[i] = o;
}

// The inverse butterflies and the reductions get their own kernel: their input ranges differ from ct's.
template <class A>
__global__ void k_eval_inv(const Item *in, Out *out, int n, uint64_t q, uint64_t aux)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const Item it = in[i];
    const typename A::Mod md = A::mod(q, aux);
    const typename A::Twid tw = A::tw(it.w, it.ws64);
    typedef typename A::elem elem;
    auto E = [&](uint64_t v) { return from_bits<A>(v); };
    auto B = [&](elem v) { return to_bits<A>(v); };
    Out o = out[i];
    elem a = E(it.x), b = E(it.y);
    A::gs(a, b, tw, md);
    o.gs_x = B(a); o.gs_y = B(b);
    a = E(it.x); b = E(it.y);
    A::gs_last(a, b, tw, tw, md);
    o.gl_x = B(a); o.gl_y = B(b);
    o.lazy = A::canon_lazy(E(it.x), md);
    o.inv = A::canon_inv(E(it.x), md);
    o.addsm = B(A::add_small(E(it.y), it.sx, md));
    out[i] = o;
}
template <class A>
__global__ void k_eval_wide(const Item *in, Out *out, int n, uint64_t q, uint64_t aux)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const typename A::Mod md = A::mod(q, aux);
    Out o = out[i];
    o.wide = A::canon_wide(from_bits<A>(in[i].x), md);
    o.acc = A::canon_acc(from_bits<A>(in[i].y), md);
    o.fwd = A::canon_fwd(from_bits<A>(in[i].w), md);        // (field reuse: w carries the canon_fwd input)
    out[i] = o;
}

static int failures = 0;
#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            std::printf("FAILED line %d  ", __LINE__);    \
            std::printf(__VA_ARGS__);                     \
            std::printf("\n");                            \
            if (++failures > 10) std::exit(1);            \
        }                                                 \
    } while (0)

template <class K, class... Args>
static void run(K kernel, std::vector<Item> &items, std::vector<Out> &outs, Item *d_in, Out *d_out, Args... args)
{
    const int n = (int)items.size();
    HIP_OK(hipMemcpy(d_in, items.data(), n * sizeof(Item), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_out, outs.data(), n * sizeof(Out), hipMemcpyHostToDevice));
    hipLaunchKernelGGL(kernel, dim3((n + 255) / 256), dim3(256), 0, 0, (const Item *)d_in, d_out, n, args...);
    HIP_OK(hipGetLastError());
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(outs.data(), d_out, n * sizeof(Out), hipMemcpyDeviceToHost));
}

constexpr int MAX_ITEMS = 1 << 20;

// ---------------------------------------------------------------- 64-bit integer policies and the 32-bit one
// fwd_in: exclusive bound of forward-butterfly inputs; prod_q: lazy products lie in [0, prod_q q); inv_q: inverse
// values in [0, inv_q q); grows: forward values are never corrected (bounds relative to the input);
// wide: canon_wide's domain; acc: canon_acc's; fwdc: canon_fwd's; mul_in: mul's y.
template <class A>
static void check_int(const char *name, uint64_t q, uint64_t aux, uint64_t mul_in, uint64_t fwd_in, uint64_t prod_q,
                      uint64_t inv_q, bool grows, uint64_t wide, uint64_t acc, uint64_t fwdc, Item *d_in, Out *d_out)
{
    std::vector<Item> items;
    const auto ws = multiplicands(q, 24);
    const auto ys = probes(mul_in < fwd_in ? mul_in : fwd_in, q, 120);
    const auto xs = probes(fwd_in, q, 30);
    for (uint64_t w : ws)
        for (uint64_t y : ys)
            for (size_t xi = 0; xi < xs.size() && (int)items.size() < MAX_ITEMS; xi += 1 + (size_t)(rnd() % 5)) {
                Item it;
                it.x = xs[xi]; it.y = y; it.w = w; it.ws64 = (uint64_t)(((u128)w << 64) / q);
                it.sx = (int32_t)(rnd() % 65) - 32; it.sy = (int32_t)(rnd() % 65) - 32;
                items.push_back(it);
            }
    std::vector<Out> outs(items.size());
    run(k_eval<A>, items, outs, d_in, d_out, q, aux);
    for (size_t i = 0; i < items.size(); ++i) {
        const Item &it = items[i];
        const Out &o = outs[i];
        const uint64_t t = (uint64_t)(((u128)it.w * it.y) % q);
        CHECK(o.mul < prod_q * q && o.mul % q == t, "%s mul q=%llu w=%llu y=%llu -> %llu", name, (unsigned long long)q,
              (unsigned long long)it.w, (unsigned long long)it.y, (unsigned long long)o.mul);
        const uint32_t y32 = (uint32_t)(it.sx & 0x3fffffff) | (uint32_t)(it.y & 0x3fffffffu);
        CHECK(o.mul32 < prod_q * q && o.mul32 % q == (uint64_t)(((u128)it.w * y32) % q), "%s mul_u32 q=%llu w=%llu y=%u", name,
              (unsigned long long)q, (unsigned long long)it.w, y32);
        bool ok = o.ct_x % q == (it.x % q + t) % q && o.ct_y % q == (it.x % q + q - t) % q;
        if (grows) ok = ok && o.ct_x < it.x + prod_q * q && o.ct_y <= it.x + prod_q * q && o.ct_x >= it.x;
        else ok = ok && o.ct_x < fwd_in && o.ct_y < fwd_in;
        CHECK(ok, "%s ct q=%llu w=%llu x=%llu y=%llu -> %llu %llu", name, (unsigned long long)q, (unsigned long long)it.w,
              (unsigned long long)it.x, (unsigned long long)it.y, (unsigned long long)o.ct_x, (unsigned long long)o.ct_y);
        const uint64_t lim = grows ? 64 * q + 33 : fwd_in;
        CHECK(o.cs_x % q == mod_of((i128)it.sx + (i128)it.w * it.sy, q) && o.cs_y % q == mod_of((i128)it.sx - (i128)it.w * it.sy, q) &&
                  o.cs_x < lim && o.cs_y < lim, "%s ct_small q=%llu w=%llu %d %d", name, (unsigned long long)q,
              (unsigned long long)it.w, it.sx, it.sy);
    }
    // inverse butterflies, narrow reductions, add_small
    items.clear();
    const auto is = probes(inv_q * q, q, 60);
    const auto ps = probes(prod_q * q, q, 20);
    for (uint64_t w : ws)
        for (uint64_t x : is)
            for (size_t yi = 0; yi < is.size() && (int)items.size() < MAX_ITEMS; yi += 1 + (size_t)(rnd() % 4)) {
                Item it;
                it.x = x; it.y = is[yi]; it.w = w; it.ws64 = (uint64_t)(((u128)w << 64) / q);
                it.sx = (int32_t)(rnd() % 65) - 32; it.sy = 0;
                items.push_back(it);
            }
    outs.assign(items.size(), Out());
    run(k_eval_inv<A>, items, outs, d_in, d_out, q, aux);
    for (size_t i = 0; i < items.size(); ++i) {
        const Item &it = items[i];
        const Out &o = outs[i];
        const uint64_t d = (it.x % q + q - it.y % q) % q, sm = (it.x % q + it.y % q) % q;
        CHECK(o.gs_x < inv_q * q && o.gs_y < inv_q * q && o.gs_x % q == sm && o.gs_y % q == (uint64_t)(((u128)it.w * d) % q),
              "%s gs q=%llu w=%llu x=%llu y=%llu", name, (unsigned long long)q, (unsigned long long)it.w,
              (unsigned long long)it.x, (unsigned long long)it.y);
        CHECK(o.gl_x < inv_q * q && o.gl_y < inv_q * q && o.gl_x % q == (uint64_t)(((u128)it.w * sm) % q) &&
                  o.gl_y % q == (uint64_t)(((u128)it.w * d) % q), "%s gs_last q=%llu w=%llu x=%llu y=%llu", name,
              (unsigned long long)q, (unsigned long long)it.w, (unsigned long long)it.x, (unsigned long long)it.y);
        CHECK(o.inv == it.x % q, "%s canon_inv %llu", name, (unsigned long long)it.x);
        if (it.y < prod_q * q)
            CHECK(o.addsm % q == mod_of((i128)it.y + it.sx, q) && o.addsm < (prod_q + 1) * q + 33, "%s add_small %llu %d", name,
                  (unsigned long long)it.y, it.sx);
    }
    (void)ps;
    // reductions with their own domains: x -> canon_wide, y -> canon_acc, w -> canon_fwd; canon_lazy on [0, 4q)
    items.clear();
    const auto wv = probes(wide, q, 100000), av = probes(acc, q, 100000), fv = probes(fwdc, q, 100000), lv = probes(4 * q, q, 100000);
    for (size_t i = 0; i < wv.size(); ++i) {
        Item it;
        it.x = wv[i]; it.y = av[i % av.size()]; it.w = fv[i % fv.size()]; it.ws64 = lv[i % lv.size()];
        it.sx = it.sy = 0;
        items.push_back(it);
    }
    outs.assign(items.size(), Out());
    run(k_eval_wide<A>, items, outs, d_in, d_out, q, aux);
    for (size_t i = 0; i < items.size(); ++i) {
        CHECK(outs[i].wide == items[i].x % q, "%s canon_wide %llu -> %llu", name, (unsigned long long)items[i].x, (unsigned long long)outs[i].wide);
        CHECK(outs[i].acc == items[i].y % q, "%s canon_acc %llu", name, (unsigned long long)items[i].y);
        CHECK(outs[i].fwd == items[i].w % q, "%s canon_fwd %llu", name, (unsigned long long)items[i].w);
    }
    // canon_lazy through the inverse kernel's x field
    items.clear();
    for (uint64_t v : lv) {
        Item it;
        it.x = v; it.y = 0; it.w = 1; it.ws64 = (uint64_t)(((u128)1 << 64) / q); it.sx = it.sy = 0;
        items.push_back(it);
    }
    outs.assign(items.size(), Out());
    run(k_eval_inv<A>, items, outs, d_in, d_out, q, aux);
    for (size_t i = 0; i < items.size(); ++i)
        CHECK(outs[i].lazy == items[i].x % q, "%s canon_lazy %llu", name, (unsigned long long)items[i].x);
}

// ---------------------------------------------------------------- residues in doubles
static uint64_t dbits(double v) { uint64_t b; __builtin_memcpy(&b, &v, 8); return b; }
static double bitsd(uint64_t b) { double v; __builtin_memcpy(&v, &b, 8); return v; }

static void check_f(uint64_t q, Item *d_in, Out *d_out)
{
    typedef ArithF A;
    const double qd = (double)q;
    const uint64_t aux = dbits(1.0 / qd);
    auto prod_bound = [&](uint64_t w, double y) { return qd / 2 + 1.5 * (double)w * std::fabs(y) * 0x1p-52 + 1.0; };
    std::vector<Item> items;
    const auto ws = multiplicands(q, 24);
    const auto mags = probes(64 * q + 1, q, 120), xm = probes(63 * q, q, 30);
    for (uint64_t w : ws)
        for (uint64_t ym : mags)
            for (size_t xi = 0; xi < xm.size() && (int)items.size() < MAX_ITEMS; xi += 1 + (size_t)(rnd() % 5)) {
                Item it;
                const double y = (rnd() & 1) ? (double)ym : -(double)ym, x = (rnd() & 1) ? (double)xm[xi] : -(double)xm[xi];
                it.x = dbits(x); it.y = dbits(y); it.w = w; it.ws64 = 0;
                it.sx = (int32_t)(rnd() % 65) - 32; it.sy = (int32_t)(rnd() % 65) - 32;
                items.push_back(it);
            }
    std::vector<Out> outs(items.size());
    run(k_eval<A>, items, outs, d_in, d_out, q, aux);
    for (size_t i = 0; i < items.size(); ++i) {
        const Item &it = items[i];
        const Out &o = outs[i];
        const double x = bitsd(it.x), y = bitsd(it.y), r = bitsd(o.mul);
        const i128 t = (i128)it.w * (i128)(long long)y;
        CHECK(r == std::floor(r) && std::fabs(r) <= prod_bound(it.w, y) && mod_of((i128)(long long)r, q) == mod_of(t, q),
              "ArithF mul q=%llu w=%llu y=%.0f -> %.0f", (unsigned long long)q, (unsigned long long)it.w, y, r);
        const double cx = bitsd(o.ct_x), cy = bitsd(o.ct_y);
        CHECK(std::fabs(cx) <= std::fabs(x) + prod_bound(it.w, y) && std::fabs(cy) <= std::fabs(x) + prod_bound(it.w, y) &&
                  mod_of((i128)(long long)cx, q) == mod_of((i128)(long long)x + t, q) &&
                  mod_of((i128)(long long)cy, q) == mod_of((i128)(long long)x - t, q),
              "ArithF ct q=%llu w=%llu x=%.0f y=%.0f", (unsigned long long)q, (unsigned long long)it.w, x, y);
        CHECK(bitsd(o.cs_x) == (double)(long long)((i128)it.sx + (i128)it.w * it.sy) &&
                  bitsd(o.cs_y) == (double)(long long)((i128)it.sx - (i128)it.w * it.sy), "ArithF ct_small %d %d", it.sx, it.sy);
    }
    // inverse butterflies on reduced values, reduce / canon_wide over the whole domain
    items.clear();
    const auto im = probes(q, q, 60);
    for (uint64_t w : ws)
        for (uint64_t xmag : im)
            for (size_t yi = 0; yi < im.size() && (int)items.size() < MAX_ITEMS; yi += 1 + (size_t)(rnd() % 4)) {
                Item it;
                const double x = (rnd() & 1) ? (double)xmag : -(double)xmag, y = (rnd() & 1) ? (double)im[yi] : -(double)im[yi];
                it.x = dbits(x); it.y = dbits(y); it.w = w; it.ws64 = 0; it.sx = (int32_t)(rnd() % 65) - 32; it.sy = 0;
                items.push_back(it);
            }
    outs.assign(items.size(), Out());
    run(k_eval_inv<A>, items, outs, d_in, d_out, q, aux);
    for (size_t i = 0; i < items.size(); ++i) {
        const Item &it = items[i];
        const Out &o = outs[i];
        const double x = bitsd(it.x), y = bitsd(it.y);
        const i128 d = (i128)(long long)x - (i128)(long long)y;
        CHECK(bitsd(o.gs_x) == x + y && std::fabs(bitsd(o.gs_y)) <= prod_bound(it.w, x - y) &&
                  mod_of((i128)(long long)bitsd(o.gs_y), q) == mod_of((i128)it.w * d, q),
              "ArithF gs q=%llu w=%llu x=%.0f y=%.0f", (unsigned long long)q, (unsigned long long)it.w, x, y);
        CHECK(o.lazy == mod_of((i128)(long long)x, q) && o.inv == o.lazy, "ArithF canon_lazy %.0f", x);
        CHECK(bitsd(o.addsm) == y + (double)it.sx, "ArithF add_small");
    }
    items.clear();
    for (uint64_t m : probes(64 * q + 1, q, 200000)) {
        Item it;
        const double v = (rnd() & 1) ? (double)m : -(double)m;
        it.x = it.y = it.w = dbits(v); it.ws64 = 0; it.sx = it.sy = 0;
        items.push_back(it);
    }
    outs.assign(items.size(), Out());
    run(k_eval_wide<A>, items, outs, d_in, d_out, q, aux);
    for (size_t i = 0; i < items.size(); ++i) {
        const uint64_t want = mod_of((i128)(long long)bitsd(items[i].x), q);
        CHECK(outs[i].wide == want && outs[i].acc == want && outs[i].fwd == want, "ArithF canon_wide q=%llu x=%.0f",
              (unsigned long long)q, bitsd(items[i].x));
    }
}

int main()
{
    Item *d_in;
    Out *d_out;
    HIP_OK(hipMalloc(&d_in, MAX_ITEMS * sizeof(Item)));
    HIP_OK(hipMalloc(&d_out, MAX_ITEMS * sizeof(Out)));
    for (uint64_t q : {(1ull << 55) - 1, 18014398508400641ull, (1ull << 44) + 1, 12289ull})
        check_int<ArithS>("ArithS", q, (uint64_t)(((u128)1 << 63) / q), 1ull << 62, (1ull << 62) - 4 * q, 4, 4, true, 1ull << 62,
                          1ull << 62, 1ull << 62, d_in, d_out);
    std::printf("ArithS ok\n");
    for (uint64_t q : {(1ull << 61) - 1, 1152921504606584833ull, (1ull << 55) + 3, 12289ull})
        check_int<ArithB>("ArithB", q, (uint64_t)(((u128)1 << 63) / q), 1ull << 63, 4 * q, 2, 2, false, 1ull << 63, 6 * q, 4 * q,
                          d_in, d_out);
    std::printf("ArithB ok\n");
    for (uint64_t q : {(1ull << 30) - 1, 1073707009ull, 12289ull, 65537ull, 3ull << 28})
        check_int<Arith32>("Arith32", q, (1ull << 32) / q, 1ull << 32, 4 * q, 2, 2, false, 1ull << 32, 4 * q, 4 * q, d_in, d_out);
    std::printf("Arith32 ok\n");
    for (uint64_t q : {(1ull << 44) - 1, 68719403009ull, 12289ull, 1073707009ull})
        check_f(q, d_in, d_out);
    std::printf("ArithF ok\n");
    HIP_OK(hipFree(d_in));
    HIP_OK(hipFree(d_out));
    if (failures) return 1;
    std::printf("all arithmetic policies hold their contracts on the device\n");
    return 0;
}
