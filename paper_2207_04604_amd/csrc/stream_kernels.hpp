// Element-wise kernels that do not depend on the engine shape (included by one translation unit).
#pragma once
#include "kernels.hpp"

// no fused multiply-add unless written out: float results here are compared bit for bit
#pragma clang fp contract(off)

namespace d2 {

// -------------------------------------------------------------------------------------
// Uniform polynomials in coefficient form: out [B][L][N]; Philox counter
// (n, ct = b, party = 0, domain | limb << 8).
// -------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_uniform(uint64_t *out, const LimbTab *tabs, uint32_t L, uint32_t log2n,
                                                 uint32_t domain, PhiloxKey key, size_t total)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    uint32_t n = (uint32_t)(i & ((1u << log2n) - 1));
    size_t poly = i >> log2n;
    uint32_t limb = (uint32_t)(poly % L), b = (uint32_t)(poly / L);
    Block4 blk = philox4x32_10(n, b, 0, counter_tag(domain, limb, 0), key);
    out[i] = uniform_mod(blk, tabs[limb]);
}

// values [L][N] (canonical) -> prepared polynomial: copy + Shoup quotients.
// K > 0: the values are the sum of K inputs.
__global__ void __launch_bounds__(256) k_prepare(uint64_t *dst, PtrList src, uint32_t K, const LimbTab *tabs,
                                                 uint32_t log2n, size_t total)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    uint64_t q = tabs[i >> log2n].q;
    uint64_t v = 0;
    for (uint32_t k = 0; k < K; ++k) v = add_mod(v, ((const uint64_t *)src.p[k])[i], q);
    dst[i] = v;
    dst[total + i] = shoup_quotient(v, q);
}

// -------------------------------------------------------------------------------------
// dst = sum of K ciphertext buffers (BFV.Add), elementwise over `total` words laid out
// [..][L][N]; K inputs by pointer; ACC: dst is also an input.
// -------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_sum(uint64_t *dst, PtrList src, uint32_t K, const LimbTab *tabs, uint32_t L,
                                             uint32_t log2n, size_t total)
{
    size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 2;
    if (i >= total) return;
    uint64_t q = tabs[(i >> log2n) % L].q;
    ulonglong2 acc = *(const ulonglong2 *)((const uint64_t *)src.p[0] + i);
    for (uint32_t k = 1; k < K; ++k) {
        ulonglong2 v = *(const ulonglong2 *)((const uint64_t *)src.p[k] + i);
        acc.x = add_mod(acc.x, v.x, q);
        acc.y = add_mod(acc.y, v.y, q);
    }
    *(ulonglong2 *)(dst + i) = acc;
}

// MBFV.Convert: dst = (c0 + sum_k h0_k, sum_k h1_k) over [C][2][L][N]; the c1 of ct is dropped.
// LN = L * N words per component.
__global__ void __launch_bounds__(256) k_convert_sum(uint64_t *dst, const uint64_t *ct, PtrList src, uint32_t K,
                                                     const LimbTab *tabs, uint32_t L, uint32_t log2n, size_t LN,
                                                     size_t total)
{
    size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 2;
    if (i >= total) return;
    uint64_t q = tabs[(i >> log2n) % L].q;
    ulonglong2 acc;
    if ((i / LN) & 1) { acc.x = 0; acc.y = 0; }
    else acc = *(const ulonglong2 *)(ct + i);
    for (uint32_t k = 0; k < K; ++k) {
        ulonglong2 v = *(const ulonglong2 *)((const uint64_t *)src.p[k] + i);
        acc.x = add_mod(acc.x, v.x, q);
        acc.y = add_mod(acc.y, v.y, q);
    }
    *(ulonglong2 *)(dst + i) = acc;
}

// Whole round: out[g] = sum of the K_g ciphertext buffers of group g (stride words apart).
// grid = (ceil(words / 512), groups); `words` = C * 2 * L * N per buffer.
// The grid walks groups and words from the last to the first: the kernel that produced the
// ciphertexts wrote them in ascending order, so the ones written last are still in the
// memory-side cache when this kernel starts (measured: 17 % less time on 393 MB of input).
__global__ void __launch_bounds__(256) k_sum_groups(GroupJobs jobs, size_t stride, const LimbTab *tabs, uint32_t L,
                                                    uint32_t log2n, size_t words)
{
    size_t i = ((size_t)(gridDim.x - 1 - blockIdx.x) * 256 + threadIdx.x) * 2;
    if (i >= words) return;
    const uint32_t job = gridDim.y - 1 - blockIdx.y, K = jobs.K[job];
    const uint64_t *src = jobs.first[job];
    uint64_t q = tabs[(i >> log2n) % L].q;
    // streaming loads: every fresh ciphertext is read exactly once here
    typedef unsigned long long v2u64 __attribute__((ext_vector_type(2)));
    const v2u64 first = __builtin_nontemporal_load((const v2u64 *)(src + i));
    ulonglong2 acc;
    acc.x = first.x;
    acc.y = first.y;
    for (uint32_t k = 1; k < K; ++k) {
        const v2u64 v = __builtin_nontemporal_load((const v2u64 *)(src + (size_t)k * stride + i));
        acc.x = add_mod(acc.x, v.x, q);
        acc.y = add_mod(acc.y, v.y, q);
    }
    *(ulonglong2 *)((uint64_t *)jobs.out[job] + i) = acc;
}

// Alg. 2 lines 9-10 on the decoded neighbourhood sum: w = sum * (1/K) - gamma * grad, every
// operation rounded to float32 on its own (no contraction), grad may be null when gamma = 0.
__global__ void __launch_bounds__(256) k_average_update(const float *sum, float inv_k, const float *grad, float gamma,
                                                        uint64_t n, float *w)
{
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float avg = sum[i] * inv_k;
    if (grad) {
        const float step = gamma * grad[i];      // not contracted (see the pragma at the top)
        w[i] = avg - step;
    } else {
        w[i] = avg;
    }
}

}  // namespace d2
