// Internal declarations shared by the API translation unit and the per-ring-degree
// kernel instantiations.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/d2mhe.h"
#include "kernels.hpp"

struct d2mhe_ctx {
    uint32_t log2n, L;
    size_t N;
    uint64_t q[d2::MAX_LIMBS];
    uint64_t psi[d2::MAX_LIMBS + 1];
    uint64_t t;
    uint32_t max_group;
    int arith;          // 0: ArithF, 1: ArithS, 2: ArithB, 3: Arith32
    d2::RoundConst rc;
    const d2::LimbTab *d_tabs;
    uint64_t *d_p1;     // prepared common random polynomial [2][L][N]
    uint32_t ntt_chunk_polys;   // polynomials per head/tail launch pair for N > 2^14 (0: all at once)
    int last_hip;
};

namespace d2 {

inline d2mhe_status hip_fail(d2mhe_ctx *ctx, hipError_t e)
{
    if (ctx) ctx->last_hip = (int)e;
    return D2MHE_ERR_HIP;
}

#define D2_HIP(ctx, call)                                        \
    do {                                                         \
        hipError_t e_ = (call);                                  \
        if (e_ != hipSuccess) return d2::hip_fail((ctx), e_);    \
    } while (0)

#define D2_LAUNCHED(ctx) D2_HIP((ctx), hipGetLastError())

// Kernel launchers of one ring degree (one engine shape); defined in inst_<log2n>.hip.
struct EngineOps {
    int elog, logb;
    d2mhe_status (*ntt)(d2mhe_ctx *, uint64_t *polys, uint32_t B, bool forward, hipStream_t);
    d2mhe_status (*keygen)(d2mhe_ctx *, uint32_t party, uint64_t *sk, uint64_t *pk0, hipStream_t);
    d2mhe_status (*encode)(d2mhe_ctx *, const float *grad, uint64_t n_values, uint64_t *pt, uint32_t C, hipStream_t);
    d2mhe_status (*decode)(d2mhe_ctx *, const uint64_t *pt, uint32_t C, uint64_t n_values, float *out, hipStream_t);
    // from_float: jobs.src holds gradients (encoded on the fly), otherwise plaintext polynomials
    d2mhe_status (*encrypt)(d2mhe_ctx *, bool from_float, const EncJobs &jobs, uint32_t njobs, uint32_t ct_base,
                            uint64_t n_values, uint32_t C, hipStream_t);
    d2mhe_status (*share)(d2mhe_ctx *, const ShareJobs &jobs, uint32_t njobs, uint32_t ct_base, uint32_t C,
                          hipStream_t);
    d2mhe_status (*combine)(d2mhe_ctx *, const uint64_t *ct, const PtrList &shares, uint32_t K, uint32_t C,
                            uint64_t *pt, hipStream_t);
    d2mhe_status (*combine_decode)(d2mhe_ctx *, const GroupJobs &jobs, uint32_t njobs, size_t stride, uint32_t C,
                                   uint64_t n_values, hipStream_t);
    // MBFV.Convert
    d2mhe_status (*receiver_keygen)(d2mhe_ctx *, uint32_t party, uint64_t *sk, uint64_t *pk, hipStream_t);
    d2mhe_status (*convert_share)(d2mhe_ctx *, const ConvJobs &jobs, uint32_t njobs, uint32_t ct_base, uint32_t C,
                                  hipStream_t);
    // y = c0 + sum h0_k + (c1 if keep_c1 + sum h1_k) sk, rounded: plaintext polynomials
    d2mhe_status (*convert_combine)(d2mhe_ctx *, const uint64_t *ct, const PtrList &shares, uint32_t K,
                                    const uint64_t *sk, bool keep_c1, uint32_t C, uint64_t *pt, hipStream_t);
    d2mhe_status (*convert_combine_decode)(d2mhe_ctx *, const RecvJobs &jobs, uint32_t njobs, size_t stride,
                                           uint32_t C, uint64_t n_values, hipStream_t);
    // MBFV.Bootstrap
    d2mhe_status (*bootstrap_alpha)(d2mhe_ctx *, uint32_t group, uint32_t ct_base, uint32_t C, uint64_t *alpha,
                                    hipStream_t);
    d2mhe_status (*bootstrap_share)(d2mhe_ctx *, const ConvJobs &jobs, uint32_t njobs, uint32_t ct_base, uint32_t C,
                                    hipStream_t);
    d2mhe_status (*bootstrap_combine)(d2mhe_ctx *, const uint64_t *ct, const PtrList &shares, uint32_t K,
                                      const uint64_t *alpha, uint32_t C, uint64_t *ct_out, hipStream_t);
};

const EngineOps *ops_f_10();
const EngineOps *ops_f_11();
const EngineOps *ops_f_12();
const EngineOps *ops_f_13();
const EngineOps *ops_f_14();
const EngineOps *ops_f_15();
const EngineOps *ops_f_16();
const EngineOps *ops_s_10();
const EngineOps *ops_s_11();
const EngineOps *ops_s_12();
const EngineOps *ops_s_13();
const EngineOps *ops_s_14();
const EngineOps *ops_s_15();
const EngineOps *ops_s_16();
const EngineOps *ops_b_10();
const EngineOps *ops_b_11();
const EngineOps *ops_b_12();
const EngineOps *ops_b_13();
const EngineOps *ops_b_14();
const EngineOps *ops_b_15();
const EngineOps *ops_b_16();
const EngineOps *ops_w_10();
const EngineOps *ops_w_11();
const EngineOps *ops_w_12();
const EngineOps *ops_w_13();
const EngineOps *ops_w_14();
const EngineOps *ops_w_15();
const EngineOps *ops_w_16();

}  // namespace d2
