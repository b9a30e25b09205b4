// Launchers for one engine shape; included by inst_<log2n>.hip, which instantiates them.
#pragma once
#include "ctx.hpp"

namespace d2 {

template <class ENG>
struct Launch {
    static d2mhe_status ntt(d2mhe_ctx *ctx, uint64_t *polys, uint32_t B, bool forward, hipStream_t st)
    {
        const uint32_t L = ctx->L, polys_n = B * L;
        if constexpr (ENG::LOGB == ENG::LOGN) {
            if (forward)
                hipLaunchKernelGGL(k_ntt_forward<ENG>, dim3(polys_n), dim3(ENG::T), 0, st, polys, ctx->d_tabs, L);
            else
                hipLaunchKernelGGL(k_ntt_inverse<ENG>, dim3(polys_n), dim3(ENG::T), 0, st, polys, ctx->d_tabs, L);
            D2_LAUNCHED(ctx);
        } else {
            // head: top stages across blocks; tail: the block-local stages.  The batch is walked in
            // chunks of whole batches that fit the second grid dimension of the head kernel.
            constexpr int LOGN = ENG::LOGN, LOGH = LOGN - ENG::LOGB;
            const uint32_t chunk_b = ctx->ntt_chunk_polys / L ? ctx->ntt_chunk_polys / L : 1;
            for (uint32_t b0 = 0; b0 < B; b0 += chunk_b) {
                const uint32_t nb = B - b0 < chunk_b ? B - b0 : chunk_b, n = nb * L;
                uint64_t *base = polys + ((size_t)b0 * L << LOGN);
                dim3 hgrid((1u << (LOGN - LOGH)) / 256, n);
                dim3 tgrid(L * (1u << LOGH) * ((nb + TAIL_TILES - 1) / TAIL_TILES));
                if (forward) {
                    hipLaunchKernelGGL((k_head_forward<typename ENG::A, LOGN, LOGH>), hgrid, dim3(256), 0, st, base,
                                       ctx->d_tabs, L, 0u);
                    D2_LAUNCHED(ctx);
                    hipLaunchKernelGGL(k_tail_forward<ENG>, tgrid, dim3(ENG::T), 0, st, base, ctx->d_tabs, L, nb);
                } else {
                    hipLaunchKernelGGL(k_tail_inverse<ENG>, tgrid, dim3(ENG::T), 0, st, base, ctx->d_tabs, L, nb);
                    D2_LAUNCHED(ctx);
                    hipLaunchKernelGGL((k_head_inverse<typename ENG::A, LOGN, LOGH>), hgrid, dim3(256), 0, st, base,
                                       ctx->d_tabs, L, 0u);
                }
                D2_LAUNCHED(ctx);
            }
        }
        return D2MHE_OK;
    }

    static d2mhe_status keygen(d2mhe_ctx *ctx, uint32_t party, uint64_t *sk, uint64_t *pk0, hipStream_t st)
    {
        hipLaunchKernelGGL(k_keygen<ENG>, dim3(ctx->L), dim3(ENG::T), 0, st, party, sk, pk0,
                           (const uint64_t *)ctx->d_p1, ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status encode(d2mhe_ctx *ctx, const float *grad, uint64_t n_values, uint64_t *pt, uint32_t C,
                               hipStream_t st)
    {
        hipLaunchKernelGGL(k_encode<ENG>, dim3(C), dim3(ENG::T), 0, st, grad, n_values, pt, ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status decode(d2mhe_ctx *ctx, const uint64_t *pt, uint32_t C, uint64_t n_values, float *out,
                               hipStream_t st)
    {
        hipLaunchKernelGGL(k_decode<ENG>, dim3(C), dim3(ENG::T), 0, st, pt, n_values, out, ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status encrypt(d2mhe_ctx *ctx, bool from_float, const EncJobs &jobs, uint32_t njobs,
                                uint32_t ct_base, uint64_t n_values, uint32_t C, hipStream_t st)
    {
        if (from_float)
            hipLaunchKernelGGL((k_encrypt<ENG, true>), dim3(C, njobs), dim3(ENG::T), 0, st, jobs, ct_base, n_values,
                               ctx->d_tabs, ctx->rc);
        else
            hipLaunchKernelGGL((k_encrypt<ENG, false>), dim3(C, njobs), dim3(ENG::T), 0, st, jobs, ct_base, n_values,
                               ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status share(d2mhe_ctx *ctx, const ShareJobs &jobs, uint32_t njobs, uint32_t ct_base, uint32_t C,
                              hipStream_t st)
    {
        hipLaunchKernelGGL(k_share<ENG>, dim3(C, njobs), dim3(ENG::T), 0, st, jobs, ct_base, ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status combine(d2mhe_ctx *ctx, const uint64_t *ct, const PtrList &shares, uint32_t K, uint32_t C,
                                uint64_t *pt, hipStream_t st)
    {
        hipLaunchKernelGGL(k_combine<ENG>, dim3(C), dim3(ENG::T), 0, st, ct, shares, K, pt, ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status combine_decode(d2mhe_ctx *ctx, const GroupJobs &jobs, uint32_t njobs, size_t stride,
                                       uint32_t C, uint64_t n_values, hipStream_t st)
    {
        hipLaunchKernelGGL(k_combine_decode<ENG>, dim3(C, njobs), dim3(ENG::T), 0, st, jobs, stride, n_values,
                           ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status receiver_keygen(d2mhe_ctx *ctx, uint32_t party, uint64_t *sk, uint64_t *pk, hipStream_t st)
    {
        hipLaunchKernelGGL(k_receiver_keygen<ENG>, dim3(ctx->L), dim3(ENG::T), 0, st, party, sk, pk, ctx->d_tabs,
                           ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status convert_share(d2mhe_ctx *ctx, const ConvJobs &jobs, uint32_t njobs, uint32_t ct_base,
                                      uint32_t C, hipStream_t st)
    {
        hipLaunchKernelGGL(k_convert_share<ENG>, dim3(C, njobs), dim3(ENG::T), 0, st, jobs, ct_base, ctx->d_tabs,
                           ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status convert_combine(d2mhe_ctx *ctx, const uint64_t *ct, const PtrList &shares, uint32_t K,
                                        const uint64_t *sk, bool keep_c1, uint32_t C, uint64_t *pt, hipStream_t st)
    {
        hipLaunchKernelGGL(k_convert_combine<ENG>, dim3(C), dim3(ENG::T), 0, st, ct, shares, K, sk, keep_c1 ? 1 : 0,
                           pt, ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status convert_combine_decode(d2mhe_ctx *ctx, const RecvJobs &jobs, uint32_t njobs, size_t stride,
                                               uint32_t C, uint64_t n_values, hipStream_t st)
    {
        hipLaunchKernelGGL(k_convert_combine_decode<ENG>, dim3(C, njobs), dim3(ENG::T), 0, st, jobs, stride,
                           n_values, ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status bootstrap_alpha(d2mhe_ctx *ctx, uint32_t group, uint32_t ct_base, uint32_t C, uint64_t *alpha,
                                        hipStream_t st)
    {
        hipLaunchKernelGGL(k_bootstrap_alpha<ENG>, dim3(C, ctx->L), dim3(ENG::T), 0, st, alpha, group, ct_base,
                           ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status bootstrap_share(d2mhe_ctx *ctx, const ConvJobs &jobs, uint32_t njobs, uint32_t ct_base,
                                        uint32_t C, hipStream_t st)
    {
        hipLaunchKernelGGL(k_bootstrap_share<ENG>, dim3(C, njobs), dim3(ENG::T), 0, st, jobs, ct_base, ctx->d_tabs,
                           ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    static d2mhe_status bootstrap_combine(d2mhe_ctx *ctx, const uint64_t *ct, const PtrList &shares, uint32_t K,
                                          const uint64_t *alpha, uint32_t C, uint64_t *ct_out, hipStream_t st)
    {
        hipLaunchKernelGGL(k_bootstrap_combine<ENG>, dim3(C), dim3(ENG::T), 0, st, ct, shares, K, alpha, ct_out,
                           ctx->d_tabs, ctx->rc);
        D2_LAUNCHED(ctx);
        return D2MHE_OK;
    }

    // full set (ring degrees a single workgroup can hold)
    static EngineOps full()
    {
        return EngineOps{ENG::ELOG, ENG::LOGB, &ntt, &keygen, &encode, &decode, &encrypt, &share, &combine,
                         &combine_decode, &receiver_keygen, &convert_share, &convert_combine,
                         &convert_combine_decode, &bootstrap_alpha, &bootstrap_share, &bootstrap_combine};
    }
    // transforms only (longer rings)
    static EngineOps transforms_only()
    {
        return EngineOps{ENG::ELOG, ENG::LOGB, &ntt,    nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                         nullptr,   nullptr,   nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    }
};

}  // namespace d2
