// Training backward of the MoC layer (plain, expert and dense SwiGLU forms): kernel sequences and
// their C entry points.
#include "api_common.h"
#include "api_launch.h"
#include "misc_kernels.h"

using namespace moc;
using namespace mocapi;

namespace {

// ---------------------------------------------------------------------------- backward
template <class E, bool DENSE>
moc_status bwd_impl(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, const int32_t* idx,
                    const E* gvals, const E* uvals, const E* dy, E* dx, E* dwg, E* dwu, E* dwd, void* ws,
                    hipStream_t st) {
    BwdWs<E> W(ws, D, DENSE);
    moc_status s;
    const int Fs = round_up(D.F, 4);      // whole 4-column groups into the padded [T, ldF] array (its padding is never read)
    GemmProblem<E> pz{kc_operand<E>(dy, D.d), kc_operand<E>(wd, D.d), D.T, D.F, D.d, 0, false};
    const size_t expand_lds = (size_t)3 * D.ldF * sizeof(E);
    if (!DENSE && expand_lds <= 160 * 1024 - 64 && !options().bwd_epilogue) {
        // dZ' = dD W_down^T (bp-1) stored densely, then the pointwise step (bp-2, bp-3) on the K stored
        // channels of every token, expanded to the dense-masked rows Z', dG, dU
        if ((s = run_gemm<E, false, false>("gemm_dz", pz, EpiStore<E>{W.dZd, D.ldF, Fs, 0}, st, &W.sk)) != MOC_OK) return s;
        auto kern = bwd_expand_kernel<E>;
        LdsAttr<bwd_expand_kernel<E>, kMaxDynLds>::use();
        Span span("bwd_pointwise_expand", st);
        hipLaunchKernelGGL(kern, dim3(D.T), dim3(256), expand_lds, st, idx, gvals, uvals, W.dZd, D.K, D.F,
                           (int64_t)D.ldF, W.Zd, W.dGd, W.dUd);
        HIP_TRY(hipGetLastError());
    } else {
        if (!DENSE) {
            Span span("build_mask", st);
            hipLaunchKernelGGL(build_mask_kernel, dim3(D.T), dim3(256), (size_t)D.nw * 4 + 16, st, idx, D.K, D.F, D.nw,
                               W.maskw, W.pref);
            HIP_TRY(hipGetLastError());
        }
        // dZ' = dD W_down^T (bp-1) with the pointwise part (bp-2, bp-3) in the epilogue
        EpiBwdPointwise<E, DENSE> epi{W.maskw, W.pref, D.nw, gvals, uvals, DENSE ? D.F : D.K, W.Zd, W.dGd, W.dUd, D.F, D.ldF};
        if ((s = run_gemm<E, false, false>("gemm_dz_pointwise", pz, epi, st)) != MOC_OK) return s;
    }
    // dW_down = Z'^T dD (bp-1); dW_gate = X^T dG, dW_up = X^T dU (bp-4): contractions over tokens,
    // both operands read k-major (token index leading)
    // (one launch for the three of them)
    const GemmProblem<E> pw[3] = {
        {km_operand<E>(W.Zd, D.ldF, D.ldF), km_operand<E>(dy, D.d, D.d), D.F, D.d, D.T, 0, false},
        {km_operand<E>(W.dGd, D.ldF, D.ldF), km_operand<E>(x, D.d, D.d), D.F, D.d, D.T, 0, false},
        {km_operand<E>(W.dUd, D.ldF, D.ldF), km_operand<E>(x, D.d, D.d), D.F, D.d, D.T, 0, false}};
    const EpiStore<E> ew[3] = {{dwd, D.d, D.d, 0}, {dwg, D.d, D.d, 0}, {dwu, D.d, D.d, 0}};
    static const char* const wnames[3] = {"gemm_dwd", "gemm_dwg", "gemm_dwu"};
    if ((s = run_gemm_batch3<E>("gemm_dw3", wnames, pw, ew, st, &W.sk)) != MOC_OK) return s;
    // dX = dG W_gate^T + dU W_up^T (bp-5): one GEMM over the concatenated contraction
    GemmProblem<E> px{kc_operand<E>(W.dGd, D.ldF, W.dUd), km_operand<E>(wg, D.d, D.d, wu), D.T, D.d, D.F, D.F, true};
    return run_gemm<E, false, true>("gemm_dx", px, EpiStore<E>{dx, D.d, D.d, 0}, st);
}

template <class E> __global__ void fill_zero_kernel(E* p, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = E(0);
}

// Backward of fwd_experts_impl: dZ' and dX as grouped launches over the experts, the pointwise step
// once over all rows, and the 3 x n_exp weight-gradient products (each contracting over its expert's
// own rows) as one grouped launch.  An expert without rows gets zero weight gradients.
template <class E>
moc_status bwd_experts_impl(const Dims& D, int n_exp, const int32_t* off, const E* x, const E* wg, const E* wu, const E* wd,
                            const int32_t* idx, const E* gvals, const E* uvals, const E* dy, E* dx, E* dwg, E* dwu, E* dwd,
                            void* ws, hipStream_t st) {
    BwdWs<E> W(ws, D, false);
    const int64_t wsz = (int64_t)D.F * D.d;
    const int Fs = round_up(D.F, 4);      // whole 4-column groups into the padded [T, ldF] array (its padding is never read)
    const size_t expand_lds = (size_t)3 * D.ldF * sizeof(E);
    if (expand_lds > 160 * 1024 - 64) return fail(MOC_ERR_UNSUPPORTED, "F = %d too large for the expert backward", D.F);
    GemmProblem<E> pr[3 * kMaxExperts];
    EpiStore<E> ee[3 * kMaxExperts];
    moc_status s;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        pr[e] = GemmProblem<E>{kc_operand<E>(dy + r0 * D.d, D.d), kc_operand<E>(wd + e * wsz, D.d), off[e + 1] - off[e], D.F, D.d, 0, false};
        ee[e] = EpiStore<E>{W.dZd + r0 * D.ldF, D.ldF, Fs, 0};
    }
    if ((s = run_gemm_grouped<E, false, false, EpiStore<E>, kMaxExperts>("gemm_dz_experts", n_exp, pr, ee, st)) != MOC_OK) return s;
    {
        auto kern = bwd_expand_kernel<E>;
        LdsAttr<bwd_expand_kernel<E>, kMaxDynLds>::use();
        Span span("bwd_pointwise_expand", st);
        hipLaunchKernelGGL(kern, dim3(D.T), dim3(256), expand_lds, st, idx, gvals, uvals, W.dZd, D.K, D.F, (int64_t)D.ldF, W.Zd,
                           W.dGd, W.dUd);
        HIP_TRY(hipGetLastError());
    }
    int np = 0;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        const int rows = off[e + 1] - off[e];
        if (rows == 0) {
            Span span("zero_expert_grads", st);
            for (E* p : {dwd + e * wsz, dwg + e * wsz, dwu + e * wsz})
                hipLaunchKernelGGL((fill_zero_kernel<E>), dim3(1024), dim3(256), 0, st, p, wsz);
            HIP_TRY(hipGetLastError());
            continue;
        }
        const E* ops[3] = {W.Zd, W.dGd, W.dUd};
        const E* rhs[3] = {dy, x, x};
        E* outs[3] = {dwd, dwg, dwu};
        for (int k = 0; k < 3; ++k) {
            pr[np] = GemmProblem<E>{km_operand<E>(ops[k] + r0 * D.ldF, D.ldF, D.ldF), km_operand<E>(rhs[k] + r0 * D.d, D.d, D.d),
                                    D.F, D.d, rows, 0, false};
            ee[np] = EpiStore<E>{outs[k] + e * wsz, D.d, D.d, 0};
            ++np;
        }
    }
    if ((s = run_gemm_grouped<E, true, true, EpiStore<E>, 3 * kMaxExperts>("gemm_dw_experts", np, pr, ee, st)) != MOC_OK) return s;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        pr[e] = GemmProblem<E>{kc_operand<E>(W.dGd + r0 * D.ldF, D.ldF, W.dUd + r0 * D.ldF),
                               km_operand<E>(wg + e * wsz, D.d, D.d, wu + e * wsz), off[e + 1] - off[e], D.d, D.F, D.F, true};
        ee[e] = EpiStore<E>{dx + r0 * D.d, D.d, D.d, 0};
    }
    return run_gemm_grouped<E, false, true, EpiStore<E>, kMaxExperts>("gemm_dx_experts", n_exp, pr, ee, st);
}

}  // namespace

extern "C" {

moc_status moc_ffn_bwd(const moc_shape* shape, const void* x, const void* wg, const void* wu, const void* wd,
                       const int32_t* idx, const void* gvals, const void* uvals, const void* dy, void* dx, void* dwg,
                       void* dwu, void* dwd, void* ws, size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(idx); CHECK_PTR(gvals); CHECK_PTR(uvals);
    CHECK_PTR(dy); CHECK_PTR(dx); CHECK_PTR(dwg); CHECK_PTR(dwu); CHECK_PTR(dwd);
    CHECK_WS(MOC_OP_BWD);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return bwd_impl<bf16_t, false>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd, idx,
                                       (const bf16_t*)gvals, (const bf16_t*)uvals, (const bf16_t*)dy, (bf16_t*)dx,
                                       (bf16_t*)dwg, (bf16_t*)dwu, (bf16_t*)dwd, ws, st);
    return bwd_impl<float, false>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, idx,
                                  (const float*)gvals, (const float*)uvals, (const float*)dy, (float*)dx, (float*)dwg,
                                  (float*)dwu, (float*)dwd, ws, st);
}

moc_status moc_swiglu_bwd(const moc_shape* shape_in, const void* x, const void* wg, const void* wu, const void* wd,
                          const void* g_save, const void* u_save, const void* dy, void* dx, void* dwg, void* dwu,
                          void* dwd, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!shape_in) return fail(MOC_ERR_BAD_ARG, "shape is NULL");
    moc_shape sh = *shape_in;
    sh.K = sh.F;
    const moc_shape* shape = &sh;
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(g_save); CHECK_PTR(u_save);
    CHECK_PTR(dy); CHECK_PTR(dx); CHECK_PTR(dwg); CHECK_PTR(dwu); CHECK_PTR(dwd);
    CHECK_WS(MOC_OP_SWIGLU_BWD);
    Dims D(sh);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (sh.dtype == MOC_BF16)
        return bwd_impl<bf16_t, true>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                      nullptr, (const bf16_t*)g_save, (const bf16_t*)u_save, (const bf16_t*)dy,
                                      (bf16_t*)dx, (bf16_t*)dwg, (bf16_t*)dwu, (bf16_t*)dwd, ws, st);
    return bwd_impl<float, true>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, nullptr,
                                 (const float*)g_save, (const float*)u_save, (const float*)dy, (float*)dx, (float*)dwg,
                                 (float*)dwu, (float*)dwd, ws, st);
}

moc_status moc_ffn_bwd_experts(const moc_shape* shape, int32_t n_experts, const int32_t* expert_offsets, const void* x,
                               const void* wg, const void* wu, const void* wd, const int32_t* idx, const void* gvals,
                               const void* uvals, const void* dy, void* dx, void* dwg, void* dwu, void* dwd, void* ws,
                               size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    if ((s = check_offsets(shape, n_experts, expert_offsets)) != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(idx); CHECK_PTR(gvals); CHECK_PTR(uvals);
    CHECK_PTR(dy); CHECK_PTR(dx); CHECK_PTR(dwg); CHECK_PTR(dwu); CHECK_PTR(dwd);
    CHECK_WS(MOC_OP_BWD);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return bwd_experts_impl<bf16_t>(D, n_experts, expert_offsets, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu,
                                        (const bf16_t*)wd, idx, (const bf16_t*)gvals, (const bf16_t*)uvals, (const bf16_t*)dy,
                                        (bf16_t*)dx, (bf16_t*)dwg, (bf16_t*)dwu, (bf16_t*)dwd, ws, st);
    return bwd_experts_impl<float>(D, n_experts, expert_offsets, (const float*)x, (const float*)wg, (const float*)wu,
                                   (const float*)wd, idx, (const float*)gvals, (const float*)uvals, (const float*)dy, (float*)dx,
                                   (float*)dwg, (float*)dwu, (float*)dwd, ws, st);
}

}  // extern "C"
