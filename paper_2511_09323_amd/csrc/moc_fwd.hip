// Training forward of the MoC layer, the dense SwiGLU forward, the expert / grouped / keyed forward
// variants and the stand-alone row selections: kernel sequences and their C entry points.
#include "api_common.h"
#include "api_launch.h"
#include "gemm_sparse.h"

using namespace moc;
using namespace mocapi;

namespace {

// ----------------------------------------------------------------------------- forward
template <class E>
moc_status fwd_impl(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, E* y, int32_t* idx, E* gvals,
                    E* uvals, void* ws, hipStream_t st, int ga = 0, int gb = 0, int key_mode = 0) {
    FwdWs<E> W(ws, D, false, key_mode != 0);
    moc_status s;
    // Columns stored by the products that fill [T, ldF] scratch arrays: F rounded up to a whole 4-column group.
    // The up to three extra columns land in the arrays' padding, which nothing reads; without them every
    // row would end in a partly filled group, whose element-wise stores cost about 10 us per product at the 1B shape.
    const int Fs = round_up(D.F, 4);
    // G = X W_gate, kept in fp32 for the selection (Eq. MoC-1)
    // and U = X W_up (Eq. MoC-1): one launch for both when possible
    GemmProblem<E> pg{kc_operand<E>(x, D.d), kc_operand<E>(wg, D.d), D.T, D.F, D.d, 0, false};
    GemmProblem<E> pu{kc_operand<E>(x, D.d), kc_operand<E>(wu, D.d), D.T, D.F, D.d, 0, false};
    if ((s = run_gemm_pair<E>("gemm_gate_up", "gemm_gate", "gemm_up", pg, EpiStore<float>{W.G, D.ldF, Fs, 0}, pu,
                              EpiStore<E>{W.U, D.ldF, Fs, 0}, st, &W.sk)) != MOC_OK)
        return s;
    // M = TopK(G); stored set; Z' = SiLU(G) . M . U (Eq. MoC-2)
    TopkArgs<E> a{W.G, D.ldF, D.F, D.K, idx, nullptr, gvals, W.U, D.ldF, uvals, W.Zd, D.ldF, nullptr};
    if (key_mode != 0) {
        // rank SiLU(G) or |SiLU(G)| instead of G; the stored gate values stay the raw ones
        if ((s = launch_key_transform(W.G, W.keys, (int64_t)D.T * D.ldF, key_mode, st)) != MOC_OK) return s;
        a.g = W.keys;
        a.g_raw = W.G;
    }
    // 256 threads per row keep up to 24 values per thread in registers; longer rows get 512 threads
    // (1024 measured slower)
    if (gb == 0) s = D.ldF > 6144 ? run_topk<E, 512, true>("topk_select_act", a, D.T, st)
                                  : run_topk<E, 256, true>("topk_select_act", a, D.T, st);
    else s = run_group_select<E, true>("group_select_act", a, D.T, ga, gb, st);      // MoC_{a:b}
    if (s != MOC_OK) return s;
    if constexpr (std::is_same<E, bf16_t>::value) {
        // MoC_{a:b} with a <= 2 leaves at most two nonzeros in every aligned group of four channels: on request the
        // down projection takes the compressed Z' and the structured-sparse matrix instruction
        if (gb != 0 && ga <= 2 && W.zc && !options().force_generic && D.d % 8 == 0 && aligned16(wd) && aligned16(y)) {
            {
                Span span("sparse_compress", st);
                const int64_t n = (int64_t)D.T * (D.ldF / 32);
                hipLaunchKernelGGL(sparse_compress_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, W.Zd, (int64_t)D.ldF,
                                   D.T, W.zc, W.zi);
                HIP_TRY(hipGetLastError());
            }
            Span span("gemm_down_sparse", st);
            SparseDownProblem sp{W.zc, W.zi, D.ldF / 2, D.ldF / 32, wd, D.d, D.d, D.T, D.d, D.ldF, D.F};
            hipError_t e = launch_gemm_sparse_down(sp, EpiStore<E>{y, D.d, D.d, 0}, st);
            if (e != hipSuccess) return fail(MOC_ERR_HIP, "gemm_down_sparse launch: %s", hipGetErrorString(e));
            return MOC_OK;
        }
    }
    return down_projection<E>(D, W.Zd, wd, y, st);
}

// ------------------------------------------------------------ MoC inside MoE experts

// Forward for rows already routed and sorted by expert (paper section "Compatibility with MoE
// architectures": every expert's MLP is a MoC network): rows off[e] .. off[e+1]-1 use the weights of
// expert e.  The three projections run as one grouped launch each over the experts; the row Top-K
// is expert-agnostic and runs once over all rows.
template <class E>
moc_status fwd_experts_impl(const Dims& D, int n_exp, const int32_t* off, const E* x, const E* wg, const E* wu, const E* wd,
                            E* y, int32_t* idx, E* gvals, E* uvals, void* ws, hipStream_t st) {
    FwdWs<E> W(ws, D, false);
    const int64_t wsz = (int64_t)D.F * D.d;
    const int Fs = round_up(D.F, 4);      // see fwd_impl
    GemmProblem<E> pr[kMaxExperts];
    EpiStore<float> eg[kMaxExperts];
    EpiStore<E> ee[kMaxExperts];
    moc_status s;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        pr[e] = GemmProblem<E>{kc_operand<E>(x + r0 * D.d, D.d), kc_operand<E>(wg + e * wsz, D.d), off[e + 1] - off[e], D.F, D.d, 0, false};
        eg[e] = EpiStore<float>{W.G + r0 * D.ldF, D.ldF, Fs, 0};
    }
    if ((s = run_gemm_grouped<E, false, false, EpiStore<float>, kMaxExperts>("gemm_gate_experts", n_exp, pr, eg, st)) != MOC_OK) return s;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        pr[e].B = kc_operand<E>(wu + e * wsz, D.d);
        ee[e] = EpiStore<E>{W.U + r0 * D.ldF, D.ldF, Fs, 0};
    }
    if ((s = run_gemm_grouped<E, false, false, EpiStore<E>, kMaxExperts>("gemm_up_experts", n_exp, pr, ee, st)) != MOC_OK) return s;
    TopkArgs<E> a{W.G, D.ldF, D.F, D.K, idx, nullptr, gvals, W.U, D.ldF, uvals, W.Zd, D.ldF, nullptr};
    s = D.ldF > 6144 ? run_topk<E, 512, true>("topk_select_act", a, D.T, st) : run_topk<E, 256, true>("topk_select_act", a, D.T, st);
    if (s != MOC_OK) return s;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        pr[e] = GemmProblem<E>{kc_operand<E>(W.Zd + r0 * D.ldF, D.ldF), km_operand<E>(wd + e * wsz, D.d, D.d), off[e + 1] - off[e], D.d, D.F, 0, true};
        ee[e] = EpiStore<E>{y + r0 * D.d, D.d, D.d, 0};
    }
    return run_gemm_grouped<E, false, true, EpiStore<E>, kMaxExperts>("gemm_down_experts", n_exp, pr, ee, st);
}

// ------------------------------------------------------------------------ dense SwiGLU
template <class E>
moc_status swiglu_fwd_impl(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, E* y, E* g_save,
                           E* u_save, void* ws, hipStream_t st) {
    FwdWs<E> W(ws, D, true);
    moc_status s;
    GemmProblem<E> pg{kc_operand<E>(x, D.d), kc_operand<E>(wg, D.d), D.T, D.F, D.d, 0, false};
    if ((s = run_gemm<E, false, false>("gemm_gate_dense", pg, EpiStore<E>{g_save, D.F, D.F, 0}, st)) != MOC_OK) return s;
    GemmProblem<E> pu{kc_operand<E>(x, D.d), kc_operand<E>(wu, D.d), D.T, D.F, D.d, 0, false};
    if ((s = run_gemm<E, false, false>("gemm_up_act_dense", pu, EpiSwigluAct<E>{g_save, u_save, W.Zd, D.F, D.ldF}, st)) != MOC_OK)
        return s;
    return down_projection<E>(D, W.Zd, wd, y, st);
}

}  // namespace

extern "C" {

moc_status moc_ffn_fwd(const moc_shape* shape, const void* x, const void* wg, const void* wu, const void* wd, void* y,
                       int32_t* idx, void* gvals, void* uvals, void* ws, size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y); CHECK_PTR(idx); CHECK_PTR(gvals); CHECK_PTR(uvals);
    CHECK_WS(MOC_OP_FWD);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return fwd_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd, (bf16_t*)y,
                                idx, (bf16_t*)gvals, (bf16_t*)uvals, ws, st);
    return fwd_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y, idx,
                           (float*)gvals, (float*)uvals, ws, st);
}

moc_status moc_swiglu_fwd(const moc_shape* shape_in, const void* x, const void* wg, const void* wu, const void* wd,
                          void* y, void* g_save, void* u_save, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!shape_in) return fail(MOC_ERR_BAD_ARG, "shape is NULL");
    moc_shape sh = *shape_in;
    sh.K = sh.F;
    const moc_shape* shape = &sh;
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y); CHECK_PTR(g_save); CHECK_PTR(u_save);
    CHECK_WS(MOC_OP_SWIGLU_FWD);
    Dims D(sh);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (sh.dtype == MOC_BF16)
        return swiglu_fwd_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                       (bf16_t*)y, (bf16_t*)g_save, (bf16_t*)u_save, ws, st);
    return swiglu_fwd_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                                  (float*)g_save, (float*)u_save, ws, st);
}

moc_status moc_topk_rows(int32_t T, int32_t F, int32_t K, const float* g, int64_t ldg, int32_t* idx, float* gsel,
                         void* hip_stream) {
    if (T < 1 || F < 1 || K < 1 || K > F) return fail(MOC_ERR_BAD_ARG, "need T >= 1 and 1 <= K <= F (T=%d F=%d K=%d)", T, F, K);
    if (F > 32768) return fail(MOC_ERR_UNSUPPORTED, "F = %d exceeds 32768", F);
    if (ldg < F) return fail(MOC_ERR_BAD_ARG, "ldg < F");
    CHECK_PTR(g); CHECK_PTR(idx); CHECK_PTR(gsel);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    TopkArgs<float> a{g, ldg, F, K, idx, gsel, nullptr, nullptr, 0, nullptr, nullptr, 0};
    return run_topk<float, 256, false>("topk_rows", a, T, st);
}

moc_status moc_ffn_fwd_keyed(const moc_shape* shape, int32_t key_mode, const void* x, const void* wg, const void* wu,
                             const void* wd, void* y, int32_t* idx, void* gvals, void* uvals, void* ws, size_t ws_bytes,
                             void* hip_stream) {
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    if ((s = check_key_mode(key_mode)) != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y); CHECK_PTR(idx); CHECK_PTR(gvals); CHECK_PTR(uvals);
    CHECK_WS(MOC_OP_FWD_KEYED);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return fwd_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd, (bf16_t*)y,
                                idx, (bf16_t*)gvals, (bf16_t*)uvals, ws, st, 0, 0, key_mode);
    return fwd_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y, idx,
                           (float*)gvals, (float*)uvals, ws, st, 0, 0, key_mode);
}

moc_status moc_topk_rows_keyed(int32_t T, int32_t F, int32_t K, int32_t key_mode, const float* g, int64_t ldg,
                               float* key_scratch, int32_t* idx, float* gsel, void* hip_stream) {
    if (T < 1 || F < 1 || K < 1 || K > F) return fail(MOC_ERR_BAD_ARG, "need T >= 1 and 1 <= K <= F (T=%d F=%d K=%d)", T, F, K);
    if (F > 32768) return fail(MOC_ERR_UNSUPPORTED, "F = %d exceeds 32768", F);
    if (ldg < F) return fail(MOC_ERR_BAD_ARG, "ldg < F");
    moc_status s = check_key_mode(key_mode);
    if (s != MOC_OK) return s;
    CHECK_PTR(g); CHECK_PTR(idx); CHECK_PTR(gsel);
    if (key_mode != MOC_KEY_GATE) CHECK_PTR(key_scratch);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    TopkArgs<float> a{g, ldg, F, K, idx, gsel, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr};
    if (key_mode != MOC_KEY_GATE) {
        // the last row is transformed up to F only: nothing past the caller's matrix is read
        if ((s = launch_key_transform(g, key_scratch, (int64_t)(T - 1) * ldg + F, key_mode, st)) != MOC_OK) return s;
        a.g = key_scratch;
        a.g_raw = g;
    }
    return run_topk<float, 256, false>("topk_rows", a, T, st);
}

moc_status moc_ffn_fwd_experts(const moc_shape* shape, int32_t n_experts, const int32_t* expert_offsets, const void* x,
                               const void* wg, const void* wu, const void* wd, void* y, int32_t* idx, void* gvals,
                               void* uvals, void* ws, size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    if ((s = check_offsets(shape, n_experts, expert_offsets)) != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y); CHECK_PTR(idx); CHECK_PTR(gvals); CHECK_PTR(uvals);
    CHECK_WS(MOC_OP_FWD);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return fwd_experts_impl<bf16_t>(D, n_experts, expert_offsets, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu,
                                        (const bf16_t*)wd, (bf16_t*)y, idx, (bf16_t*)gvals, (bf16_t*)uvals, ws, st);
    return fwd_experts_impl<float>(D, n_experts, expert_offsets, (const float*)x, (const float*)wg, (const float*)wu,
                                   (const float*)wd, (float*)y, idx, (float*)gvals, (float*)uvals, ws, st);
}

moc_status moc_ffn_fwd_grouped(const moc_shape* shape, int32_t ga, int32_t gb, const void* x, const void* wg,
                               const void* wu, const void* wd, void* y, int32_t* idx, void* gvals, void* uvals, void* ws,
                               size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    if ((s = check_group(shape->F, shape->K, ga, gb)) != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y); CHECK_PTR(idx); CHECK_PTR(gvals); CHECK_PTR(uvals);
    CHECK_WS(MOC_OP_FWD);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return fwd_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd, (bf16_t*)y,
                                idx, (bf16_t*)gvals, (bf16_t*)uvals, ws, st, ga, gb);
    return fwd_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y, idx,
                           (float*)gvals, (float*)uvals, ws, st, ga, gb);
}

moc_status moc_topk_grouped_rows(int32_t T, int32_t F, int32_t ga, int32_t gb, const float* g, int64_t ldg, int32_t* idx,
                                 float* gsel, void* hip_stream) {
    if (T < 1 || F < 1) return fail(MOC_ERR_BAD_ARG, "need T >= 1 and F >= 1 (T=%d F=%d)", T, F);
    if (gb < 1 || F % gb != 0) return fail(MOC_ERR_BAD_ARG, "b = %d must divide F = %d", gb, F);
    moc_status s = check_group(F, F / gb * ga, ga, gb);
    if (s != MOC_OK) return s;
    if (ldg < F) return fail(MOC_ERR_BAD_ARG, "ldg < F");
    CHECK_PTR(g); CHECK_PTR(idx); CHECK_PTR(gsel);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    TopkArgs<float> a{g, ldg, F, F / gb * ga, idx, gsel, nullptr, nullptr, 0, nullptr, nullptr, 0};
    return run_group_select<float, false>("group_select_rows", a, T, ga, gb, st);
}

}  // extern "C"
