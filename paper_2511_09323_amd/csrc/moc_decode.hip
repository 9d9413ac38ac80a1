// Decode path of the MoC layer (row-wide, keyed and grouped selection): kernel sequences and their
// C entry points.
#include "api_common.h"
#include "api_launch.h"
#include "decode_kernels.h"

using namespace moc;
using namespace mocapi;

namespace {

// ------------------------------------------------------------------------------ decode
template <class E, int BT>
moc_status decode_gate(const Dims& D, const E* x, const E* wg, float* g, hipStream_t st) {
    const size_t lds = (size_t)BT * D.d * sizeof(E);
    if (lds > 160 * 1024 - 64) return fail(MOC_ERR_UNSUPPORTED, "decode: d = %d too large for LDS staging", D.d);
    auto kern = decode_gate_kernel<E, BT>;
    LdsAttr<decode_gate_kernel<E, BT>, kMaxDynLds>::use();
    Span span("decode_gate", st);
    const int per_cu = lds > 80 * 1024 ? 1 : (lds > 40 * 1024 ? 2 : 4);
    const int grid = std::min((D.F + 3) / 4, 256 * per_cu);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, x, wg, D.T, D.d, D.F, g, (int64_t)D.ldF);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

// Gate projection fused with the grouped selection (MoC_{a:b}) on the vector ALU.
template <class E, int BT, int GB>
moc_status decode_gate_group(const Dims& D, const E* x, const E* wg, int ga, int32_t* idx, float* gsel, hipStream_t st) {
    const size_t lds = (size_t)BT * D.d * sizeof(E);
    if (lds > 156 * 1024) return fail(MOC_ERR_UNSUPPORTED, "decode: d = %d too large for LDS staging", D.d);
    auto kern = decode_gate_group_kernel<E, BT, GB>;
    LdsAttr<decode_gate_group_kernel<E, BT, GB>, 156 * 1024>::use();
    Span span("decode_gate_select", st);
    const int per_cu = lds > 76 * 1024 ? 1 : (lds > 36 * 1024 ? 2 : (lds > 16 * 1024 ? 4 : 8));
    const int grid = std::min(D.F / GB, 256 * per_cu);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, x, wg, D.T, D.d, D.F, ga, D.K, idx, gsel);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

template <class E, int BT>
moc_status decode_gate_group_b(const Dims& D, const E* x, const E* wg, int ga, int gb, int32_t* idx, float* gsel,
                               hipStream_t st) {
    if (gb == 4) return decode_gate_group<E, BT, 4>(D, x, wg, ga, idx, gsel, st);
    if (gb == 8) return decode_gate_group<E, BT, 8>(D, x, wg, ga, idx, gsel, st);
    return decode_gate_group<E, BT, 16>(D, x, wg, ga, idx, gsel, st);
}

template <int GB, int RG, int KS, int BTOK, int UN>
moc_status launch_decode_gate_mfma_shape(const Dims& D, const bf16_t* x, const bf16_t* wg, float* g, int ga, int32_t* idx,
                                         float* gsel, hipStream_t st) {
    const size_t lds = decode_gate_mfma_lds(D.d, RG, KS, BTOK);
    auto kern = decode_gate_mfma_kernel<GB, RG, KS, BTOK, UN>;
    LdsAttr<decode_gate_mfma_kernel<GB, RG, KS, BTOK, UN>, kMaxDynLds>::use();
    Span span(GB == 0 ? "decode_gate" : "decode_gate_select", st);
    const int rows = RG * 16;
    hipLaunchKernelGGL(kern, dim3((D.F + rows - 1) / rows), dim3(RG * KS * 64), lds, st, x, wg, D.T, D.d, D.F, g,
                       (int64_t)D.ldF, ga, D.K, idx, gsel);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

// small = true: at most four tokens, d a multiple of 4096 (16 rows per workgroup, eight shares of the
// contraction); otherwise up to 16 tokens, d a multiple of 1024 (48 rows, four shares).
template <int GB>
moc_status launch_decode_gate_mfma(const Dims& D, const bf16_t* x, const bf16_t* wg, float* g, int ga, int32_t* idx,
                                   float* gsel, bool small, hipStream_t st) {
    if (small) return launch_decode_gate_mfma_shape<GB, 1, 8, 4, 8>(D, x, wg, g, ga, idx, gsel, st);
    return launch_decode_gate_mfma_shape<GB, 3, 4, 16, 4>(D, x, wg, g, ga, idx, gsel, st);
}

template <class E, int BT, int GA>
moc_status launch_decode_fused_t(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, int32_t* idx,
                                 float* part, int P, hipStream_t st) {
    const size_t lds = (size_t)BT * D.d * sizeof(E);
    auto kern = decode_fused_group_kernel<E, BT, GA>;
    LdsAttr<decode_fused_group_kernel<E, BT, GA>, 64 * 1024>::use();
    Span span("decode_fused_gate_select_gather", st);
    hipLaunchKernelGGL(kern, dim3(P), dim3(512), lds, st, x, wg, wu, wd, D.T, D.d, D.F, D.K, idx, part);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

template <class E>
moc_status launch_decode_fused(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, int ga, int32_t* idx,
                               float* part, int P, hipStream_t st) {
    if (ga == 1) return launch_decode_fused_t<E, 1, 1>(D, x, wg, wu, wd, idx, part, P, st);
    return launch_decode_fused_t<E, 1, 2>(D, x, wg, wu, wd, idx, part, P, st);
}

// ga:gb = 0:0 is the row-wide Top-K; otherwise the grouped selection of MoC_{a:b}, which is decided
// inside the gate kernel (a group's channels meet in one workgroup) and needs no selection launch.
template <class E>
moc_status decode_impl(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, E* y, int32_t* idx_out,
                       void* ws, hipStream_t st, int ga = 0, int gb = 0, int key_mode = 0) {
    DecodeWs W(ws, D);
    const int B = D.T;
    int32_t* idx = idx_out ? idx_out : W.idx;
    moc_status s;
    // MOC_DECODE_FUSED=0 keeps grouped decode on the separate gate+select and gather launches;
    // MOC_DECODE_FUSED_P=n sets the workgroup count of the single-launch kernel.
    if (gb == 8 && (ga == 1 || ga == 2) && B == 1 && D.d <= 8 * 64 * Chunk<E>::N && options().decode_fused &&
        !options().force_generic) {
        // MoC_{a:8}, one token: gate, selection and gather in one launch, then the deterministic
        // reduction.  Two workgroups are resident per CU; the groups are dealt out evenly.
        const int ngroups = D.F / 8;
        const int rounds = (ngroups + kDecodeFusedMaxP - 1) / kDecodeFusedMaxP;
        const int want = options().decode_fused_p > 0 ? options().decode_fused_p : (ngroups + rounds - 1) / rounds;
        const int P = std::min(ngroups, std::max(1, std::min(kDecodeFusedMaxP, want)));
        if ((s = launch_decode_fused<E>(D, x, wg, wu, wd, ga, idx, W.part, P, st)) != MOC_OK) return s;
        Span span("decode_reduce", st);
        const int64_t n = (int64_t)B * D.d;
        hipLaunchKernelGGL((decode_reduce_kernel<E>), dim3((unsigned)((n + 63) / 64)), dim3(1024), 0, st, W.part, P, n, y);
        HIP_TRY(hipGetLastError());
        return MOC_OK;
    }
    const bool bf16_mfma = std::is_same<E, bf16_t>::value && !options().force_generic;
    // two to four tokens: the MFMA kernel's strided row reads stream slower than the row-per-wavefront
    // GEMV (26.7 against 24.8 us at the 7B shape), but with the selection fused in it beats the
    // workgroup-per-group GEMV (28.3 against 30.8 us), so it serves the grouped variant only
    const bool mfma_small = bf16_mfma && gb != 0 && B >= 2 && B <= 4 && D.d % 4096 == 0 &&
                            decode_gate_mfma_lds(D.d, 1, 8, 4) <= 64 * 1024;
    const bool mfma_large = bf16_mfma && B > 4 && D.d % 1024 == 0 && decode_gate_mfma_lds(D.d, 3, 4, 16) <= 160 * 1024 - 64;
    if (mfma_small || mfma_large) {
        const bf16_t* xb = reinterpret_cast<const bf16_t*>(x);
        const bf16_t* wb = reinterpret_cast<const bf16_t*>(wg);
        if (gb == 0) s = launch_decode_gate_mfma<0>(D, xb, wb, W.g, 0, idx, W.gsel, mfma_small, st);
        else if (gb == 4) s = launch_decode_gate_mfma<4>(D, xb, wb, W.g, ga, idx, W.gsel, mfma_small, st);
        else if (gb == 8) s = launch_decode_gate_mfma<8>(D, xb, wb, W.g, ga, idx, W.gsel, mfma_small, st);
        else s = launch_decode_gate_mfma<16>(D, xb, wb, W.g, ga, idx, W.gsel, mfma_small, st);
    } else if (gb == 0) {
        if (B == 1) s = decode_gate<E, 1>(D, x, wg, W.g, st);
        else if (B <= 4) s = decode_gate<E, 4>(D, x, wg, W.g, st);
        else s = decode_gate<E, 16>(D, x, wg, W.g, st);
    } else {
        if (B == 1) s = decode_gate_group_b<E, 1>(D, x, wg, ga, gb, idx, W.gsel, st);
        else if (B <= 4) s = decode_gate_group_b<E, 4>(D, x, wg, ga, gb, idx, W.gsel, st);
        else s = decode_gate_group_b<E, 16>(D, x, wg, ga, gb, idx, W.gsel, st);
    }
    if (s != MOC_OK) return s;
    if (gb == 0) {
        TopkArgs<float> a{W.g, D.ldF, D.F, D.K, idx, W.gsel, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr};
        if (key_mode != 0) {
            if ((s = launch_key_transform(W.g, W.gkeys, (int64_t)B * D.ldF, key_mode, st)) != MOC_OK) return s;
            a.g = W.gkeys;
            a.g_raw = W.g;
        }
        if ((s = run_topk<float, 1024, false>("decode_topk", a, B, st)) != MOC_OK) return s;
    }
    const int P = decode_splits(B, D.K);
    constexpr int NIT = 8;
    const size_t fused_lds = (size_t)D.d * sizeof(E) + (size_t)8 * D.d * sizeof(float);
    if (D.d <= 64 * Chunk<E>::N * NIT && fused_lds <= 160 * 1024 - 64) {
        auto kern = B > 1 ? decode_updown_kernel<E, NIT, true> : decode_updown_kernel<E, NIT, false>;
        LdsAttr<decode_updown_kernel<E, NIT, true>, kMaxDynLds>::use();
        LdsAttr<decode_updown_kernel<E, NIT, false>, kMaxDynLds>::use();
        Span span("decode_updown", st);
        hipLaunchKernelGGL(kern, dim3(P * B), dim3(512), fused_lds, st, x, wu, wd, idx, W.gsel, D.d, D.K, P, B, W.part);
        HIP_TRY(hipGetLastError());
    } else {
        {
            const size_t lds = (size_t)D.d * sizeof(E);
            if (lds > 64 * 1024) return fail(MOC_ERR_UNSUPPORTED, "decode: d = %d too large", D.d);
            Span span("decode_up", st);
            const int gx = std::max(1, std::min((D.K + 3) / 4, 1024 / B));
            hipLaunchKernelGGL((decode_up_kernel<E>), dim3(gx, B), dim3(256), lds, st, x, wu, idx, W.gsel, D.d, D.K, W.z);
            HIP_TRY(hipGetLastError());
        }
        Span span("decode_down", st);
        constexpr int SLICE = 64 * Chunk<E>::N * 4;
        hipLaunchKernelGGL((decode_down_kernel<E, 4>), dim3(P, B, (D.d + SLICE - 1) / SLICE), dim3(256), 0, st, wd, idx,
                           W.z, D.d, D.K, P, W.part);
        HIP_TRY(hipGetLastError());
    }
    {
        Span span("decode_reduce", st);
        const int64_t n = (int64_t)B * D.d;
        hipLaunchKernelGGL((decode_reduce_kernel<E>), dim3((unsigned)((n + 63) / 64)), dim3(1024), 0, st, W.part, P, n,
                           y);
        HIP_TRY(hipGetLastError());
    }
    return MOC_OK;
}

}  // namespace

extern "C" {

moc_status moc_ffn_decode(const moc_shape* shape, const void* x, const void* wg, const void* wu, const void* wd,
                          void* y, int32_t* idx_or_null, void* ws, size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, true);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y);
    if (idx_or_null && !aligned16(idx_or_null)) return fail(MOC_ERR_BAD_ARG, "idx is not 16-byte aligned");
    CHECK_WS(MOC_OP_DECODE);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return decode_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                   (bf16_t*)y, idx_or_null, ws, st);
    return decode_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                              idx_or_null, ws, st);
}

moc_status moc_ffn_decode_static(const moc_shape* shape, const void* x, const void* wg, const void* wu, const void* wd,
                                 void* y, int32_t* idx_or_null, void* hip_stream) {
    moc_status s = check_shape(shape, true);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y);
    if (idx_or_null && !aligned16(idx_or_null)) return fail(MOC_ERR_BAD_ARG, "idx is not 16-byte aligned");
    const size_t need = moc_workspace_bytes(shape, MOC_OP_DECODE);
    if (need > kStaticScratchBytes)
        return fail(MOC_ERR_UNSUPPORTED, "decode scratch for this shape is %zu bytes, the static buffer holds %zu", need,
                    kStaticScratchBytes);
    void* ws = nullptr;                     // this device's copy of the static scratch array
    if ((s = ensure_init(&ws)) != MOC_OK) return s;
    Dims D(*shape);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return decode_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                   (bf16_t*)y, idx_or_null, ws, st);
    return decode_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                              idx_or_null, ws, st);
}

moc_status moc_ffn_decode_keyed(const moc_shape* shape, int32_t key_mode, const void* x, const void* wg, const void* wu,
                                const void* wd, void* y, int32_t* idx_or_null, void* ws, size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, true);
    if (s != MOC_OK) return s;
    if ((s = check_key_mode(key_mode)) != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y);
    if (idx_or_null && !aligned16(idx_or_null)) return fail(MOC_ERR_BAD_ARG, "idx is not 16-byte aligned");
    CHECK_WS(MOC_OP_DECODE);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return decode_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                   (bf16_t*)y, idx_or_null, ws, st, 0, 0, key_mode);
    return decode_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                              idx_or_null, ws, st, 0, 0, key_mode);
}

moc_status moc_ffn_decode_grouped(const moc_shape* shape, int32_t ga, int32_t gb, const void* x, const void* wg,
                                  const void* wu, const void* wd, void* y, int32_t* idx_or_null, void* ws,
                                  size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, true);
    if (s != MOC_OK) return s;
    if ((s = check_group(shape->F, shape->K, ga, gb)) != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y);
    if (idx_or_null && !aligned16(idx_or_null)) return fail(MOC_ERR_BAD_ARG, "idx is not 16-byte aligned");
    CHECK_WS(MOC_OP_DECODE);
    Dims D(*shape);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return decode_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                   (bf16_t*)y, idx_or_null, ws, st, ga, gb);
    return decode_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                              idx_or_null, ws, st, ga, gb);
}

}  // extern "C"
