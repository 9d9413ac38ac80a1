// Decode path of the MoC layer (row-wide, keyed and grouped selection): kernel sequences and their
// C entry points.
#include "api_common.h"
#include "api_launch.h"
#include <atomic>
#include <random>

#include "decode_kernels.h"
#include "decode_persist.h"
#include "decode_select_gather.h"

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

// ------------------------------------------------------- row-wide decode in one persistent launch
static_assert(sizeof(DecodeSync) <= kDecodeSyncBytes, "workspace reserve for the decode flags");

// Host call counter that makes the flag epochs of different calls differ (decode_persist.h); seeded
// randomly so that flags left in reused memory by another process cannot match either.
std::atomic<uint32_t> g_decode_salt{std::random_device{}()};

constexpr int kPersistentDynLds = 158 * 1024;      // the persistent kernels also hold about 1.2 KB of static LDS

struct DecodePlan {
    bool ok = false;
    int variant = 0;              // 0: row per wavefront, one token; 1: row per wavefront, up to 4; 2: MFMA gate, up to 16
    int nt = 0, nch = 0, bt = 0;
    int nwg = 0, P = 1, C = 1, rmax = 1;
    int off_own = 0, off_over = 0;
    size_t lds = 0;
};

// The single-launch kernel serves the row-wide Top-K on the raw gate when the shape fits its
// assumptions (whole weight rows in registers, the gate row of a token in one workgroup's registers,
// 16-byte column segments); everything else stays on the separate launches.
template <class E>
DecodePlan plan_persistent(const Dims& D, int num_cu) {
    DecodePlan pl;
    constexpr int CN = Chunk<E>::N;
    const int B = D.T, d = D.d, F = D.F;
    const bool bf16 = std::is_same<E, bf16_t>::value;
    if (num_cu < kDecMaxB || options().force_generic || !options().decode_persistent) return pl;   // workgroup b selects for token b
    if (d % CN != 0 || d > 64 * CN * 8) return pl;
    if (B <= 4) {
        pl.variant = B == 1 ? 0 : 1;
        pl.bt = B == 1 ? 1 : 4;
        pl.nt = 1024;
    } else {
        if (!bf16 || d % 1024 != 0) return pl;
        pl.variant = 2;
        pl.bt = 16;
        pl.nt = 768;
    }
    const int nwv = pl.nt / 64;
    const int nch = (F + pl.nt * 4 - 1) / (pl.nt * 4);
    pl.nch = nch <= 3 ? 3 : (nch <= 4 ? 4 : 8);
    if (nch > 8) return pl;
    pl.nwg = std::min(num_cu, kDecMaxWG);
    // x, own gate values, phase-overlaid area
    const size_t xbytes = pl.variant == 2 ? (size_t)16 * (d * 2 + 16) : (size_t)pl.bt * d * sizeof(E);
    size_t own;
    if (pl.variant == 2) {
        const int nblk = (F + 47) / 48;
        pl.rmax = (nblk + pl.nwg - 1) / pl.nwg;
        own = (size_t)pl.rmax * 48 * 17 * sizeof(float);
    } else {
        pl.rmax = (F + pl.nwg * nwv - 1) / (pl.nwg * nwv);
        own = (size_t)nwv * pl.rmax * pl.bt * sizeof(float);
    }
    pl.off_own = (int)round_up_sz(xbytes, 16);
    pl.off_over = (int)round_up_sz(pl.off_own + own, 16);
    const size_t over = std::max(kDecSelLds, pl.variant == 2 ? (size_t)12 * 256 * sizeof(float) : (size_t)0);
    // down projection: C column slices of LPR 16-byte chunks each, P channel ranges
    const int total = (int)((size_t)d * sizeof(E) / 16);
    const int tb = pl.bt > 8 ? 8 : pl.bt;
    int best_lpr = 0;
    size_t best_vol = 0;
    bool best_good = false;
    for (int lpr = 64; lpr >= 1; lpr >>= 1) {
        if (total % lpr != 0) continue;
        const int C = total / lpr;
        if (C > pl.nwg) continue;
        // the last B workgroups write the index lists: they get no share of the down projection if possible
        const int P = std::max(1, std::min(std::max(pl.nwg - B, C) / C, F));
        const int seg = d / C;
        const size_t vol = (size_t)P * B * d * sizeof(float), last = (size_t)P * B * seg * sizeof(float);
        const size_t dl = round_up_sz(((size_t)(F + P - 1) / P + 1) * 8, 16) + (size_t)nwv * tb * seg * sizeof(float);
        if (dl > (size_t)kPersistentDynLds || vol > kDecodePartBudget) continue;
        const bool good = last <= 96 * 1024;
        if (best_lpr == 0 || (good && !best_good) || (good == best_good && !good && vol < best_vol)) {
            if (best_lpr != 0 && best_good) continue;        // keep the first (widest) good split
            best_lpr = lpr; best_vol = vol; best_good = good;
        }
    }
    if (best_lpr == 0) return pl;
    pl.C = total / best_lpr;
    pl.P = std::max(1, std::min(std::max(pl.nwg - B, pl.C) / pl.C, F));
    const size_t dl = round_up_sz(((size_t)(F + pl.P - 1) / pl.P + 1) * 8, 16) + (size_t)nwv * tb * (d / pl.C) * sizeof(float);
    // more than half of a compute unit's LDS, so that the dispatcher places one workgroup per unit
    pl.lds = std::max(std::max((size_t)pl.off_over + over, dl), (size_t)84 * 1024);
    if (pl.lds > (size_t)kPersistentDynLds) return pl;
    pl.ok = true;
    return pl;
}

template <class E, int BT, int NCH>
moc_status launch_persistent_rows(const DecodePlan& pl, const DecArgs<E>& a, hipStream_t st) {
    auto kern = decode_persistent_kernel<E, BT, 1024, NCH>;
    LdsAttr<decode_persistent_kernel<E, BT, 1024, NCH>, kPersistentDynLds>::use();
    Span span("decode_persistent", st);
    hipLaunchKernelGGL(kern, dim3(pl.nwg), dim3(1024), pl.lds, st, a);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

template <int NCH>
moc_status launch_persistent_mfma(const DecodePlan& pl, const DecArgs<bf16_t>& a, hipStream_t st) {
    auto kern = decode_persistent_mfma_kernel<NCH>;
    LdsAttr<decode_persistent_mfma_kernel<NCH>, kPersistentDynLds>::use();
    Span span("decode_persistent", st);
    hipLaunchKernelGGL(kern, dim3(pl.nwg), dim3(768), pl.lds, st, a);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

template <class E>
moc_status decode_persistent(const DecodePlan& pl, const Dims& D, const DecodeWs& W, const E* x, const E* wg, const E* wu,
                             const E* wd, E* y, int32_t* idx, hipStream_t st) {
    DecArgs<E> a;
    a.x = x; a.wg = wg; a.wu = wu; a.wd = wd; a.y = y; a.idx = idx;
    a.B = D.T; a.d = D.d; a.F = D.F; a.K = D.K; a.ldF = D.ldF;
    a.g2 = W.g2; a.zt = W.zt; a.part = W.part2;
    a.sync = static_cast<DecodeSync*>(W.sync);
    a.salt = g_decode_salt.fetch_add(1, std::memory_order_relaxed);
    a.P = pl.P; a.C = pl.C; a.rmax = pl.rmax; a.off_own = pl.off_own; a.off_over = pl.off_over;
    if (pl.variant == 0)
        return pl.nch == 3   ? launch_persistent_rows<E, 1, 3>(pl, a, st)
               : pl.nch == 4 ? launch_persistent_rows<E, 1, 4>(pl, a, st)
                             : launch_persistent_rows<E, 1, 8>(pl, a, st);
    if (pl.variant == 1)
        return pl.nch == 3   ? launch_persistent_rows<E, 4, 3>(pl, a, st)
               : pl.nch == 4 ? launch_persistent_rows<E, 4, 4>(pl, a, st)
                             : launch_persistent_rows<E, 4, 8>(pl, a, st);
    if constexpr (std::is_same<E, bf16_t>::value)
        return pl.nch == 3   ? launch_persistent_mfma<3>(pl, a, st)
               : pl.nch == 4 ? launch_persistent_mfma<4>(pl, a, st)
                             : launch_persistent_mfma<8>(pl, a, st);
    return fail(MOC_ERR_UNSUPPORTED, "decode: no single-launch kernel for this shape");
}

// ga:gb = 0:0 is the row-wide Top-K; otherwise the grouped selection of MoC_{a:b}, which is decided
// inside the gate kernel (a group's channels meet in one workgroup) and needs no selection launch.
// Selection + gather of row-wide decode in one launch (decode_select_gather.h).
constexpr int kSelectGatherMaxLds = 156 * 1024;
template <class E, int NCH>
moc_status launch_select_gather_nch(const Dims& D, const E* x, const E* wu, const E* wd, const float* g, int32_t* idx, float* part,
                                    int P, hipStream_t st) {
    constexpr int NIT = 8;
    auto kern = decode_select_gather_kernel<E, NIT, NCH>;
    LdsAttr<decode_select_gather_kernel<E, NIT, NCH>, kSelectGatherMaxLds>::use();      // (the kernel has 160 bytes of static LDS)
    Span span("decode_select_gather", st);
    hipLaunchKernelGGL(kern, dim3(P * D.T), dim3(512), decode_select_gather_lds<E>(D.d), st, x, wu, wd, g, (int64_t)D.ldF, D.F, D.d,
                       D.K, P, D.T, idx, part);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}
template <class E>
moc_status launch_select_gather(const Dims& D, const E* x, const E* wu, const E* wd, const float* g, int32_t* idx, float* part, int P,
                                hipStream_t st) {
    if (D.F <= 2 * 2048) return launch_select_gather_nch<E, 2>(D, x, wu, wd, g, idx, part, P, st);
    if (D.F <= 6 * 2048) return launch_select_gather_nch<E, 6>(D, x, wu, wd, g, idx, part, P, st);
    return launch_select_gather_nch<E, 16>(D, x, wu, wd, g, idx, part, P, st);
}

template <class E>
moc_status decode_impl(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, E* y, int32_t* idx_out,
                       void* ws, hipStream_t st, int ga = 0, int gb = 0, int key_mode = 0) {
    DecodeWs W(ws, D);
    const int B = D.T;
    int32_t* idx = idx_out ? idx_out : W.idx;
    moc_status s;
    // the gather stage stages one token's x in LDS: refuse a d it cannot hold before anything is launched
    // (the gate stage checks its own staging in its launcher, which is the first launch)
    constexpr int NIT = 8;
    const size_t fused_lds = (size_t)D.d * sizeof(E) + (size_t)8 * D.d * sizeof(float);
    const bool gather_fused = D.d <= 64 * Chunk<E>::N * NIT && fused_lds <= 160 * 1024 - 64;
    if (!gather_fused && (size_t)D.d * sizeof(E) > 64 * 1024) return fail(MOC_ERR_UNSUPPORTED, "decode: d = %d too large", D.d);
    if (gb == 0 && key_mode == 0) {
        // row-wide Top-K on the raw gate: gate, selection, up and down projection in one launch
        const DecodePlan pl = plan_persistent<E>(D, device_cu_count());
        if (pl.ok) return decode_persistent<E>(pl, D, W, x, wg, wu, wd, y, idx, st);
    }
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
    const int P = decode_splits(B, D.K);
    if (gb == 0 && key_mode == 0 && gather_fused && options().decode_select_gather && (D.F + P - 1) / P <= kDsgMaxRange &&
        decode_select_gather_lds<E>(D.d) <= (size_t)kSelectGatherMaxLds) {
        // selection and gather in one launch: every workgroup finds its token's threshold itself
        if ((s = launch_select_gather<E>(D, x, wu, wd, W.g, idx, W.part, P, st)) != MOC_OK) return s;
        Span span("decode_reduce", st);
        const int64_t n = (int64_t)B * D.d;
        hipLaunchKernelGGL((decode_reduce_kernel<E>), dim3((unsigned)((n + 63) / 64)), dim3(1024), 0, st, W.part, P, n, y);
        HIP_TRY(hipGetLastError());
        return MOC_OK;
    }
    if (gb == 0) {
        TopkArgs<float> a{W.g, D.ldF, D.F, D.K, idx, W.gsel, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr};
        if (key_mode != 0) {
            if ((s = launch_key_transform(W.g, W.gkeys, (int64_t)B * D.ldF, key_mode, st)) != MOC_OK) return s;
            a.g = W.gkeys;
            a.g_raw = W.g;
        }
        if ((s = run_topk<float, 1024, false>("decode_topk", a, B, st)) != MOC_OK) return s;
    }
    if (gather_fused) {
        auto kern = B > 1 ? decode_updown_kernel<E, NIT, true> : decode_updown_kernel<E, NIT, false>;
        LdsAttr<decode_updown_kernel<E, NIT, true>, kMaxDynLds>::use();
        LdsAttr<decode_updown_kernel<E, NIT, false>, kMaxDynLds>::use();
        Span span("decode_updown", st);
        hipLaunchKernelGGL(kern, dim3(P * B), dim3(512), fused_lds, st, x, wu, wd, idx, W.gsel, D.d, D.K, P, B, W.part);
        HIP_TRY(hipGetLastError());
    } else {
        {
            const size_t lds = (size_t)D.d * sizeof(E);
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
