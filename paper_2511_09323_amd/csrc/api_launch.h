// Launch helpers shared by the entry-point files: GEMM dispatch (tile choice, MFMA or generic
// kernel, batched / paired / grouped launches), the row Top-K and grouped-selection launchers.
#pragma once
#include <algorithm>
#include <type_traits>

#include "api_common.h"
#include "epilogue.h"
#include "gemm_generic.h"
#include "gemm_mfma.h"
#include "group_select.h"
#include "kernel_attrs.h"
#include "topk.h"

namespace mocapi {
using namespace moc;

// ------------------------------------------------------------------------ GEMM dispatch
// Workgroups of a persistent GEMM launch: one per compute unit (the kernels' LDS use allows no more),
// or 0 (one workgroup per tile) with MOC_GEMM_PERSISTENT=0.
inline int persistent_workgroups() { return options().gemm_persistent ? device_cu_count() : 0; }

template <int BM, int BN, bool AKM, bool BKM, class Epi>
hipError_t launch_mfma_tail(const MfmaProblem& pr, const Epi& epi, hipStream_t st) {
    const bool tail = pr.Kc % kMfmaBK != 0 || pr.Kc2 % kMfmaBK != 0;
    // Four wavefronts, three k-slices in flight from global memory.  Measured over the whole training step:
    // three slices beat two by 1.3 %, four give nothing more; eight wavefronts (2 x 4) are faster in
    // isolation at short contractions but 2.5 % slower over the step.
    if (!tail) return launch_gemm_bf16_mfma<BM, BN, AKM, BKM, 0, Epi, 4, 3>(pr, epi, st, persistent_workgroups());
    if constexpr (AKM != BKM) {
        const GemmOperand<bf16_t>& kc = AKM ? pr.B : pr.A;
        const int kmax = std::max(pr.Kc, pr.Kc2);
        if (pr.kc_zero_padded && kc.ld >= round_up(kmax, kMfmaBK))
            return launch_gemm_bf16_mfma<BM, BN, AKM, BKM, 2, Epi, 4, 3>(pr, epi, st, persistent_workgroups());
    }
    return launch_gemm_bf16_mfma<BM, BN, AKM, BKM, 1, Epi, 4, 3>(pr, epi, st, persistent_workgroups());
}

// Runs C = A B^T (+ second segment) with the epilogue `epi`.  AKM / BKM state the operand layouts
// at compile time (they must match pr.A.km / pr.B.km).  bf16 problems that satisfy the MFMA
// kernel's assumptions go to the matrix cores, everything else to the generic kernel.
inline StreamKArgs streamk_args(const StreamKArea& a, int nk) {
    return StreamKArgs{a.part, a.flag, next_streamk_tag(), std::max(1, nk / 8), std::max(0, options().gemm_streamk_spin)};
}
inline int streamk_workgroups() { return std::min(persistent_workgroups(), kStreamKSlots) / 8 * 8; }

// `sk`, if given and carved, lets a product whose whole tiles would leave part of the chip idle in their last
// round split its work along the contraction instead (256 x 256 tiles, contraction a multiple of 32).
template <class E, bool AKM, bool BKM, class Epi>
moc_status run_gemm(const char* name, const GemmProblem<E>& pr, const Epi& epi, hipStream_t st, const StreamKArea* sk = nullptr) {
    Span span(name, st);
    if constexpr (std::is_same<E, bf16_t>::value) {
        if (!options().force_generic && mfma_problem_ok(pr)) {
            if (sk && sk->part && options().gemm_streamk && options().tile == 0 && pr.Kc % kMfmaBK == 0 && pr.Kc2 % kMfmaBK == 0) {
                const int64_t tiles = (int64_t)((pr.M + 255) / 256) * ((pr.N + 255) / 256);
                const int nk = (pr.Kc + pr.Kc2) / kMfmaBK, wgs = streamk_workgroups();
                if (streamk_pays(tiles, nk, wgs)) {
                    hipError_t e = launch_gemm_bf16_mfma_streamk<256, 256, AKM, BKM, 0, Epi, 4, 3>(pr, epi, streamk_args(*sk, nk), wgs, st);
                    if (e != hipSuccess) return fail(MOC_ERR_HIP, "%s launch: %s", name, hipGetErrorString(e));
                    return MOC_OK;
                }
            }
            // tile shape: fewest rounds of workgroups over the 256 CUs, weighted by tile area and the
            // measured efficiency of the smaller shapes (they stage more LDS bytes per FLOP)
            struct Cand { int bm, bn; double penalty; };
            static const Cand cands[3] = {{256, 256, 1.0}, {256, 192, 1.15}, {128, 128, 1.6}};
            int best = 0;
            double best_cost = 0.0;
            for (int c = 0; c < 3; ++c) {
                const int64_t tiles = (int64_t)((pr.M + cands[c].bm - 1) / cands[c].bm) * ((pr.N + cands[c].bn - 1) / cands[c].bn);
                const double cost = (double)((tiles + 255) / 256) * cands[c].bm * cands[c].bn * cands[c].penalty;
                if (c == 0 || cost < best_cost) { best = c; best_cost = cost; }
            }
            if (options().tile == 256) best = 0;
            if (options().tile == 192) best = 1;
            if (options().tile == 128) best = 2;
            hipError_t e = best == 0   ? launch_mfma_tail<256, 256, AKM, BKM, Epi>(pr, epi, st)
                           : best == 1 ? launch_mfma_tail<256, 192, AKM, BKM, Epi>(pr, epi, st)
                                       : launch_mfma_tail<128, 128, AKM, BKM, Epi>(pr, epi, st);
            if (e != hipSuccess) return fail(MOC_ERR_HIP, "%s launch: %s", name, hipGetErrorString(e));
            return MOC_OK;
        }
    }
    launch_gemm_generic<E, Epi>(pr, epi, st);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

// Three independent products of one shape (both operands k-major, plain stores) in one launch when
// the MFMA kernel takes them; otherwise one run_gemm each.  Same tile choice as run_gemm, over the
// tiles of all three.
template <class E>
moc_status run_gemm_batch3(const char* name, const char* const names[3], const GemmProblem<E> pr[3], const EpiStore<E> epi[3],
                           hipStream_t st, const StreamKArea* sk = nullptr) {
    if constexpr (std::is_same<E, bf16_t>::value) {
        const bool same = pr[0].M == pr[1].M && pr[0].M == pr[2].M && pr[0].N == pr[1].N && pr[0].N == pr[2].N &&
                          pr[0].Kc == pr[1].Kc && pr[0].Kc == pr[2].Kc && pr[0].Kc % kMfmaBK == 0 && pr[0].Kc2 == 0 &&
                          pr[1].Kc2 == 0 && pr[2].Kc2 == 0;
        if (same && !options().force_generic && mfma_problem_ok(pr[0]) && mfma_problem_ok(pr[1]) && mfma_problem_ok(pr[2])) {
            struct Cand { int bm, bn; double penalty; };
            static const Cand cands[3] = {{256, 256, 1.0}, {256, 192, 1.15}, {128, 128, 1.6}};
            int best = 0;
            double best_cost = 0.0;
            for (int c = 0; c < 3; ++c) {
                const int64_t tiles = 3 * (int64_t)((pr[0].M + cands[c].bm - 1) / cands[c].bm) * ((pr[0].N + cands[c].bn - 1) / cands[c].bn);
                const double cost = (double)((tiles + 255) / 256) * cands[c].bm * cands[c].bn * cands[c].penalty;
                if (c == 0 || cost < best_cost) { best = c; best_cost = cost; }
            }
            if (options().tile == 256) best = 0;
            if (options().tile == 192) best = 1;
            if (options().tile == 128) best = 2;
            MfmaBatch<EpiStore<E>, 3> b;
            for (int i = 0; i < 3; ++i) { b.pr[i] = pr[i]; b.epi[i] = epi[i]; }
            Span span(name, st);
            if (sk && sk->part && options().gemm_streamk && options().tile == 0) {
                const int64_t tiles = 3 * (int64_t)((pr[0].M + 255) / 256) * ((pr[0].N + 255) / 256);
                const int nk = pr[0].Kc / kMfmaBK, wgs = streamk_workgroups();
                if (streamk_pays(tiles, nk, wgs)) {
                    hipError_t e = launch_gemm_bf16_mfma_batch_streamk<256, 256, true, true, 0, EpiStore<E>, 3, 4, 3>(b, streamk_args(*sk, nk), wgs, st);
                    if (e != hipSuccess) return fail(MOC_ERR_HIP, "%s launch: %s", name, hipGetErrorString(e));
                    return MOC_OK;
                }
            }
            hipError_t e = best == 0   ? launch_gemm_bf16_mfma_batch<256, 256, true, true, 0, EpiStore<E>, 3, 4, 3>(b, st, persistent_workgroups())
                           : best == 1 ? launch_gemm_bf16_mfma_batch<256, 192, true, true, 0, EpiStore<E>, 3, 4, 3>(b, st, persistent_workgroups())
                                       : launch_gemm_bf16_mfma_batch<128, 128, true, true, 0, EpiStore<E>, 3, 4, 3>(b, st, persistent_workgroups());
            if (e != hipSuccess) return fail(MOC_ERR_HIP, "%s launch: %s", name, hipGetErrorString(e));
            return MOC_OK;
        }
    }
    for (int i = 0; i < 3; ++i) {
        moc_status s = run_gemm<E, true, true>(names[i], pr[i], epi[i], st, sk);
        if (s != MOC_OK) return s;
    }
    return MOC_OK;
}

// Two independent products of one shape (both operands k-contiguous, contraction a multiple of 32)
// with different epilogues in one launch when the MFMA kernel takes them; otherwise one run_gemm each.
template <class E, class EpiA, class EpiB>
moc_status run_gemm_pair(const char* name, const char* name_a, const char* name_b, const GemmProblem<E>& pa, const EpiA& ea,
                         const GemmProblem<E>& pb, const EpiB& eb, hipStream_t st, const StreamKArea* sk = nullptr) {
    if constexpr (std::is_same<E, bf16_t>::value) {
        const bool same = pa.M == pb.M && pa.N == pb.N && pa.Kc == pb.Kc && pa.Kc % kMfmaBK == 0 && pa.Kc2 == 0 && pb.Kc2 == 0;
        if (same && !options().force_generic && mfma_problem_ok(pa) && mfma_problem_ok(pb)) {
            struct Cand { int bm, bn; double penalty; };
            static const Cand cands[3] = {{256, 256, 1.0}, {256, 192, 1.15}, {128, 128, 1.6}};
            int best = 0;
            double best_cost = 0.0, best_single = 0.0;
            for (int c = 0; c < 3; ++c) {
                const int64_t tiles = (int64_t)((pa.M + cands[c].bm - 1) / cands[c].bm) * ((pa.N + cands[c].bn - 1) / cands[c].bn);
                const double unit = (double)cands[c].bm * cands[c].bn * cands[c].penalty;
                const double cost = (double)((2 * tiles + 255) / 256) * unit;
                const double single = (double)((tiles + 255) / 256) * unit;
                if (c == 0 || cost < best_cost) { best = c; best_cost = cost; }
                if (c == 0 || single < best_single) best_single = single;
            }
            if (options().tile == 256) best = 0;
            if (options().tile == 192) best = 1;
            if (options().tile == 128) best = 2;
            // worth one launch only when the two together need fewer rounds of workgroups than apart
            if (!(best_cost < 2.0 * best_single)) {
                moc_status s = run_gemm<E, false, false>(name_a, pa, ea, st, sk);
                if (s != MOC_OK) return s;
                return run_gemm<E, false, false>(name_b, pb, eb, st, sk);
            }
            Span span(name, st);
            hipError_t e = best == 0   ? launch_gemm_bf16_mfma_pair<256, 256, false, false, 0, EpiA, EpiB, 4, 3>(pa, ea, pb, eb, st)
                           : best == 1 ? launch_gemm_bf16_mfma_pair<256, 192, false, false, 0, EpiA, EpiB, 4, 3>(pa, ea, pb, eb, st)
                                       : launch_gemm_bf16_mfma_pair<128, 128, false, false, 0, EpiA, EpiB, 4, 3>(pa, ea, pb, eb, st);
            if (e != hipSuccess) return fail(MOC_ERR_HIP, "%s launch: %s", name, hipGetErrorString(e));
            return MOC_OK;
        }
    }
    moc_status s = run_gemm<E, false, false>(name_a, pa, ea, st, sk);
    if (s != MOC_OK) return s;
    return run_gemm<E, false, false>(name_b, pb, eb, st, sk);
}

// Up to NB products that differ only in their row counts (and, for weight gradients, in their
// contraction lengths) in one launch: one per expert of an MoE layer.  Problems with M = 0 are
// skipped.  Falls back to one run_gemm per problem when the MFMA kernel cannot take all of them.
template <class E, bool AKM, bool BKM, class Epi, int NB>
moc_status run_gemm_grouped(const char* name, int nprob, const GemmProblem<E>* pr, const Epi* epi, hipStream_t st) {
    if constexpr (std::is_same<E, bf16_t>::value) {
        bool ok = !options().force_generic && nprob <= NB;
        bool tail = false, padded = true;
        int64_t total_m = 0;
        for (int z = 0; z < nprob && ok; ++z) {
            if (pr[z].M == 0) continue;
            ok = mfma_problem_ok(pr[z]) && pr[z].N == pr[0].N && (pr[z].Kc2 == 0) == (pr[0].Kc2 == 0);
            tail = tail || pr[z].Kc % kMfmaBK != 0 || pr[z].Kc2 % kMfmaBK != 0;
            const GemmOperand<bf16_t>& kc = AKM ? pr[z].B : pr[z].A;
            padded = padded && pr[z].kc_zero_padded && kc.ld >= round_up(std::max(pr[z].Kc, pr[z].Kc2), kMfmaBK);
            total_m += pr[z].M;
        }
        if (ok && total_m > 0) {
            struct Cand { int bm, bn; double penalty; };
            static const Cand cands[3] = {{256, 256, 1.0}, {256, 192, 1.15}, {128, 128, 1.6}};
            int best = 0;
            double best_cost = 0.0;
            for (int c = 0; c < 3; ++c) {
                int64_t tiles = 0;
                for (int z = 0; z < nprob; ++z)
                    tiles += (int64_t)((pr[z].M + cands[c].bm - 1) / cands[c].bm) * ((pr[0].N + cands[c].bn - 1) / cands[c].bn);
                const double cost = (double)((tiles + 255) / 256) * cands[c].bm * cands[c].bn * cands[c].penalty;
                if (c == 0 || cost < best_cost) { best = c; best_cost = cost; }
            }
            if (options().tile == 256) best = 0;
            if (options().tile == 192) best = 1;
            if (options().tile == 128) best = 2;
            MfmaGroup<Epi, NB> g;
            for (int z = 0; z < nprob; ++z) { g.pr[z] = pr[z]; g.epi[z] = epi[z]; }
            const int mode = !tail ? 0 : ((AKM != BKM && padded) ? 2 : 1);
            Span span(name, st);
            hipError_t e = hipSuccess;
#define MOC_GROUP_LAUNCH(BM_, BN_)                                                                                          \
    (mode == 0   ? launch_gemm_bf16_mfma_group<BM_, BN_, AKM, BKM, 0, Epi, NB, 4, 3>(g, nprob, st)                            \
     : mode == 2 ? launch_gemm_bf16_mfma_group<BM_, BN_, AKM, BKM, (AKM != BKM ? 2 : 1), Epi, NB, 4, 3>(g, nprob, st)        \
                 : launch_gemm_bf16_mfma_group<BM_, BN_, AKM, BKM, 1, Epi, NB, 4, 3>(g, nprob, st))
            e = best == 0 ? MOC_GROUP_LAUNCH(256, 256) : best == 1 ? MOC_GROUP_LAUNCH(256, 192) : MOC_GROUP_LAUNCH(128, 128);
#undef MOC_GROUP_LAUNCH
            if (e != hipSuccess) return fail(MOC_ERR_HIP, "%s launch: %s", name, hipGetErrorString(e));
            return MOC_OK;
        }
    }
    for (int z = 0; z < nprob; ++z) {
        if (pr[z].M == 0) continue;
        moc_status s = run_gemm<E, AKM, BKM>(name, pr[z], epi[z], st);
        if (s != MOC_OK) return s;
    }
    return MOC_OK;
}

// LDS-resident Top-K: any row length up to the LDS capacity, any alignment.
template <class E, int NT, int VEC, bool FUSED>
moc_status run_topk_lds(const char* name, const TopkArgs<E>& a, int T, hipStream_t st) {
    const size_t lds = topk_lds_bytes(a.F, NT, VEC);
    if (lds > 160 * 1024 - 64) return fail(MOC_ERR_UNSUPPORTED, "F = %d needs %zu bytes of LDS for Top-K", a.F, lds);
    auto kern = topk_rows_lds_kernel<E, NT, VEC, FUSED>;
    LdsAttr<topk_rows_lds_kernel<E, NT, VEC, FUSED>, kMaxDynLds>::use();
    Span span(name, st);
    hipLaunchKernelGGL(kern, dim3(T), dim3(NT), lds, st, a);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

constexpr size_t kTopkRegDynMax = 96 * 1024;     // slot lists + dense row of the register-resident kernel

template <class E, int NT, int NCH, bool FUSED>
moc_status launch_topk_reg(const char* name, const TopkArgs<E>& a, int T, hipStream_t st) {
    const size_t dyn = topk_reg_dyn_lds(a.K, FUSED ? a.ldz : 0, sizeof(E), FUSED);
    auto kern = topk_rows_kernel<E, NT, NCH, FUSED>;
    LdsAttr<topk_rows_kernel<E, NT, NCH, FUSED>, (int)kTopkRegDynMax>::use();
    Span span(name, st);
    hipLaunchKernelGGL(kern, dim3(T), dim3(NT), dyn, st, a);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

// Row Top-K with NT threads per row.  Rows that are 16-byte aligned and short enough stay in
// registers; everything else goes through the LDS-resident kernel.
template <class E, int NT, bool FUSED>
moc_status run_topk(const char* name, const TopkArgs<E>& a, int T, hipStream_t st) {
    const bool aligned = a.ldg % 4 == 0 && aligned16(a.g);
    const int cover = FUSED ? (int)std::max<int64_t>(a.F, a.ldz) : a.F;
    const int nch = (cover + NT * 4 - 1) / (NT * 4);
    // very large K (slot lists beyond the LDS budget of the register kernel) goes to the LDS-resident kernel
    const bool lists_fit = topk_reg_dyn_lds(a.K, FUSED ? a.ldz : 0, sizeof(E), FUSED) <= kTopkRegDynMax;
    if (aligned && lists_fit) {
        if (nch <= 1) return launch_topk_reg<E, NT, 1, FUSED>(name, a, T, st);
        if (nch <= 2) return launch_topk_reg<E, NT, 2, FUSED>(name, a, T, st);
        if (nch <= 3) return launch_topk_reg<E, NT, 3, FUSED>(name, a, T, st);
        if (NT == 256 || NT == 512) {
            if (nch <= 4) return launch_topk_reg<E, NT, 4, FUSED>(name, a, T, st);
            if (nch <= 6) return launch_topk_reg<E, NT, 6, FUSED>(name, a, T, st);
            if (nch <= 8) return launch_topk_reg<E, NT, 8, FUSED>(name, a, T, st);
            if (NT == 256 && nch <= 11) return launch_topk_reg<E, NT, 11, FUSED>(name, a, T, st);
        }
        return run_topk_lds<E, NT, 4, FUSED>(name, a, T, st);
    }
    if (aligned) return run_topk_lds<E, NT, 4, FUSED>(name, a, T, st);
    if (FUSED) return fail(MOC_ERR_BAD_ARG, "%s: unaligned workspace", name);
    return run_topk_lds<E, NT, 1, FUSED>(name, a, T, st);
}

// Grouped Top-K of MoC_{a:b}: one thread per group of gb channels.
template <class E, bool FUSED>
moc_status run_group_select(const char* name, const TopkArgs<E>& a, int T, int ga, int gb, hipStream_t st) {
    const int vec_ok = a.ldg % 4 == 0 && aligned16(a.g);
    if (FUSED && (!vec_ok || a.ldz % 64 != 0 || a.ldu % 64 != 0)) return fail(MOC_ERR_BAD_ARG, "%s: unaligned workspace", name);
    const int64_t groups = (int64_t)T * ((FUSED ? a.ldz : (int64_t)a.F) / gb);
    const unsigned grid = (unsigned)((groups + 255) / 256);
    Span span(name, st);
    if (gb == 4) hipLaunchKernelGGL((group_select_kernel<E, 4, FUSED>), dim3(grid), dim3(256), 0, st, a, T, ga, vec_ok);
    else if (gb == 8) hipLaunchKernelGGL((group_select_kernel<E, 8, FUSED>), dim3(grid), dim3(256), 0, st, a, T, ga, vec_ok);
    else hipLaunchKernelGGL((group_select_kernel<E, 16, FUSED>), dim3(grid), dim3(256), 0, st, a, T, ga, vec_ok);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

// keys = SiLU(g) or |SiLU(g)| over n contiguous fp32 values (Top-K position variants)
inline moc_status launch_key_transform(const float* g, float* keys, int64_t n, int key_mode, hipStream_t st) {
    Span span("topk_key_transform", st);
    const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + 255) / 256, 16384));
    hipLaunchKernelGGL(topk_key_transform_kernel, dim3(grid), dim3(256), 0, st, g, keys, n, key_mode);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

// D = Z' W_down (Eq. MoC-2 / FFN-2): Z' is [T, ldF] with zeros past F, W_down [F, d] is read k-major.
template <class E>
moc_status down_projection(const Dims& D, const E* Zd, const E* wd, E* y, hipStream_t st) {
    GemmProblem<E> pr{kc_operand<E>(Zd, D.ldF), km_operand<E>(wd, D.d, D.d), D.T, D.d, D.F, 0, true};
    return run_gemm<E, false, true>("gemm_down", pr, EpiStore<E>{y, D.d, D.d, 0}, st);
}

}  // namespace mocapi
