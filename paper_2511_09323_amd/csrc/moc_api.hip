// C ABI of the MoC FFN library (see include/moc.h): argument checks, workspace carving and the
// kernel sequence of every entry point.  No device memory is allocated here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <type_traits>
#include <vector>

#include "../../include/moc.h"
#include "common.h"
#include "decode_kernels.h"
#include "group_select.h"
#include "epilogue.h"
#include "gemm_generic.h"
#include "gemm_mfma.h"
#include "misc_kernels.h"
#include "topk.h"

using namespace moc;

namespace {

// ------------------------------------------------------------------------------- errors
thread_local char g_err[512] = "";

moc_status fail(moc_status s, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return s;
}

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail(MOC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// ---------------------------------------------------------------------- per-kernel timing
struct TimingEntry {
    std::string name;
    double ms = 0.0;
    int64_t launches = 0;
};
struct PendingSpan {
    int entry;
    hipEvent_t start, stop;
};
bool g_timing_on = false;
std::vector<TimingEntry> g_entries;
std::vector<PendingSpan> g_pending;
std::vector<hipEvent_t> g_event_pool;

hipEvent_t take_event() {
    if (!g_event_pool.empty()) {
        hipEvent_t e = g_event_pool.back();
        g_event_pool.pop_back();
        return e;
    }
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

int entry_index(const char* name) {
    for (size_t i = 0; i < g_entries.size(); ++i)
        if (g_entries[i].name == name) return (int)i;
    g_entries.push_back(TimingEntry{name, 0.0, 0});
    return (int)g_entries.size() - 1;
}

// Brackets the launches made during its lifetime with two events on the stream.
struct Span {
    hipStream_t st;
    hipEvent_t start = nullptr, stop = nullptr;
    int entry = -1;
    Span(const char* name, hipStream_t s) : st(s) {
        if (!g_timing_on) return;
        start = take_event();
        stop = take_event();
        if (!start || !stop) return;
        entry = entry_index(name);
        hipEventRecord(start, st);
    }
    ~Span() {
        if (entry < 0) return;
        hipEventRecord(stop, st);
        g_pending.push_back(PendingSpan{entry, start, stop});
    }
};

// ------------------------------------------------------------------------ small helpers
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

struct Carver {   // hands out 256-byte aligned pieces of the workspace
    unsigned char* base;
    size_t off = 0;
    explicit Carver(void* p) : base(static_cast<unsigned char*>(p)) {}
    template <class T> T* take(size_t count) {
        T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += round_up_sz(count * sizeof(T), 256);
        return r;
    }
};

int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    return v ? atoi(v) : dflt;
}

struct Options {
    int force_generic;   // MOC_FORCE_GENERIC=1: never use the MFMA GEMM
    int tile;            // MOC_GEMM_TILE=256|192|128 forces a tile shape, 0 = choose by problem size
    Options() : force_generic(env_int("MOC_FORCE_GENERIC", 0)), tile(env_int("MOC_GEMM_TILE", 0)) {}
};
const Options& options() {
    static Options o;
    return o;
}

moc_status check_shape(const moc_shape* s, bool decode) {
    if (!s) return fail(MOC_ERR_BAD_ARG, "shape is NULL");
    if (s->dtype != MOC_F32 && s->dtype != MOC_BF16) return fail(MOC_ERR_BAD_ARG, "unknown dtype %d", s->dtype);
    if (s->T < 1 || s->d < 1 || s->F < 1) return fail(MOC_ERR_BAD_ARG, "T, d, F must be >= 1 (got %d, %d, %d)", s->T, s->d, s->F);
    if (s->K < 1 || s->K > s->F) return fail(MOC_ERR_BAD_ARG, "K must satisfy 1 <= K <= F (got K=%d, F=%d)", s->K, s->F);
    if (s->F > 32768) return fail(MOC_ERR_UNSUPPORTED, "F = %d exceeds 32768", s->F);
    if (s->dtype == MOC_BF16 && s->d % 8 != 0) return fail(MOC_ERR_BAD_ARG, "bf16 needs d %% 8 == 0 (got %d)", s->d);
    if (s->dtype == MOC_F32 && s->d % 4 != 0 && decode) return fail(MOC_ERR_BAD_ARG, "fp32 decode needs d %% 4 == 0 (got %d)", s->d);
    if ((int64_t)s->T * s->F >= (1ll << 40)) return fail(MOC_ERR_UNSUPPORTED, "T*F too large");
    if (decode && s->T > 16) return fail(MOC_ERR_BAD_ARG, "decode batch must be <= 16 (got %d)", s->T);
    return MOC_OK;
}

#define CHECK_PTR(p)                                                                   \
    do {                                                                               \
        if ((p) == nullptr) return fail(MOC_ERR_BAD_ARG, "%s is NULL", #p);            \
        if (!aligned16(p)) return fail(MOC_ERR_BAD_ARG, "%s is not 16-byte aligned", #p); \
    } while (0)

// ------------------------------------------------------------------------ GEMM dispatch
template <int BM, int BN, bool AKM, bool BKM, class Epi>
hipError_t launch_mfma_tail(const MfmaProblem& pr, const Epi& epi, hipStream_t st) {
    const bool tail = pr.Kc % kMfmaBK != 0 || pr.Kc2 % kMfmaBK != 0;
    // Four wavefronts, three k-slices in flight from global memory.  Measured over the whole training step:
    // three slices beat two by 1.3 %, four give nothing more; eight wavefronts (2 x 4) are faster in
    // isolation at short contractions but 2.5 % slower over the step.
    if (!tail) return launch_gemm_bf16_mfma<BM, BN, AKM, BKM, 0, Epi, 4, 3>(pr, epi, st);
    if constexpr (AKM != BKM) {
        const GemmOperand<bf16_t>& kc = AKM ? pr.B : pr.A;
        const int kmax = std::max(pr.Kc, pr.Kc2);
        if (pr.kc_zero_padded && kc.ld >= round_up(kmax, kMfmaBK))
            return launch_gemm_bf16_mfma<BM, BN, AKM, BKM, 2, Epi, 4, 3>(pr, epi, st);
    }
    return launch_gemm_bf16_mfma<BM, BN, AKM, BKM, 1, Epi, 4, 3>(pr, epi, st);
}

// Runs C = A B^T (+ second segment) with the epilogue `epi`.  AKM / BKM state the operand layouts
// at compile time (they must match pr.A.km / pr.B.km).  bf16 problems that satisfy the MFMA
// kernel's assumptions go to the matrix cores, everything else to the generic kernel.
template <class E, bool AKM, bool BKM, class Epi>
moc_status run_gemm(const char* name, const GemmProblem<E>& pr, const Epi& epi, hipStream_t st) {
    Span span(name, st);
    if constexpr (std::is_same<E, bf16_t>::value) {
        if (!options().force_generic && mfma_problem_ok(pr)) {
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
                           hipStream_t st) {
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
            hipError_t e = best == 0   ? launch_gemm_bf16_mfma_batch<256, 256, true, true, 0, EpiStore<E>, 3, 4, 3>(b, st)
                           : best == 1 ? launch_gemm_bf16_mfma_batch<256, 192, true, true, 0, EpiStore<E>, 3, 4, 3>(b, st)
                                       : launch_gemm_bf16_mfma_batch<128, 128, true, true, 0, EpiStore<E>, 3, 4, 3>(b, st);
            if (e != hipSuccess) return fail(MOC_ERR_HIP, "%s launch: %s", name, hipGetErrorString(e));
            return MOC_OK;
        }
    }
    for (int i = 0; i < 3; ++i) {
        moc_status s = run_gemm<E, true, true>(names[i], pr[i], epi[i], st);
        if (s != MOC_OK) return s;
    }
    return MOC_OK;
}

// Two independent products of one shape (both operands k-contiguous, contraction a multiple of 32)
// with different epilogues in one launch when the MFMA kernel takes them; otherwise one run_gemm each.
template <class E, class EpiA, class EpiB>
moc_status run_gemm_pair(const char* name, const char* name_a, const char* name_b, const GemmProblem<E>& pa, const EpiA& ea,
                         const GemmProblem<E>& pb, const EpiB& eb, hipStream_t st) {
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
                moc_status s = run_gemm<E, false, false>(name_a, pa, ea, st);
                if (s != MOC_OK) return s;
                return run_gemm<E, false, false>(name_b, pb, eb, st);
            }
            Span span(name, st);
            hipError_t e = best == 0   ? launch_gemm_bf16_mfma_pair<256, 256, false, false, 0, EpiA, EpiB, 4, 3>(pa, ea, pb, eb, st)
                           : best == 1 ? launch_gemm_bf16_mfma_pair<256, 192, false, false, 0, EpiA, EpiB, 4, 3>(pa, ea, pb, eb, st)
                                       : launch_gemm_bf16_mfma_pair<128, 128, false, false, 0, EpiA, EpiB, 4, 3>(pa, ea, pb, eb, st);
            if (e != hipSuccess) return fail(MOC_ERR_HIP, "%s launch: %s", name, hipGetErrorString(e));
            return MOC_OK;
        }
    }
    moc_status s = run_gemm<E, false, false>(name_a, pa, ea, st);
    if (s != MOC_OK) return s;
    return run_gemm<E, false, false>(name_b, pb, eb, st);
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
    static size_t attr_bytes = 0;
    if (lds > attr_bytes) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024 - 64));
        attr_bytes = 160 * 1024 - 64;
    }
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
    static bool attr = false;
    if (!attr) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)kTopkRegDynMax));
        attr = true;
    }
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
moc_status check_group(int F, int K, int ga, int gb) {
    if (gb != 4 && gb != 8 && gb != 16) return fail(MOC_ERR_BAD_ARG, "group size b must be 4, 8 or 16 (got %d)", gb);
    if (ga < 1 || ga > gb) return fail(MOC_ERR_BAD_ARG, "a must satisfy 1 <= a <= b (got a=%d, b=%d)", ga, gb);
    if (F % gb != 0) return fail(MOC_ERR_BAD_ARG, "b = %d must divide F = %d", gb, F);
    if (K != F / gb * ga) return fail(MOC_ERR_BAD_ARG, "K = %d must equal a*F/b = %d", K, F / gb * ga);
    return MOC_OK;
}

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

// ------------------------------------------------------------------- workspace layouts
struct Dims {
    int T, d, F, K;
    int ldF, nw;
    explicit Dims(const moc_shape& s) : T(s.T), d(s.d), F(s.F), K(s.K) {
        ldF = round_up(F, 64);
        nw = ldF / 32;
    }
};

template <class E> struct FwdWs {      // dense scratch of the forward: fp32 gate, U, masked Z'
    float *G, *keys;                   // keys: transformed selection keys (Top-K position variants only)
    E *U, *Zd;
    size_t bytes;
    FwdWs(void* ws, const Dims& D, bool dense, bool keyed = false) {
        Carver c(ws);
        G = dense ? nullptr : c.take<float>((size_t)D.T * D.ldF);
        U = dense ? nullptr : c.take<E>((size_t)D.T * D.ldF);
        Zd = c.take<E>((size_t)D.T * D.ldF);
        keys = keyed ? c.take<float>((size_t)D.T * D.ldF) : nullptr;
        bytes = c.off;
    }
};

// keys = SiLU(g) or |SiLU(g)| over n contiguous fp32 values (Top-K position variants)
moc_status launch_key_transform(const float* g, float* keys, int64_t n, int key_mode, hipStream_t st) {
    Span span("topk_key_transform", st);
    const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + 255) / 256, 16384));
    hipLaunchKernelGGL(topk_key_transform_kernel, dim3(grid), dim3(256), 0, st, g, keys, n, key_mode);
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

template <class E> struct BwdWs {      // dense [T, ldF] operands (+ the bit mask of the fallback path)
    uint32_t* maskw;
    uint16_t* pref;
    E *dZd, *Zd, *dGd, *dUd;
    size_t bytes;
    BwdWs(void* ws, const Dims& D, bool dense) {
        Carver c(ws);
        maskw = dense ? nullptr : c.take<uint32_t>((size_t)D.T * D.nw);
        pref = dense ? nullptr : c.take<uint16_t>((size_t)D.T * D.nw);
        dZd = dense ? nullptr : c.take<E>((size_t)D.T * D.ldF);
        Zd = c.take<E>((size_t)D.T * D.ldF);
        dGd = c.take<E>((size_t)D.T * D.ldF);
        dUd = c.take<E>((size_t)D.T * D.ldF);
        bytes = c.off;
    }
};

// Channel shares per token in the gather stage: shares x tokens fills the 256 CUs once (one
// 512-thread workgroup per CU), and a multiple of 8 shares lets the kernel keep each share on one XCD.
int decode_splits(int B, int K) {
    const int by_batch = std::max(8, 256 / B / 8 * 8);
    const int by_k = (K + 7) / 8;
    return std::max(1, std::min(by_batch, by_k));
}

constexpr int kDecodeFusedMaxP = 512;

struct DecodeWs {
    float *g, *gkeys, *gsel, *z, *part;
    int32_t* idx;
    size_t bytes;
    DecodeWs(void* ws, const Dims& D) {
        Carver c(ws);
        g = c.take<float>((size_t)D.T * D.ldF);
        gkeys = c.take<float>((size_t)D.T * D.ldF);
        gsel = c.take<float>((size_t)D.T * D.K);
        z = c.take<float>((size_t)D.T * D.K);
        idx = c.take<int32_t>((size_t)D.T * D.K);
        // partial outputs: one per channel share, or one per workgroup of the single-launch grouped kernel
        const int shares = std::max(decode_splits(D.T, D.K), D.T == 1 ? kDecodeFusedMaxP : 0);
        part = c.take<float>((size_t)shares * D.T * D.d);
        bytes = c.off;
    }
};

template <class E> size_t workspace_for(const Dims& D, int op) {
    switch (op) {
        case MOC_OP_FWD: return FwdWs<E>(nullptr, D, false).bytes;
        case MOC_OP_BWD: return BwdWs<E>(nullptr, D, false).bytes;
        case MOC_OP_DECODE: return DecodeWs(nullptr, D).bytes;
        case MOC_OP_SWIGLU_FWD: return FwdWs<E>(nullptr, D, true).bytes;
        case MOC_OP_SWIGLU_BWD: return BwdWs<E>(nullptr, D, true).bytes;
        case MOC_OP_FWD_KEYED: return FwdWs<E>(nullptr, D, false, true).bytes;
    }
    return 0;
}

// D = Z' W_down (Eq. MoC-2 / FFN-2): Z' is [T, ldF] with zeros past F, W_down [F, d] is read k-major.
template <class E>
moc_status down_projection(const Dims& D, const E* Zd, const E* wd, E* y, hipStream_t st) {
    GemmProblem<E> pr{kc_operand<E>(Zd, D.ldF), km_operand<E>(wd, D.d, D.d), D.T, D.d, D.F, 0, true};
    return run_gemm<E, false, true>("gemm_down", pr, EpiStore<E>{y, D.d, D.d, 0}, st);
}

// ----------------------------------------------------------------------------- forward
template <class E>
moc_status fwd_impl(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, E* y, int32_t* idx, E* gvals,
                    E* uvals, void* ws, hipStream_t st, int ga = 0, int gb = 0, int key_mode = 0) {
    FwdWs<E> W(ws, D, false, key_mode != 0);
    moc_status s;
    // G = X W_gate, kept in fp32 for the selection (Eq. MoC-1)
    // and U = X W_up (Eq. MoC-1): one launch for both when possible
    GemmProblem<E> pg{kc_operand<E>(x, D.d), kc_operand<E>(wg, D.d), D.T, D.F, D.d, 0, false};
    GemmProblem<E> pu{kc_operand<E>(x, D.d), kc_operand<E>(wu, D.d), D.T, D.F, D.d, 0, false};
    if ((s = run_gemm_pair<E>("gemm_gate_up", "gemm_gate", "gemm_up", pg, EpiStore<float>{W.G, D.ldF, D.F, 0}, pu,
                              EpiStore<E>{W.U, D.ldF, D.F, 0}, st)) != MOC_OK)
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
    return down_projection<E>(D, W.Zd, wd, y, st);
}

// ---------------------------------------------------------------------------- backward
template <class E, bool DENSE>
moc_status bwd_impl(const Dims& D, const E* x, const E* wg, const E* wu, const E* wd, const int32_t* idx,
                    const E* gvals, const E* uvals, const E* dy, E* dx, E* dwg, E* dwu, E* dwd, void* ws,
                    hipStream_t st) {
    BwdWs<E> W(ws, D, DENSE);
    moc_status s;
    GemmProblem<E> pz{kc_operand<E>(dy, D.d), kc_operand<E>(wd, D.d), D.T, D.F, D.d, 0, false};
    const size_t expand_lds = (size_t)3 * D.ldF * sizeof(E);
    if (!DENSE && expand_lds <= 160 * 1024 - 64) {
        // dZ' = dD W_down^T (bp-1) stored densely, then the pointwise step (bp-2, bp-3) on the K stored
        // channels of every token, expanded to the dense-masked rows Z', dG, dU
        if ((s = run_gemm<E, false, false>("gemm_dz", pz, EpiStore<E>{W.dZd, D.ldF, D.F, 0}, st)) != MOC_OK) return s;
        auto kern = bwd_expand_kernel<E>;
        static bool attr = false;
        if (!attr) {
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        160 * 1024 - 64));
            attr = true;
        }
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
    if ((s = run_gemm_batch3<E>("gemm_dw3", wnames, pw, ew, st)) != MOC_OK) return s;
    // dX = dG W_gate^T + dU W_up^T (bp-5): one GEMM over the concatenated contraction
    GemmProblem<E> px{kc_operand<E>(W.dGd, D.ldF, W.dUd), km_operand<E>(wg, D.d, D.d, wu), D.T, D.d, D.F, D.F, true};
    return run_gemm<E, false, true>("gemm_dx", px, EpiStore<E>{dx, D.d, D.d, 0}, st);
}

// ------------------------------------------------------------ MoC inside MoE experts
constexpr int kMaxExperts = 8;

// Forward for rows already routed and sorted by expert (paper section "Compatibility with MoE
// architectures": every expert's MLP is a MoC network): rows off[e] .. off[e+1]-1 use the weights of
// expert e.  The three projections run as one grouped launch each over the experts; the row Top-K
// is expert-agnostic and runs once over all rows.
template <class E>
moc_status fwd_experts_impl(const Dims& D, int n_exp, const int32_t* off, const E* x, const E* wg, const E* wu, const E* wd,
                            E* y, int32_t* idx, E* gvals, E* uvals, void* ws, hipStream_t st) {
    FwdWs<E> W(ws, D, false);
    const int64_t wsz = (int64_t)D.F * D.d;
    GemmProblem<E> pr[kMaxExperts];
    EpiStore<float> eg[kMaxExperts];
    EpiStore<E> ee[kMaxExperts];
    moc_status s;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        pr[e] = GemmProblem<E>{kc_operand<E>(x + r0 * D.d, D.d), kc_operand<E>(wg + e * wsz, D.d), off[e + 1] - off[e], D.F, D.d, 0, false};
        eg[e] = EpiStore<float>{W.G + r0 * D.ldF, D.ldF, D.F, 0};
    }
    if ((s = run_gemm_grouped<E, false, false, EpiStore<float>, kMaxExperts>("gemm_gate_experts", n_exp, pr, eg, st)) != MOC_OK) return s;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        pr[e].B = kc_operand<E>(wu + e * wsz, D.d);
        ee[e] = EpiStore<E>{W.U + r0 * D.ldF, D.ldF, D.F, 0};
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
    const size_t expand_lds = (size_t)3 * D.ldF * sizeof(E);
    if (expand_lds > 160 * 1024 - 64) return fail(MOC_ERR_UNSUPPORTED, "F = %d too large for the expert backward", D.F);
    GemmProblem<E> pr[3 * kMaxExperts];
    EpiStore<E> ee[3 * kMaxExperts];
    moc_status s;
    for (int e = 0; e < n_exp; ++e) {
        const int64_t r0 = off[e];
        pr[e] = GemmProblem<E>{kc_operand<E>(dy + r0 * D.d, D.d), kc_operand<E>(wd + e * wsz, D.d), off[e + 1] - off[e], D.F, D.d, 0, false};
        ee[e] = EpiStore<E>{W.dZd + r0 * D.ldF, D.ldF, D.F, 0};
    }
    if ((s = run_gemm_grouped<E, false, false, EpiStore<E>, kMaxExperts>("gemm_dz_experts", n_exp, pr, ee, st)) != MOC_OK) return s;
    {
        auto kern = bwd_expand_kernel<E>;
        static bool attr = false;
        if (!attr) {
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        160 * 1024 - 64));
            attr = true;
        }
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

// ------------------------------------------------------------------------------ decode
template <class E, int BT>
moc_status decode_gate(const Dims& D, const E* x, const E* wg, float* g, hipStream_t st) {
    const size_t lds = (size_t)BT * D.d * sizeof(E);
    if (lds > 160 * 1024 - 64) return fail(MOC_ERR_UNSUPPORTED, "decode: d = %d too large for LDS staging", D.d);
    auto kern = decode_gate_kernel<E, BT>;
    static bool attr = false;
    if (!attr) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024 - 64));
        attr = true;
    }
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
    static bool attr = false;
    if (!attr) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    156 * 1024));
        attr = true;
    }
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
    static bool attr = false;
    if (!attr) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024 - 64));
        attr = true;
    }
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
    static bool attr = false;
    if (!attr) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    64 * 1024));
        attr = true;
    }
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
    // MOC_DECODE_FUSED=0 (read at every call) keeps grouped decode on the separate gate+select and gather
    // launches; MOC_DECODE_FUSED_P=n sets the workgroup count of the single-launch kernel.
    if (gb == 8 && (ga == 1 || ga == 2) && B == 1 && D.d <= 8 * 64 * Chunk<E>::N && env_int("MOC_DECODE_FUSED", 1) &&
        !options().force_generic) {
        // MoC_{a:8}, one token: gate, selection and gather in one launch, then the deterministic
        // reduction.  Two workgroups are resident per CU; the groups are dealt out evenly.
        const int ngroups = D.F / 8;
        const int rounds = (ngroups + kDecodeFusedMaxP - 1) / kDecodeFusedMaxP;
        const int want = env_int("MOC_DECODE_FUSED_P", (ngroups + rounds - 1) / rounds);
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
        static bool attr[2] = {false, false};
        if (!attr[B > 1]) {
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        160 * 1024 - 64));
            attr[B > 1] = true;
        }
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

// =============================================================================== C ABI
extern "C" {

size_t moc_workspace_bytes(const moc_shape* shape, int op) {
    if (check_shape(shape, op == MOC_OP_DECODE) != MOC_OK) return 0;
    if (op < MOC_OP_FWD || op > MOC_OP_FWD_KEYED) return 0;
    Dims D(*shape);
    return shape->dtype == MOC_BF16 ? workspace_for<bf16_t>(D, op) : workspace_for<float>(D, op);
}

#define CHECK_WS(op)                                                                                  \
    do {                                                                                              \
        CHECK_PTR(ws);                                                                                \
        size_t need_ = moc_workspace_bytes(shape, op);                                                \
        if (ws_bytes < need_) return fail(MOC_ERR_WORKSPACE, "workspace: %zu bytes given, %zu needed", ws_bytes, need_); \
    } while (0)

moc_status moc_ffn_fwd(const moc_shape* shape, const void* x, const void* wg, const void* wu, const void* wd, void* y,
                       int32_t* idx, void* gvals, void* uvals, void* ws, size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y); CHECK_PTR(idx); CHECK_PTR(gvals); CHECK_PTR(uvals);
    CHECK_WS(MOC_OP_FWD);
    Dims D(*shape);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return fwd_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd, (bf16_t*)y,
                                idx, (bf16_t*)gvals, (bf16_t*)uvals, ws, st);
    return fwd_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y, idx,
                           (float*)gvals, (float*)uvals, ws, st);
}

moc_status moc_ffn_bwd(const moc_shape* shape, const void* x, const void* wg, const void* wu, const void* wd,
                       const int32_t* idx, const void* gvals, const void* uvals, const void* dy, void* dx, void* dwg,
                       void* dwu, void* dwd, void* ws, size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, false);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(idx); CHECK_PTR(gvals); CHECK_PTR(uvals);
    CHECK_PTR(dy); CHECK_PTR(dx); CHECK_PTR(dwg); CHECK_PTR(dwu); CHECK_PTR(dwd);
    CHECK_WS(MOC_OP_BWD);
    Dims D(*shape);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return bwd_impl<bf16_t, false>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd, idx,
                                       (const bf16_t*)gvals, (const bf16_t*)uvals, (const bf16_t*)dy, (bf16_t*)dx,
                                       (bf16_t*)dwg, (bf16_t*)dwu, (bf16_t*)dwd, ws, st);
    return bwd_impl<float, false>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, idx,
                                  (const float*)gvals, (const float*)uvals, (const float*)dy, (float*)dx, (float*)dwg,
                                  (float*)dwu, (float*)dwd, ws, st);
}

moc_status moc_ffn_decode(const moc_shape* shape, const void* x, const void* wg, const void* wu, const void* wd,
                          void* y, int32_t* idx_or_null, void* ws, size_t ws_bytes, void* hip_stream) {
    moc_status s = check_shape(shape, true);
    if (s != MOC_OK) return s;
    CHECK_PTR(x); CHECK_PTR(wg); CHECK_PTR(wu); CHECK_PTR(wd); CHECK_PTR(y);
    if (idx_or_null && !aligned16(idx_or_null)) return fail(MOC_ERR_BAD_ARG, "idx is not 16-byte aligned");
    CHECK_WS(MOC_OP_DECODE);
    Dims D(*shape);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return decode_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                   (bf16_t*)y, idx_or_null, ws, st);
    return decode_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                              idx_or_null, ws, st);
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
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (sh.dtype == MOC_BF16)
        return swiglu_fwd_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                       (bf16_t*)y, (bf16_t*)g_save, (bf16_t*)u_save, ws, st);
    return swiglu_fwd_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                                  (float*)g_save, (float*)u_save, ws, st);
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
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (sh.dtype == MOC_BF16)
        return bwd_impl<bf16_t, true>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                      nullptr, (const bf16_t*)g_save, (const bf16_t*)u_save, (const bf16_t*)dy,
                                      (bf16_t*)dx, (bf16_t*)dwg, (bf16_t*)dwu, (bf16_t*)dwd, ws, st);
    return bwd_impl<float, true>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, nullptr,
                                 (const float*)g_save, (const float*)u_save, (const float*)dy, (float*)dx, (float*)dwg,
                                 (float*)dwu, (float*)dwd, ws, st);
}

moc_status moc_topk_rows(int32_t T, int32_t F, int32_t K, const float* g, int64_t ldg, int32_t* idx, float* gsel,
                         void* hip_stream) {
    if (T < 1 || F < 1 || K < 1 || K > F) return fail(MOC_ERR_BAD_ARG, "need T >= 1 and 1 <= K <= F (T=%d F=%d K=%d)", T, F, K);
    if (F > 32768) return fail(MOC_ERR_UNSUPPORTED, "F = %d exceeds 32768", F);
    if (ldg < F) return fail(MOC_ERR_BAD_ARG, "ldg < F");
    CHECK_PTR(g); CHECK_PTR(idx); CHECK_PTR(gsel);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    TopkArgs<float> a{g, ldg, F, K, idx, gsel, nullptr, nullptr, 0, nullptr, nullptr, 0};
    return run_topk<float, 256, false>("topk_rows", a, T, st);
}

static moc_status check_key_mode(int32_t key_mode) {
    if (key_mode < MOC_KEY_GATE || key_mode > MOC_KEY_ABS_SILU) return fail(MOC_ERR_BAD_ARG, "unknown selection key %d", key_mode);
    return MOC_OK;
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
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return fwd_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd, (bf16_t*)y,
                                idx, (bf16_t*)gvals, (bf16_t*)uvals, ws, st, 0, 0, key_mode);
    return fwd_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y, idx,
                           (float*)gvals, (float*)uvals, ws, st, 0, 0, key_mode);
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
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return decode_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                   (bf16_t*)y, idx_or_null, ws, st, 0, 0, key_mode);
    return decode_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                              idx_or_null, ws, st, 0, 0, key_mode);
}

moc_status moc_topk_rows_keyed(int32_t T, int32_t F, int32_t K, int32_t key_mode, const float* g, int64_t ldg,
                               float* key_scratch, int32_t* idx, float* gsel, void* hip_stream) {
    if (T < 1 || F < 1 || K < 1 || K > F) return fail(MOC_ERR_BAD_ARG, "need T >= 1 and 1 <= K <= F (T=%d F=%d K=%d)", T, F, K);
    if (F > 32768) return fail(MOC_ERR_UNSUPPORTED, "F = %d exceeds 32768", F);
    if (ldg < F) return fail(MOC_ERR_BAD_ARG, "ldg < F");
    moc_status s = check_key_mode(key_mode);
    if (s != MOC_OK) return s;
    CHECK_PTR(g); CHECK_PTR(idx); CHECK_PTR(gsel);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    TopkArgs<float> a{g, ldg, F, K, idx, gsel, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr};
    if (key_mode != MOC_KEY_GATE) {
        CHECK_PTR(key_scratch);
        // the last row is transformed up to F only: nothing past the caller's matrix is read
        if ((s = launch_key_transform(g, key_scratch, (int64_t)(T - 1) * ldg + F, key_mode, st)) != MOC_OK) return s;
        a.g = key_scratch;
        a.g_raw = g;
    }
    return run_topk<float, 256, false>("topk_rows", a, T, st);
}

static moc_status check_offsets(const moc_shape* shape, int32_t n_experts, const int32_t* off) {
    if (n_experts < 1 || n_experts > kMaxExperts) return fail(MOC_ERR_UNSUPPORTED, "n_experts must be 1..%d (got %d)", kMaxExperts, n_experts);
    if (!off) return fail(MOC_ERR_BAD_ARG, "expert_offsets is NULL");
    if (off[0] != 0 || off[n_experts] != shape->T) return fail(MOC_ERR_BAD_ARG, "expert_offsets must run from 0 to T");
    for (int e = 0; e < n_experts; ++e)
        if (off[e + 1] < off[e]) return fail(MOC_ERR_BAD_ARG, "expert_offsets must ascend");
    return MOC_OK;
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
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return fwd_experts_impl<bf16_t>(D, n_experts, expert_offsets, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu,
                                        (const bf16_t*)wd, (bf16_t*)y, idx, (bf16_t*)gvals, (bf16_t*)uvals, ws, st);
    return fwd_experts_impl<float>(D, n_experts, expert_offsets, (const float*)x, (const float*)wg, (const float*)wu,
                                   (const float*)wd, (float*)y, idx, (float*)gvals, (float*)uvals, ws, st);
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
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return bwd_experts_impl<bf16_t>(D, n_experts, expert_offsets, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu,
                                        (const bf16_t*)wd, idx, (const bf16_t*)gvals, (const bf16_t*)uvals, (const bf16_t*)dy,
                                        (bf16_t*)dx, (bf16_t*)dwg, (bf16_t*)dwu, (bf16_t*)dwd, ws, st);
    return bwd_experts_impl<float>(D, n_experts, expert_offsets, (const float*)x, (const float*)wg, (const float*)wu,
                                   (const float*)wd, idx, (const float*)gvals, (const float*)uvals, (const float*)dy, (float*)dx,
                                   (float*)dwg, (float*)dwu, (float*)dwd, ws, st);
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
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return fwd_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd, (bf16_t*)y,
                                idx, (bf16_t*)gvals, (bf16_t*)uvals, ws, st, ga, gb);
    return fwd_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y, idx,
                           (float*)gvals, (float*)uvals, ws, st, ga, gb);
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
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (shape->dtype == MOC_BF16)
        return decode_impl<bf16_t>(D, (const bf16_t*)x, (const bf16_t*)wg, (const bf16_t*)wu, (const bf16_t*)wd,
                                   (bf16_t*)y, idx_or_null, ws, st, ga, gb);
    return decode_impl<float>(D, (const float*)x, (const float*)wg, (const float*)wu, (const float*)wd, (float*)y,
                              idx_or_null, ws, st, ga, gb);
}

moc_status moc_topk_grouped_rows(int32_t T, int32_t F, int32_t ga, int32_t gb, const float* g, int64_t ldg, int32_t* idx,
                                 float* gsel, void* hip_stream) {
    if (T < 1 || F < 1) return fail(MOC_ERR_BAD_ARG, "need T >= 1 and F >= 1 (T=%d F=%d)", T, F);
    if (gb < 1 || F % gb != 0) return fail(MOC_ERR_BAD_ARG, "b = %d must divide F = %d", gb, F);
    moc_status s = check_group(F, F / gb * ga, ga, gb);
    if (s != MOC_OK) return s;
    if (ldg < F) return fail(MOC_ERR_BAD_ARG, "ldg < F");
    CHECK_PTR(g); CHECK_PTR(idx); CHECK_PTR(gsel);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    TopkArgs<float> a{g, ldg, F, F / gb * ga, idx, gsel, nullptr, nullptr, 0, nullptr, nullptr, 0};
    return run_group_select<float, false>("group_select_rows", a, T, ga, gb, st);
}

moc_status moc_rmsnorm(int32_t T, int32_t d, int32_t dtype, const void* h, const void* gain, float eps, void* out,
                       void* hip_stream) {
    if (T < 1 || d < 1) return fail(MOC_ERR_BAD_ARG, "T and d must be >= 1");
    if (dtype != MOC_F32 && dtype != MOC_BF16) return fail(MOC_ERR_BAD_ARG, "unknown dtype %d", dtype);
    CHECK_PTR(h); CHECK_PTR(gain); CHECK_PTR(out);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Span span("rmsnorm", st);
    if (dtype == MOC_BF16) {
        const bf16_t *hp = (const bf16_t*)h, *gp = (const bf16_t*)gain;
        bf16_t* op = (bf16_t*)out;
        if (d % 8 == 0 && d <= 256 * 8 * 2)
            hipLaunchKernelGGL((rmsnorm_kernel<bf16_t, true, 2>), dim3(T), dim3(256), 0, st, hp, gp, eps, d, op);
        else
            hipLaunchKernelGGL((rmsnorm_kernel<bf16_t, false, 1>), dim3(T), dim3(256), 0, st, hp, gp, eps, d, op);
    } else {
        const float *hp = (const float*)h, *gp = (const float*)gain;
        float* op = (float*)out;
        if (d % 4 == 0 && d <= 256 * 4 * 4)
            hipLaunchKernelGGL((rmsnorm_kernel<float, true, 4>), dim3(T), dim3(256), 0, st, hp, gp, eps, d, op);
        else
            hipLaunchKernelGGL((rmsnorm_kernel<float, false, 1>), dim3(T), dim3(256), 0, st, hp, gp, eps, d, op);
    }
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

moc_status moc_residual_add(int32_t T, int32_t d, int32_t dtype, void* h_inout, const void* y, void* hip_stream) {
    if (T < 1 || d < 1) return fail(MOC_ERR_BAD_ARG, "T and d must be >= 1");
    if (dtype != MOC_F32 && dtype != MOC_BF16) return fail(MOC_ERR_BAD_ARG, "unknown dtype %d", dtype);
    CHECK_PTR(h_inout); CHECK_PTR(y);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Span span("residual_add", st);
    const int64_t n = (int64_t)T * d;
    if (dtype == MOC_BF16) {
        const bool vec = n % 8 == 0;
        const int64_t work = vec ? n / 8 : n;
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((work + 255) / 256, 16384));
        if (vec) hipLaunchKernelGGL((residual_add_kernel<bf16_t, true>), dim3(grid), dim3(256), 0, st, (bf16_t*)h_inout, (const bf16_t*)y, n);
        else hipLaunchKernelGGL((residual_add_kernel<bf16_t, false>), dim3(grid), dim3(256), 0, st, (bf16_t*)h_inout, (const bf16_t*)y, n);
    } else {
        const bool vec = n % 4 == 0;
        const int64_t work = vec ? n / 4 : n;
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((work + 255) / 256, 16384));
        if (vec) hipLaunchKernelGGL((residual_add_kernel<float, true>), dim3(grid), dim3(256), 0, st, (float*)h_inout, (const float*)y, n);
        else hipLaunchKernelGGL((residual_add_kernel<float, false>), dim3(grid), dim3(256), 0, st, (float*)h_inout, (const float*)y, n);
    }
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

void moc_timing_enable(int on) { g_timing_on = on != 0; }

int32_t moc_timing_collect(void) {
    for (const PendingSpan& p : g_pending) {
        float ms = 0.0f;
        if (hipEventSynchronize(p.stop) == hipSuccess && hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
            g_entries[p.entry].ms += ms;
            g_entries[p.entry].launches += 1;
        }
        g_event_pool.push_back(p.start);
        g_event_pool.push_back(p.stop);
    }
    g_pending.clear();
    return (int32_t)g_entries.size();
}

moc_status moc_timing_get(int32_t i, char* name, int32_t name_cap, double* total_ms, int64_t* launches) {
    if (i < 0 || i >= (int32_t)g_entries.size()) return fail(MOC_ERR_BAD_ARG, "timing entry %d out of range", i);
    if (name && name_cap > 0) {
        strncpy(name, g_entries[i].name.c_str(), name_cap - 1);
        name[name_cap - 1] = 0;
    }
    if (total_ms) *total_ms = g_entries[i].ms;
    if (launches) *launches = g_entries[i].launches;
    return MOC_OK;
}

void moc_timing_reset(void) {
    moc_timing_collect();
    g_entries.clear();
}

const char* moc_status_string(int status) {
    switch (status) {
        case MOC_OK: return "MOC_OK";
        case MOC_ERR_BAD_ARG: return "MOC_ERR_BAD_ARG";
        case MOC_ERR_WORKSPACE: return "MOC_ERR_WORKSPACE";
        case MOC_ERR_UNSUPPORTED: return "MOC_ERR_UNSUPPORTED";
        case MOC_ERR_HIP: return "MOC_ERR_HIP";
    }
    return "MOC_ERR_UNKNOWN";
}

const char* moc_last_error(void) { return g_err; }

const char* moc_version(void) { return "moc-ffn 0.1 gfx950"; }

}  // extern "C"
