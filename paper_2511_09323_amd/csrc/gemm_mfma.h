// bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16).
//
//   C[m, n] = sum_k A[m, k] B[n, k]  (+ a second operand pair accumulated into the same tile)
//
// Both operands are row-major with the contraction index contiguous, every contraction length is
// a multiple of BK and every leading dimension a multiple of 8 elements (the host checks this).
// One workgroup computes a BM x BN tile; its WGM x WGN wavefronts each own a (BM/WGM) x (BN/WGN)
// sub-tile made of 32x32 MFMA blocks.  k-slices of BK elements are staged global -> registers ->
// LDS, two LDS stages, one barrier per slice.  LDS rows are padded by 16 bytes so that the
// 16-byte fragment reads of 16 consecutive rows fall on disjoint banks.
//
// Operand roles: the B rows (n) feed the MFMA "A" input and the A rows (m) the MFMA "B" input, so
// a lane ends up with four consecutive n for one m -- the shape the epilogues want for
// row-major [m, n] stores.
#pragma once
#include "common.h"
#include "gemm_generic.h"

namespace moc {

template <int BM, int BN, int BK, int WGM, int WGN> struct MfmaCfg {
    static constexpr int kThreads = WGM * WGN * 64;
    static constexpr int kPitch = BK * 2 + 16;                 // bytes per LDS row
    static constexpr int kStage = (BM + BN) * kPitch;          // bytes per stage
    static constexpr int kLds = 2 * kStage;
};

template <int BM, int BN, int BK, int WGM, int WGN, class Epi>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_nt_bf16_mfma_kernel(GemmOperands<bf16_t> op, int M, int N,
                                                                            int tiles_m, int tiles_n, Epi epi) {
    using Cfg = MfmaCfg<BM, BN, BK, WGM, WGN>;
    constexpr int NTHR = Cfg::kThreads;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int PITCH = Cfg::kPitch;
    constexpr int CH = BK / 8;                 // 16-byte chunks per tile row
    constexpr int LA = BM * CH / NTHR, LB = BN * CH / NTHR;
    static_assert(BM * CH % NTHR == 0 && BN * CH % NTHR == 0, "staging must divide evenly");
    extern __shared__ __align__(16) unsigned char smem[];

    // ---- workgroup -> tile: contiguous tile ranges per XCD (workgroup w runs on XCD w % 8),
    //      tiles ordered in bands of 8 tile-rows so one XCD's L2 sees few distinct panels.
    const int nblk = tiles_m * tiles_n;
    const int w = blockIdx.x;
    const int xcd = w & 7, local = w >> 3;
    const int logical = xcd * (nblk >> 3) + min(xcd, nblk & 7) + local;
    constexpr int GROUP = 8;
    const int band = logical / (GROUP * tiles_n);
    const int first_m = band * GROUP;
    const int gsz = min(tiles_m - first_m, GROUP);
    const int in_band = logical - band * GROUP * tiles_n;
    const int tile_m = first_m + in_band % gsz;
    const int tile_n = in_band / gsz;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;

    // ---- staging assignment: chunk c = tid + i * NTHR -> (row c / CH, 16-byte chunk c % CH).
    //      Rows past the matrix edge are clamped to the last row (their results are never stored).
    int a_off[LA], b_off[LB];      // element offsets from the tile's first row
    int a_lds[LA], b_lds[LB];      // byte offsets inside a stage
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        int c = tid + i * NTHR, row = c / CH, ch = c % CH;
        a_off[i] = (min(m0 + row, M - 1) - m0) * (int)op.lda + ch * 8;
        a_lds[i] = row * PITCH + ch * 16;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        int c = tid + i * NTHR, row = c / CH, ch = c % CH;
        b_off[i] = (min(n0 + row, N - 1) - n0) * (int)op.ldb + ch * 8;
        b_lds[i] = BM * PITCH + row * PITCH + ch * 16;
    }
    const int nk0 = op.Kc / BK;
    const int nk = nk0 + (op.A2 ? op.Kc2 / BK : 0);
    const bf16_t* a_base0 = op.A + (int64_t)m0 * op.lda;
    const bf16_t* b_base0 = op.B + (int64_t)n0 * op.ldb;
    const bf16_t* a_base1 = op.A2 ? op.A2 + (int64_t)m0 * op.lda2 : nullptr;
    const bf16_t* b_base1 = op.B2 ? op.B2 + (int64_t)n0 * op.ldb2 : nullptr;

    u32x4_t ra[LA], rb[LB];
    auto fetch = [&](int kt) {
        const bool seg = kt >= nk0;
        const int koff = (seg ? kt - nk0 : kt) * BK;
        const bf16_t* ab = (seg ? a_base1 : a_base0) + koff;
        const bf16_t* bb = (seg ? b_base1 : b_base0) + koff;
#pragma unroll
        for (int i = 0; i < LA; ++i) ra[i] = *reinterpret_cast<const u32x4_t*>(ab + a_off[i]);
#pragma unroll
        for (int i = 0; i < LB; ++i) rb[i] = *reinterpret_cast<const u32x4_t*>(bb + b_off[i]);
    };
    auto stash = [&](int stage) {
        unsigned char* base = smem + stage * Cfg::kStage;
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<u32x4_t*>(base + a_lds[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<u32x4_t*>(base + b_lds[i]) = rb[i];
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // fragment addresses inside a stage: row (lane % 32), k offset 8 * (lane / 32) elements
    const int frag_off = (lane & 31) * PITCH + (lane >> 5) * 16;
    const int a_frag0 = (wm0)*PITCH + frag_off;                 // A rows (m) -> MFMA B input
    const int b_frag0 = BM * PITCH + (wn0)*PITCH + frag_off;    // B rows (n) -> MFMA A input

    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) fetch(kt + 1);
        const unsigned char* base = smem + (kt & 1) * Cfg::kStage;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8_t fn[TN], fm[TM];
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fn[j] = *reinterpret_cast<const bf16x8_t*>(base + b_frag0 + j * 32 * PITCH + kk * 32);
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fm[i] = *reinterpret_cast<const bf16x8_t*>(base + a_frag0 + i * 32 * PITCH + kk * 32);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fn[j], fm[i], acc[i][j], 0, 0, 0);
        }
        if (more) stash((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: acc[i][j][4*ii + r] is C[m, n] with m = .. + lane % 32, n = .. + 8*ii + 4*(lane/32) + r
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm0 + i * 32 + (lane & 31);
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                const int n = n0 + wn0 + j * 32 + 8 * ii + 4 * (lane >> 5);
                float v[4] = {acc[i][j][4 * ii], acc[i][j][4 * ii + 1], acc[i][j][4 * ii + 2], acc[i][j][4 * ii + 3]};
                epi.store4(m, n, v);
            }
        }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, class Epi>
inline hipError_t launch_gemm_nt_bf16_mfma_cfg(const GemmOperands<bf16_t>& op, int M, int N, const Epi& epi,
                                               hipStream_t st) {
    using Cfg = MfmaCfg<BM, BN, BK, WGM, WGN>;
    auto kern = gemm_nt_bf16_mfma_kernel<BM, BN, BK, WGM, WGN, Epi>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(Cfg::kThreads), Cfg::kLds, st, op, M, N, tiles_m,
                       tiles_n, epi);
    return hipGetLastError();
}

// True when the MFMA kernel's layout assumptions hold for this operand set.
inline bool mfma_operands_ok(const GemmOperands<bf16_t>& op) {
    auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    bool ok = op.Kc > 0 && op.Kc % 64 == 0 && op.lda % 8 == 0 && op.ldb % 8 == 0 && al16(op.A) && al16(op.B);
    if (op.A2) ok = ok && op.Kc2 > 0 && op.Kc2 % 64 == 0 && op.lda2 % 8 == 0 && op.ldb2 % 8 == 0 && al16(op.A2) && al16(op.B2);
    return ok;
}

}  // namespace moc
