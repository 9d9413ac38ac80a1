// Down projection of the grouped variant MoC_{a:b} with a <= 2 on the structured-sparse matrix instruction
// (v_smfmac_f32_32x32x32_bf16): D[m, n] = sum_k Z'[m, k] W_down[k, n] with at most two nonzeros in every aligned
// group of four k, which a:b selection with a <= 2 and b in {4, 8, 16} guarantees (paper item "MoC with
// structured 2:8 sparsity").  One instruction then covers 32 k for the price of 16.
//
// Z' comes compressed (sparse_compress_kernel): per row and block of 32 k, sixteen kept values zc[m][16 blk ..]
// (two per group of four, groups stored in the order 0,1,4,5 | 2,3,6,7: the first eight values feed lanes 0..31
// of the instruction, the other eight lanes 32..63) and one position word zi[m][blk] (two bits per value: its
// place inside its group of four; low half-word for the first eight values).  Groups with fewer than two
// nonzeros are filled up with zeros at unused positions, positions ascending as the instruction requires.
// W_down is read k-major like the dense kernel's KM operand.  Same tile (256 x 256), staging depth and
// epilogue as the dense kernel; the A stage shrinks from 64 to 32 + 4 bytes per row.
//
// Measured at the 1B shape (T 8192, d_ffn 5464, d 2048, 2:8): 0.175 ms plus 0.031 ms for the compression, against
// 0.157 ms for the dense kernel on the dense-masked Z' -- the product is bound by staging W_down and by the LDS
// fragment reads, which the sparse instruction does not reduce -- so the library uses it only when
// MOC_GROUPED_SPARSE=1 asks for it.
#pragma once
#include "common.h"
#include "gemm_generic.h"
#include "gemm_mfma.h"
#include "kernel_attrs.h"

namespace moc {

typedef __bf16 sp_bf16x16_t __attribute__((ext_vector_type(16)));

struct SparseDownProblem {
    const bf16_t* zc;    // [M, ldzc] compressed values, ldzc = Kpad / 2
    const uint32_t* zi;  // [M, ldzi] position words, ldzi = Kpad / 32
    int64_t ldzc, ldzi;
    const bf16_t* w;     // [Krows, ldw] k-major dense operand
    int64_t ldw;
    int wext;            // readable columns of w (multiple of 8)
    int M, N, Kpad, Krows;   // Kpad: multiple of 32 (Z is zero past Krows); w rows past Krows-1 are clamped
};

constexpr int kSpStageA = 256 * 32;             // compressed values: 256 rows x 32 bytes
constexpr int kSpStageI = 256 * 4;              // position words
constexpr int kSpPitchB = 256 * 2 + 64;
constexpr int kSpStageB = 32 * kSpPitchB;
constexpr int kSpStage = kSpStageA + kSpStageI + kSpStageB;
constexpr int kSpLds = 3 * kSpStage;

template <class Epi>
__global__ __launch_bounds__(256) void gemm_sparse_down_kernel(SparseDownProblem pr, int tiles_m, int tiles_n, Epi epi) {
    constexpr int BM = 256, BN = 256, WM = 128, WN = 128, TM = 4, TN = 4;
    extern __shared__ __align__(16) unsigned char smem[];
    const int M = pr.M, N = pr.N;
    const int logical = xcd_contiguous_index(blockIdx.x, tiles_m * tiles_n);
    constexpr int GROUP = 8;
    const int band = logical / (GROUP * tiles_n);
    const int first_m = band * GROUP;
    const int gsz = min(tiles_m - first_m, GROUP);
    const int in_band = logical - band * GROUP * tiles_n;
    const int m0 = (first_m + in_band % gsz) * BM;
    const int n0 = (in_band / gsz) * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

    // staging: A values 2 chunks (row c/2, half c%2), position word 1 (row tid), B 4 chunks (k row c/32, col chunk c%32)
    int a_off[2], a_lds[2], b_col[4], b_lds[4], b_k[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + i * 256, row = c >> 1, h = c & 1;
        a_off[i] = min(m0 + row, M - 1) * (int)pr.ldzc + h * 8;
        a_lds[i] = row * 32 + h * 16;
    }
    const int i_off = min(m0 + tid, M - 1) * (int)pr.ldzi;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + i * 256, krow = c >> 5, ch = c & 31;
        b_col[i] = min(n0 + ch * 8, pr.wext - 8);
        b_lds[i] = kSpStageA + kSpStageI + krow * kSpPitchB + ch * 16;
        b_k[i] = krow;
    }
    const int nk = pr.Kpad / 32;
    u32x4_t ga[2][2], gb[2][4];
    uint32_t gi[2];
    auto fetch = [&](int buf, int kt) {
        kt = min(kt, nk - 1);
#pragma unroll
        for (int i = 0; i < 2; ++i) ga[buf][i] = *reinterpret_cast<const u32x4_t*>(pr.zc + a_off[i] + kt * 16);
        gi[buf] = pr.zi[i_off + kt];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int krow = min(kt * 32 + b_k[i], pr.Krows - 1);
            gb[buf][i] = *reinterpret_cast<const u32x4_t*>(pr.w + (int64_t)krow * pr.ldw + b_col[i]);
        }
    };
    auto stash = [&](int buf, int stage) {
        unsigned char* base = smem + stage * kSpStage;
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<u32x4_t*>(base + a_lds[i]) = ga[buf][i];
        *reinterpret_cast<uint32_t*>(base + kSpStageA + tid * 4) = gi[buf];
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4_t*>(base + b_lds[i]) = gb[buf][i];
    };
    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    bf16x8_t fz[2][TM];
    int fidx[2][TM];
    sp_bf16x16_t fw[2][TN];
    auto load_frags = [&](int fb, int stage) {
        const unsigned char* base = smem + stage * kSpStage;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = wm0 + i * 32 + (lane & 31);
            fz[fb][i] = *reinterpret_cast<const bf16x8_t*>(base + row * 32 + (lane >> 5) * 16);
            const uint32_t wd = *reinterpret_cast<const uint32_t*>(base + kSpStageA + row * 4);
            fidx[fb][i] = (int)((lane >> 5) ? (wd >> 16) : (wd & 0xFFFFu));
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            // lane (col = lane % 32 of block j, half hb = lane / 32) needs k = 16 hb .. 16 hb + 15: four transposing reads
            typedef s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
            const int col = wn0 + j * 32 + 16 * ((lane >> 4) & 1) + (lane & 3) * 4;
            const int krow = 16 * (lane >> 5) + ((lane & 15) >> 2);
            const unsigned char* p = base + kSpStageA + kSpStageI + krow * kSpPitchB + col * 2;
            s16x4_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
            s16x4_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * kSpPitchB));
            s16x4_t r2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 8 * kSpPitchB));
            s16x4_t r3 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 12 * kSpPitchB));
            typedef short s16x16_t __attribute__((ext_vector_type(16)));
            typedef short s16x8_t __attribute__((ext_vector_type(8)));
            s16x8_t lo = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
            s16x8_t hi = __builtin_shufflevector(r2, r3, 0, 1, 2, 3, 4, 5, 6, 7);
            s16x16_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
            fw[fb][j] = __builtin_bit_cast(sp_bf16x16_t, v);
        }
    };
    auto mma = [&](int fb) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(fz[fb][i], fw[fb][j], acc[i][j], fidx[fb][i], 0, 0);
    };

    fetch(0, 0);
    fetch(1, 1);
    stash(0, 0);
    stash(1, 1);
    fetch(0, 2);
    fetch(1, 3);
    __syncthreads();
    int st_cur = 0, st_next = 1, st_fill = 2;
    load_frags(0, 0);
    // slice kt: fragments of slice kt are in buffer kt & 1; those of slice kt+1 (visible since the last
    // barrier) are read while the MFMAs of slice kt run
    auto slice = [&](auto buf_c, int kt) {
        constexpr int buf = decltype(buf_c)::value;
        load_frags(buf ^ 1, st_next);
        stash(buf, st_fill);
        fetch(buf, kt + 4);
        mma(buf);
        constexpr int NM = TM * TN;
        SchedSeq<0, NM, 0, NM / 2, 2 * TM + 4 * TN, NM / 2, NM, 7, 0, NM, 7>::apply();
        __syncthreads();
        const int t = st_cur;
        st_cur = st_next;
        st_next = st_fill;
        st_fill = t;
    };
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        slice(std::integral_constant<int, 0>{}, kt);
        slice(std::integral_constant<int, 1>{}, kt + 1);
    }
    if (kt < nk) slice(std::integral_constant<int, 0>{}, kt);

    // epilogue: acc[i][j][4 ii + r] = D[m = .. + 8 ii + 4 (lane / 32) + r][n = .. + lane % 32]; staged per 32-row
    // block in a wave-private [32][WN] fp32 area, then handed to the functor as row segments
    {
        constexpr int EPITCH = WN * 4 + 16;
        static_assert(4 * 32 * EPITCH <= kSpLds, "epilogue staging must fit");
        unsigned char* area = smem + wave * (32 * EPITCH);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    const int col = j * 32 + (lane & 31);
                    *reinterpret_cast<float*>(area + row * EPITCH + col * 4) = acc[i][j][e];
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            constexpr int LPR = WN / 4, RPI = 64 / LPR;
#pragma unroll 4
            for (int it = 0; it < 32 / RPI; ++it) {
                const int row = it * RPI + lane / LPR, c4 = lane % LPR;
                const f32x4_t t = *reinterpret_cast<const f32x4_t*>(area + row * EPITCH + c4 * 16);
                const int m = m0 + wm0 + i * 32 + row;
                const float v[4] = {t[0], t[1], t[2], t[3]};
                if (m < M) epi.store4(m, n0 + wn0 + c4 * 4, v);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// Z' [T, ldz] dense-masked (ldz a multiple of 32, zero past the last channel) -> compressed form.  One thread
// per row and block of 32 channels.  A value counts as present when it is not +-0.
static __global__ __launch_bounds__(256) void sparse_compress_kernel(const bf16_t* __restrict__ zd, int64_t ldz, int T,
                                                                     bf16_t* __restrict__ zc, uint32_t* __restrict__ zi) {
    const int nblk = (int)(ldz / 32);
    const int64_t g = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (g >= (int64_t)T * nblk) return;
    const int64_t row = g / nblk;
    const int blk = (int)(g - row * nblk);
    const bf16_t* src = zd + row * ldz + blk * 32;
    uint16_t in[32];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(src + q * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            in[q * 8 + 2 * e] = (uint16_t)(v[e] & 0xFFFFu);
            in[q * 8 + 2 * e + 1] = (uint16_t)(v[e] >> 16);
        }
    }
    uint16_t out[16];
    uint32_t word = 0;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int grp = (s & 1) + ((s >> 1) & 1) * 4 + (s >> 2) * 2;      // 0,1,4,5,2,3,6,7
        // positions of the first two nonzeros; missing ones are filled with unused positions, ascending
        int p0 = -1, p1 = -1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool nz = (in[grp * 4 + i] & 0x7FFFu) != 0;
            if (nz && p0 < 0) p0 = i;
            else if (nz && p1 < 0) p1 = i;
        }
        if (p0 < 0) { p0 = 0; p1 = 1; }
        else if (p1 < 0) {
            if (p0 == 3) { p1 = 3; p0 = 2; }
            else p1 = 3;
        }
        uint16_t v0 = 0, v1 = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i == p0) v0 = in[grp * 4 + i];
            if (i == p1) v1 = in[grp * 4 + i];
        }
        out[s * 2] = v0;
        out[s * 2 + 1] = v1;
        word |= ((uint32_t)p0 << (4 * s)) | ((uint32_t)p1 << (4 * s + 2));
    }
    bf16_t* dst = zc + row * (ldz / 2) + blk * 16;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        u32x4_t v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (uint32_t)out[q * 8 + 2 * e] | ((uint32_t)out[q * 8 + 2 * e + 1] << 16);
        *reinterpret_cast<u32x4_t*>(dst + q * 8) = v;
    }
    zi[row * nblk + blk] = word;
}

template <class Epi>
inline hipError_t launch_gemm_sparse_down(const SparseDownProblem& p, const Epi& epi, hipStream_t st) {
    auto kern = gemm_sparse_down_kernel<Epi>;
    LdsAttr<gemm_sparse_down_kernel<Epi>, kSpLds>::use();      // attribute set at library set-up
    const int tiles_m = (p.M + 255) / 256, tiles_n = (p.N + 255) / 256;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), kSpLds, st, p, tiles_m, tiles_n, epi);
    return hipGetLastError();
}

}  // namespace moc
