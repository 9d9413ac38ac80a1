// Decode path (paper section "Accelerated inference"): g = x W_gate over every channel, Top-K per
// token, then u_j = x . W_up[:, j] and y += SiLU(g_j) u_j w_j only for the selected channels j.
// All three weights are channel-major [F, d], so one channel is one contiguous row in each.
//
// The kernels stream weight rows with 16-byte loads, one wavefront per row (or row segment), and
// keep x in LDS.  All are bandwidth-bound; the arithmetic is fp32 FMA on the vector ALU.
#pragma once
#include "common.h"
#include "group_select.h"

namespace moc {

template <class E> struct Chunk;   // 16 bytes of E as floats
template <> struct Chunk<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(u32x4_t t, float* v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(t[i]);
    }
    static __device__ __forceinline__ void load(const float* p, float* v) {
        unpack(*reinterpret_cast<const u32x4_t*>(p), v);
    }
    // acc + sum of the products of the elements of two chunks
    static __device__ __forceinline__ float dot(u32x4_t a, u32x4_t b, float acc) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = fmaf(__uint_as_float(a[i]), __uint_as_float(b[i]), acc);
        return acc;
    }
};
template <> struct Chunk<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(u32x4_t t, float* v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(t[i] << 16);
            v[2 * i + 1] = __uint_as_float(t[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
        unpack(*reinterpret_cast<const u32x4_t*>(p), v);
    }
    // (v_dot2c_f32_bf16 would halve the instruction count but measured slower here.)
    static __device__ __forceinline__ float dot(u32x4_t a, u32x4_t b, float acc) {
        float w[N], x[N];
        unpack(a, w);
        unpack(b, x);
#pragma unroll
        for (int i = 0; i < N; ++i) acc = fmaf(w[i], x[i], acc);
        return acc;
    }
};

// g[b, j] = x[b] . wg[j]  for every channel j and every token b < B (B <= BT).
// x is staged in LDS ([BT, d] of E); each wavefront walks rows j = global wave id, += total waves.
template <class E, int BT>
__global__ __launch_bounds__(256) void decode_gate_kernel(const E* __restrict__ x, const E* __restrict__ wg, int B,
                                                          int d, int F, float* __restrict__ g, int64_t ldg) {
    constexpr int CN = Chunk<E>::N;
    extern __shared__ __align__(16) unsigned char dec_smem[];
    E* xs = reinterpret_cast<E*>(dec_smem);
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), nwave = gridDim.x * 4;
    constexpr int UN = 8;      // 16-byte chunks of a row per lane: rows of up to 64 * CN * UN elements in one go
    const bool whole_rows = d <= 64 * CN * UN;
    u32x4_t cur[UN], nxt[UN];
    auto fetch = [&](u32x4_t (&r)[UN], int j) {
        const E* wrow = wg + (int64_t)j * d;
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = (u * 64 + lane) * CN;
            r[u] = u32x4_t{0, 0, 0, 0};
            if (k < d) r[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + k));
        }
    };
    if (whole_rows && wave < F) fetch(cur, wave);          // in flight while x is staged
    for (int i = threadIdx.x * CN; i < BT * d; i += 256 * CN) {
        int b = i / d;
        u32x4_t v = {0, 0, 0, 0};
        if (b < B) v = *reinterpret_cast<const u32x4_t*>(x + i);
        *reinterpret_cast<u32x4_t*>(xs + i) = v;
    }
    __syncthreads();
    if (whole_rows) {
        // whole row in registers; the next row's loads are issued before this row is reduced
        for (int j = wave; j < F; j += nwave) {
            const bool more = j + nwave < F;
            if (more) fetch(nxt, j + nwave);
            float acc[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) acc[b] = 0.0f;
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int k = (u * 64 + lane) * CN;
                if (k < d) {
#pragma unroll
                    for (int b = 0; b < BT; ++b)
                        acc[b] = Chunk<E>::dot(cur[u], *reinterpret_cast<const u32x4_t*>(xs + b * d + k), acc[b]);
                }
            }
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                float s = wave_sum(acc[b]);
                if (lane == 0 && b < B) g[(int64_t)b * ldg + j] = s;
            }
            if (more) {
#pragma unroll
                for (int u = 0; u < UN; ++u) cur[u] = nxt[u];
            }
        }
        return;
    }
    for (int j = wave; j < F; j += nwave) {
        const E* wrow = wg + (int64_t)j * d;
        float acc[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) acc[b] = 0.0f;
        for (int k0 = lane * CN; k0 < d; k0 += 64 * CN * UN) {
            u32x4_t raw[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int k = k0 + u * 64 * CN;
                raw[u] = u32x4_t{0, 0, 0, 0};
                if (k < d) raw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + k));
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int k = k0 + u * 64 * CN;
                if (k < d) {
#pragma unroll
                    for (int b = 0; b < BT; ++b)
                        acc[b] = Chunk<E>::dot(raw[u], *reinterpret_cast<const u32x4_t*>(xs + b * d + k), acc[b]);
                }
            }
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float s = wave_sum(acc[b]);
            if (lane == 0 && b < B) g[(int64_t)b * ldg + j] = s;
        }
    }
}

// Grouped selection of MoC_{a:b} for one group and one token: vals[i * stride] are the gate values of
// channels c0 .. c0 + GB - 1; the kept channels go to slots q*ga .. q*ga + ga - 1 of the token's row.
template <int GB>
__device__ __forceinline__ void decode_group_select(const float* vals, int stride, int c0, int q, int ga,
                                                    int32_t* idx_row, float* gsel_row) {
    float v[GB];
#pragma unroll
    for (int i = 0; i < GB; ++i) v[i] = vals[i * stride];
    int rank[GB];
    group_ranks<GB>(v, rank);
    int r = 0;
#pragma unroll
    for (int i = 0; i < GB; ++i) {
        if (rank[i] < ga && r < ga) {                  // r < ga only matters for non-finite input
            idx_row[q * ga + r] = c0 + i;
            gsel_row[q * ga + r] = v[i];
            ++r;
        }
    }
}

// Gate projection fused with the grouped selection of MoC_{a:b}: a workgroup owns one group of GB
// consecutive channels at a time (wave w computes rows w, w + 4, ... of the group), the GB x B gate
// values meet in LDS and thread b selects for token b.  No gate row is written to memory.
template <class E, int BT, int GB>
__global__ __launch_bounds__(256) void decode_gate_group_kernel(const E* __restrict__ x, const E* __restrict__ wg,
                                                                int B, int d, int F, int ga, int K,
                                                                int32_t* __restrict__ idx, float* __restrict__ gsel) {
    constexpr int CN = Chunk<E>::N;
    extern __shared__ __align__(16) unsigned char dec_smem[];
    E* xs = reinterpret_cast<E*>(dec_smem);
    __shared__ float gl[2][GB][BT];
    for (int i = threadIdx.x * CN; i < BT * d; i += 256 * CN) {
        int b = i / d;
        u32x4_t v = {0, 0, 0, 0};
        if (b < B) v = *reinterpret_cast<const u32x4_t*>(x + i);
        *reinterpret_cast<u32x4_t*>(xs + i) = v;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int UN = 8;      // 16-byte chunks of the row in flight per lane
    int it = 0;
    for (int q = blockIdx.x; q < F / GB; q += gridDim.x, ++it) {
        for (int rr = wave; rr < GB; rr += 4) {
            const E* wrow = wg + (int64_t)(q * GB + rr) * d;
            float acc[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) acc[b] = 0.0f;
            for (int k0 = lane * CN; k0 < d; k0 += 64 * CN * UN) {
                u32x4_t raw[UN];
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int k = k0 + u * 64 * CN;
                    raw[u] = u32x4_t{0, 0, 0, 0};
                    if (k < d) raw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + k));
                }
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int k = k0 + u * 64 * CN;
                    if (k < d) {
#pragma unroll
                        for (int b = 0; b < BT; ++b)
                            acc[b] = Chunk<E>::dot(raw[u], *reinterpret_cast<const u32x4_t*>(xs + b * d + k), acc[b]);
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                float s = wave_sum(acc[b]);
                if (lane == 0) gl[it & 1][rr][b] = s;
            }
        }
        __syncthreads();       // gl[it & 1] complete; gl[(it + 1) & 1] is free again (read two barriers ago)
        if (threadIdx.x < B)
            decode_group_select<GB>(&gl[it & 1][0][threadIdx.x], BT, q * GB, q, ga, idx + (int64_t)threadIdx.x * K,
                                    gsel + (int64_t)threadIdx.x * K);
    }
}

// Gate projection for batches of 2..16 tokens on the matrix cores (bf16 only):
//   g[b, j] = x[b] . wg[j]  as D[row j][token b] tiles of v_mfma_f32_16x16x32_bf16.
// A workgroup of RG * KS wavefronts owns 16 RG consecutive channel rows: wave w works on row group
// w / KS (16 rows) and on share w % KS of the contraction, UN steps of 64 k (8 KB at UN = 4) in
// flight per wave.  Lane l of a wave reads 32 contiguous bytes of row l % 16 per step (4 lanes cover
// a 128-byte line); x[BTOK, d] sits in LDS (rows padded by 16 bytes) and supplies the second MFMA
// input with the same k assignment (token slots from BTOK up are zero).  The KS partial tiles of a
// row group are summed through LDS.  Needs d % (64 KS UN) == 0.
// Two shapes are used: (RG 3, KS 4, BTOK 16, UN 4), 768 threads, 48 rows, one workgroup per CU because
// x fills most of the LDS; and for at most four tokens (RG 1, KS 8, BTOK 4, UN 8), 512 threads, 16
// rows, every load of a wave in flight at once and several workgroups per CU.
// GB = 0 writes the gate rows g[B, ldg]; GB = 4, 8, 16 selects the a largest of every GB channels
// instead (MoC_{a:b}; the rows of a workgroup are a whole number of groups) and writes idx / gsel
// [B, K] only.
typedef __bf16 dec_bf16x8_t __attribute__((ext_vector_type(8)));
template <int GB, int RG, int KS, int BTOK, int UN>
__global__ __launch_bounds__(RG * KS * 64) void decode_gate_mfma_kernel(const bf16_t* __restrict__ x,
                                                                         const bf16_t* __restrict__ wg, int B, int d, int F,
                                                                         float* __restrict__ g, int64_t ldg, int ga, int K,
                                                                         int32_t* __restrict__ idx, float* __restrict__ gsel) {
    constexpr int NT = RG * KS * 64, ROWS = RG * 16;
    static_assert(GB == 0 || ROWS % GB == 0, "a workgroup's rows must be whole groups");
    extern __shared__ __align__(16) unsigned char dec_smem[];
    const int xpitch = d * 2 + 16;                                   // bytes per staged token row
    float* red = reinterpret_cast<float*>(dec_smem + BTOK * xpitch); // [RG row groups][KS shares][256]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rg = wave / KS, ks = wave % KS;
    const int row0 = blockIdx.x * ROWS + rg * 16;
    const int kq = d / KS;                                           // contraction share of this wave
    const int q = lane >> 4;                                         // 16-element k sub-block of a 64-wide step
    const bf16_t* wrow = wg + (int64_t)min(row0 + (lane & 15), F - 1) * d + ks * kq + q * 16;
    // first weights in flight before x is staged
    u32x4_t w0[UN], w1[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
        w0[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + u * 64));
        w1[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + u * 64 + 8));
    }
    for (int i = tid * 8; i < BTOK * d; i += NT * 8) {
        const int b = i / d, k = i - b * d;
        u32x4_t v = {0, 0, 0, 0};
        if (b < B) v = *reinterpret_cast<const u32x4_t*>(x + i);
        *reinterpret_cast<u32x4_t*>(dec_smem + b * xpitch + k * 2) = v;
    }
    __syncthreads();
    const bool tok = (lane & 15) < BTOK;                             // this lane's token slot holds a token
    const unsigned char* xl = dec_smem + (tok ? (lane & 15) : 0) * xpitch + (ks * kq + q * 16) * 2;
    f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
    const int nstep = kq / 64;
    for (int s0 = 0; s0 < nstep; s0 += UN) {
        u32x4_t c0[UN], c1[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) { c0[u] = w0[u]; c1[u] = w1[u]; }
        if (s0 + UN < nstep) {
            const int nxt = min(s0 + UN, nstep - UN);                // clamped prefetch of the next UN steps
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                w0[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + (nxt + u) * 64));
                w1[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + (nxt + u) * 64 + 8));
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            if (s0 + u < nstep) {
                u32x4_t x0 = {0, 0, 0, 0}, x1 = {0, 0, 0, 0};
                if (BTOK == 16 || tok) {
                    x0 = *reinterpret_cast<const u32x4_t*>(xl + (s0 + u) * 128);
                    x1 = *reinterpret_cast<const u32x4_t*>(xl + (s0 + u) * 128 + 16);
                }
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dec_bf16x8_t, c0[u]),
                                                              __builtin_bit_cast(dec_bf16x8_t, x0), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dec_bf16x8_t, c1[u]),
                                                              __builtin_bit_cast(dec_bf16x8_t, x1), acc, 0, 0, 0);
            }
        }
    }
    // acc[r] = D[row 4*(lane/16) + r][token lane % 16] over this wave's share of k
    *reinterpret_cast<f32x4_t*>(red + ((rg * KS + ks) * 64 + lane) * 4) = acc;
    __syncthreads();
    float* tile = red + RG * KS * 256;                               // [ROWS][17], grouped selection only
    if (ks == 0) {
        f32x4_t s = acc;
#pragma unroll
        for (int o = 1; o < KS; ++o) s += *reinterpret_cast<const f32x4_t*>(red + ((rg * KS + o) * 64 + lane) * 4);
        const int b = lane & 15, r = row0 + 4 * (lane >> 4);
        if (GB == 0) {
            if (b < B) {
                if (r + 3 < F) *reinterpret_cast<f32x4_t*>(g + (int64_t)b * ldg + r) = s;
                else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (r + e < F) g[(int64_t)b * ldg + r + e] = s[e];
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) tile[(rg * 16 + 4 * (lane >> 4) + e) * 17 + b] = s[e];
        }
    }
    if (GB != 0) {
        __syncthreads();
        constexpr int GBS = GB == 0 ? 8 : GB;
        const int grp = tid >> 4, b = tid & 15;                     // group of this workgroup's rows, token
        const int c0 = blockIdx.x * ROWS + grp * GBS;
        if (grp < ROWS / GBS && b < B && c0 < F)
            decode_group_select<GBS>(tile + grp * GBS * 17 + b, 17, c0, c0 / GBS, ga, idx + (int64_t)b * K,
                                     gsel + (int64_t)b * K);
    }
}

// LDS bytes of decode_gate_mfma_kernel.
inline size_t decode_gate_mfma_lds(int d, int RG, int KS, int BTOK) {
    return (size_t)BTOK * (d * 2 + 16) + (size_t)RG * KS * 256 * sizeof(float) + (size_t)RG * 16 * 17 * sizeof(float);
}

// z[b, s] = SiLU(gsel[b, s]) * (x[b] . wu[idx[b, s]])  for every selected (token, channel) pair.
// grid = (row groups, B); x[b] is staged in LDS.
template <class E>
__global__ __launch_bounds__(256) void decode_up_kernel(const E* __restrict__ x, const E* __restrict__ wu,
                                                        const int32_t* __restrict__ idx,
                                                        const float* __restrict__ gsel, int d, int K,
                                                        float* __restrict__ z) {
    constexpr int CN = Chunk<E>::N;
    extern __shared__ __align__(16) unsigned char dec_smem[];
    E* xs = reinterpret_cast<E*>(dec_smem);
    const int b = blockIdx.y;
    for (int i = threadIdx.x * CN; i < d; i += 256 * CN)
        *reinterpret_cast<u32x4_t*>(xs + i) = *reinterpret_cast<const u32x4_t*>(x + (int64_t)b * d + i);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), nwave = gridDim.x * 4;
    for (int s = wave; s < K; s += nwave) {
        const int j = idx[(int64_t)b * K + s];
        const E* wrow = wu + (int64_t)j * d;
        float acc = 0.0f;
        for (int k = lane * CN; k < d; k += 64 * CN) {
            float w[CN], xv[CN];
            Chunk<E>::load(wrow + k, w);
            Chunk<E>::load(xs + k, xv);
#pragma unroll
            for (int e = 0; e < CN; ++e) acc = fmaf(w[e], xv[e], acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) z[(int64_t)b * K + s] = silu_f32(gsel[(int64_t)b * K + s]) * acc;
    }
}

// part[p, b, c] = sum over the p-th share of token b's selected channels of z[b, s] * wd[idx[b, s], c]
// for the 64*CN*DIT-wide slice of columns c chosen by blockIdx.z.  grid = (P, B, slices).
template <class E, int DIT>
__global__ __launch_bounds__(256) void decode_down_kernel(const E* __restrict__ wd, const int32_t* __restrict__ idx,
                                                          const float* __restrict__ z, int d, int K, int P,
                                                          float* __restrict__ part) {
    constexpr int CN = Chunk<E>::N;
    constexpr int SLICE = 64 * CN * DIT;
    __shared__ float red[4][SLICE];
    const int p = blockIdx.x, b = blockIdx.y, c0 = blockIdx.z * SLICE;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (K + P - 1) / P;
    const int s_begin = p * per, s_end = min(K, s_begin + per);
    float acc[DIT][CN];
#pragma unroll
    for (int i = 0; i < DIT; ++i)
#pragma unroll
        for (int e = 0; e < CN; ++e) acc[i][e] = 0.0f;
    for (int s = s_begin + wave; s < s_end; s += 4) {
        const int j = idx[(int64_t)b * K + s];
        const float zz = z[(int64_t)b * K + s];
        const E* wrow = wd + (int64_t)j * d + c0;
#pragma unroll
        for (int i = 0; i < DIT; ++i) {
            const int c = i * 64 * CN + lane * CN;
            if (c0 + c < d) {
                float w[CN];
                Chunk<E>::load(wrow + c, w);
#pragma unroll
                for (int e = 0; e < CN; ++e) acc[i][e] = fmaf(zz, w[e], acc[i][e]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < DIT; ++i)
#pragma unroll
        for (int e = 0; e < CN; ++e) red[wave][i * 64 * CN + lane * CN + e] = acc[i][e];
    __syncthreads();
    for (int c = threadIdx.x; c < SLICE; c += 256) {
        if (c0 + c < d)
            part[((int64_t)p * gridDim.y + b) * d + c0 + c] = red[0][c] + red[1][c] + red[2][c] + red[3][c];
    }
}

// Fused gather stage for one token per workgroup column: for the p-th share of token b's selected
// channels, u = x[b] . wu[j], z' = SiLU(g) u, and part[p, b, :] = sum z' wd[j, :].  A wavefront
// owns a channel at a time and has both of its rows (one of wu, one of wd, NIT 16-byte chunks per
// lane each) in flight before it waits.  P * B workgroups of 512 threads; needs d <= 64 * CN * NIT.
// Workgroup w of the P * B launched handles (share p, token b).  idx rows ascend, so share p of every
// token covers about the same channel range: when P is a multiple of 8 the workgroups of one share
// are placed on one XCD (w % 8), whose L2 then serves the rows that several tokens selected
// (SHARED = true also drops the non-temporal hint so that those rows stay in L2).
template <class E, int NIT, bool SHARED>
__global__ __launch_bounds__(512) void decode_updown_kernel(const E* __restrict__ x, const E* __restrict__ wu,
                                                            const E* __restrict__ wd,
                                                            const int32_t* __restrict__ idx,
                                                            const float* __restrict__ gsel, int d, int K, int P, int B,
                                                            float* __restrict__ part) {
    constexpr int CN = Chunk<E>::N;
    constexpr int NWV = 8;
    extern __shared__ __align__(16) unsigned char dec_smem[];
    E* xs = reinterpret_cast<E*>(dec_smem);
    float* red = reinterpret_cast<float*>(dec_smem + (size_t)d * sizeof(E));     // [NWV][d]
    int p, b;
    if (SHARED && P % 8 == 0) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        p = xcd + 8 * (slot / B);
        b = slot % B;
    } else {
        p = blockIdx.x / B;
        b = blockIdx.x % B;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (K + P - 1) / P;
    const int s_begin = p * per, s_end = min(K, s_begin + per);
    float acc[NIT][CN];
#pragma unroll
    for (int i = 0; i < NIT; ++i)
#pragma unroll
        for (int e = 0; e < CN; ++e) acc[i][e] = 0.0f;
    u32x4_t ru[NIT], rd[NIT];
    float gj = 0.0f;
    // rows of channel slot s (both matrices) -> registers; all loads are issued before any is used
    auto fetch_rows = [&](int s) {
        const int j = idx[(int64_t)b * K + s];
        gj = gsel[(int64_t)b * K + s];
        const E* urow = wu + (int64_t)j * d;
        const E* drow = wd + (int64_t)j * d;
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int k = i * 64 * CN + lane * CN;
            ru[i] = u32x4_t{0, 0, 0, 0};
            if (k < d) ru[i] = SHARED ? *reinterpret_cast<const u32x4_t*>(urow + k)
                                      : __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(urow + k));
        }
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int k = i * 64 * CN + lane * CN;
            rd[i] = u32x4_t{0, 0, 0, 0};
            if (k < d) rd[i] = SHARED ? *reinterpret_cast<const u32x4_t*>(drow + k)
                                      : __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(drow + k));
        }
    };
    int s = s_begin + wave;
    if (s < s_end) fetch_rows(s);          // in flight while x is staged
    for (int i = threadIdx.x * CN; i < d; i += 512 * CN)
        *reinterpret_cast<u32x4_t*>(xs + i) = *reinterpret_cast<const u32x4_t*>(x + (int64_t)b * d + i);
    __syncthreads();
    while (s < s_end) {
        float dot = 0.0f;
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int k = i * 64 * CN + lane * CN;
            if (k < d) {
                dot = Chunk<E>::dot(ru[i], *reinterpret_cast<const u32x4_t*>(xs + k), dot);
            }
        }
        dot = wave_sum(dot);
        const float zz = silu_f32(gj) * dot;
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            float w[CN];
            Chunk<E>::unpack(rd[i], w);
#pragma unroll
            for (int e = 0; e < CN; ++e) acc[i][e] = fmaf(zz, w[e], acc[i][e]);
        }
        s += NWV;
        if (s < s_end) fetch_rows(s);
    }
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
        const int k = i * 64 * CN + lane * CN;
        if (k < d) {
#pragma unroll
            for (int e = 0; e < CN; ++e) red[wave * d + k + e] = acc[i][e];
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < d; c += 512) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) s += red[w * d + c];
        part[((int64_t)p * B + b) * d + c] = s;
    }
}

// Whole decode step of MoC_{a:8} (a = GA = 1 or 2) in one launch, for up to BT tokens (the host uses it
// for single tokens only: with more tokens per workgroup the separate launches measured faster).  The grouped
// selection is local to 8 consecutive channels, so a workgroup that has computed the gate values of
// a group knows the group's kept channels at once and can fetch their W_up / W_down rows itself: no
// launch boundary between gate, selection and gather.  512 threads; per group
//   gate:   wave w reads row 8q + w of W_gate (prefetched during the previous group) and reduces its
//           dot products with the BT staged tokens;
//   select: after one barrier every thread ranks the 8 x BT gate values (same rule as
//           group_select_kernel) and knows the BT*GA (token, channel) pairs;
//   gather: wave w reads slice w (d/8 elements) of both rows of every pair, together with the next
//           group's gate row; partial dots with x meet in LDS (second barrier); then
//           acc[token][own columns] += SiLU(g) u W_down[j][own columns].
// part[p, b, :] gets the workgroup's partial output (p = blockIdx.x); decode_reduce_kernel sums them.
// Needs d % CN == 0 and d <= 8 * 64 * CN (one 16-byte chunk per lane and slice).
template <class E, int BT, int GA>
__global__ __launch_bounds__(512) void decode_fused_group_kernel(const E* __restrict__ x, const E* __restrict__ wg,
                                                                 const E* __restrict__ wu, const E* __restrict__ wd,
                                                                 int B, int d, int F, int K, int32_t* __restrict__ idx,
                                                                 float* __restrict__ part) {
    constexpr int CN = Chunk<E>::N;
    constexpr int GB = 8, NWV = 8, NE = BT * GA;
    static_assert(GA == 1 || GA == 2, "the ordered pair below covers one or two kept channels");
    constexpr int UN = 8;                       // 16-byte chunks of a gate row per lane
    extern __shared__ __align__(16) unsigned char dec_smem[];
    E* xs = reinterpret_cast<E*>(dec_smem);     // [BT][d]
    __shared__ float gl[2][GB][BT];
    __shared__ float dl[2][NE][NWV];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ngroups = F / GB;
    int q = blockIdx.x;
    u32x4_t raw[UN];
    auto fetch_gate = [&](int qq) {
        const E* wrow = wg + (int64_t)(qq * GB + wave) * d;
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = (u * 64 + lane) * CN;
            raw[u] = u32x4_t{0, 0, 0, 0};
            if (k < d) raw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + k));
        }
    };
    if (q < ngroups) fetch_gate(q);             // in flight while x is staged
    for (int i = tid * CN; i < BT * d; i += 512 * CN) {
        const int b = i / d;
        u32x4_t v = {0, 0, 0, 0};
        if (b < B) v = *reinterpret_cast<const u32x4_t*>(x + i);
        *reinterpret_cast<u32x4_t*>(xs + i) = v;
    }
    __syncthreads();
    const int kslice = (wave * 64 + lane) * CN;  // this thread's columns in the gather stage
    const bool have_slice = kslice < d;
    float acc[BT][CN];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < CN; ++e) acc[b][e] = 0.0f;
    int it = 0;
    for (; q < ngroups; q += gridDim.x, ++it) {
        // ---- gate values of this wave's row for every token
        float ga_[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) ga_[b] = 0.0f;
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = (u * 64 + lane) * CN;
            if (k < d) {
#pragma unroll
                for (int b = 0; b < BT; ++b)
                    ga_[b] = Chunk<E>::dot(raw[u], *reinterpret_cast<const u32x4_t*>(xs + b * d + k), ga_[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const float s = wave_sum(ga_[b]);
            if (lane == 0) gl[it & 1][wave][b] = s;
        }
        __syncthreads();
        // ---- selection (every thread, same result) and the loads that depend on it
        int jsel[NE];
        float gsel[NE];
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float v[GB];
#pragma unroll
            for (int i = 0; i < GB; ++i) v[i] = gl[it & 1][i][b];
            int rank[GB];
            group_ranks<GB>(v, rank);
            // kept channels in ascending order: with GA <= 2 they are the lowest and the highest kept index
            int lo = -1, hi = 0;
#pragma unroll
            for (int i = 0; i < GB; ++i) {
                if (rank[i] < GA) {
                    if (lo < 0) lo = i;
                    hi = i;
                }
            }
            if (lo < 0) lo = 0;                                  // only for non-finite input
            float vlo = v[0], vhi = v[0];
#pragma unroll
            for (int i = 1; i < GB; ++i) {
                vlo = (i == lo) ? v[i] : vlo;
                vhi = (i == hi) ? v[i] : vhi;
            }
            jsel[b * GA] = q * GB + lo;
            gsel[b * GA] = vlo;
            if (GA == 2) {
                jsel[b * GA + 1] = q * GB + hi;
                gsel[b * GA + 1] = vhi;
            }
        }
        if (tid < B * GA) {
            // tid = b * GA + r
#pragma unroll
            for (int e = 0; e < NE; ++e)
                if (tid == e) idx[(int64_t)(e / GA) * K + q * GA + (e % GA)] = jsel[e];
        }
        u32x4_t ru[NE], rd[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            ru[e] = u32x4_t{0, 0, 0, 0};
            rd[e] = u32x4_t{0, 0, 0, 0};
            if (have_slice && e / GA < B) {
                ru[e] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wu + (int64_t)jsel[e] * d + kslice));
                rd[e] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wd + (int64_t)jsel[e] * d + kslice));
            }
        }
        if (q + (int)gridDim.x < ngroups) fetch_gate(q + gridDim.x);     // next group's gate row, in flight with the gather
        // ---- partial dots of the up projection over this wave's slice
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            float dot = 0.0f;
            if (have_slice) {
                dot = Chunk<E>::dot(ru[e], *reinterpret_cast<const u32x4_t*>(xs + (e / GA) * d + kslice), dot);
            }
            dot = wave_sum(dot);
            if (lane == 0) dl[it & 1][e][wave] = dot;
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            float u = 0.0f;
#pragma unroll
            for (int w = 0; w < NWV; ++w) u += dl[it & 1][e][w];
            const float zz = silu_f32(gsel[e]) * u;
            float w[CN];
            Chunk<E>::unpack(rd[e], w);
#pragma unroll
            for (int c = 0; c < CN; ++c) acc[e / GA][c] = fmaf(zz, w[c], acc[e / GA][c]);
        }
    }
    if (have_slice) {
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            if (b < B) {
                float* dst = part + ((int64_t)blockIdx.x * B + b) * d + kslice;
#pragma unroll
                for (int c = 0; c < CN; c += 4)
                    *reinterpret_cast<f32x4_t*>(dst + c) = f32x4_t{acc[b][c], acc[b][c + 1], acc[b][c + 2], acc[b][c + 3]};
            }
        }
    }
}

// y[b, c] = sum_p part[p, b, c] in a fixed order (deterministic).  A 1024-thread workgroup owns 64
// columns; its sixteen wavefronts each sum a sixteenth of the P partials with the loads in flight
// together, and the sixteen sums are combined through LDS.
template <class E>
__global__ __launch_bounds__(1024) void decode_reduce_kernel(const float* __restrict__ part, int P, int64_t n,
                                                             E* __restrict__ y) {
    __shared__ float red[16][64];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * 64 + lane;
    const int per = (P + 15) / 16;
    const int p0 = q * per, p1 = min(P, p0 + per);
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    if (c < n) {
        int p = p0;
        for (; p + 3 < p1; p += 4) {
            const float a0 = part[(int64_t)p * n + c], a1 = part[(int64_t)(p + 1) * n + c];
            const float a2 = part[(int64_t)(p + 2) * n + c], a3 = part[(int64_t)(p + 3) * n + c];
            s0 += a0; s1 += a1; s2 += a2; s3 += a3;
        }
        for (; p < p1; ++p) s0 += part[(int64_t)p * n + c];
    }
    red[q][lane] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (q == 0 && c < n) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += red[w][lane];
        Elem<E>::store(y + c, t);
    }
}

}  // namespace moc
