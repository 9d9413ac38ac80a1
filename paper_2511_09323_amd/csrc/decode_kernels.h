// Decode path (paper section "Accelerated inference"): g = x W_gate over every channel, Top-K per
// token, then u_j = x . W_up[:, j] and y += SiLU(g_j) u_j w_j only for the selected channels j.
// All three weights are channel-major [F, d], so one channel is one contiguous row in each.
//
// The kernels stream weight rows with 16-byte loads, one wavefront per row (or row segment), and
// keep x in LDS.  All are bandwidth-bound; the arithmetic is fp32 FMA on the vector ALU.
#pragma once
#include "common.h"

namespace moc {

template <class E> struct Chunk;   // 16 bytes of E as floats
template <> struct Chunk<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const float* p, float* v) {
        f32x4_t t = *reinterpret_cast<const f32x4_t*>(p);
        v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
    }
};
template <> struct Chunk<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
        u32x4_t t = *reinterpret_cast<const u32x4_t*>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(t[i] << 16);
            v[2 * i + 1] = __uint_as_float(t[i] & 0xFFFF0000u);
        }
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
    for (int i = threadIdx.x * CN; i < BT * d; i += 256 * CN) {
        int b = i / d;
        u32x4_t v = {0, 0, 0, 0};
        if (b < B) v = *reinterpret_cast<const u32x4_t*>(x + i);
        *reinterpret_cast<u32x4_t*>(xs + i) = v;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), nwave = gridDim.x * 4;
    for (int j = wave; j < F; j += nwave) {
        const E* wrow = wg + (int64_t)j * d;
        float acc[BT];
#pragma unroll
        for (int b = 0; b < BT; ++b) acc[b] = 0.0f;
        for (int k = lane * CN; k < d; k += 64 * CN) {
            float w[CN];
            Chunk<E>::load(wrow + k, w);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                float xv[CN];
                Chunk<E>::load(xs + b * d + k, xv);
#pragma unroll
                for (int e = 0; e < CN; ++e) acc[b] = fmaf(w[e], xv[e], acc[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float s = wave_sum(acc[b]);
            if (lane == 0 && b < B) g[(int64_t)b * ldg + j] = s;
        }
    }
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

// y[b, c] = sum_p part[p, b, c], fixed order (deterministic).
template <class E>
__global__ void decode_reduce_kernel(const float* __restrict__ part, int P, int64_t n, E* __restrict__ y) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.0f;
        for (int p = 0; p < P; ++p) s += part[(int64_t)p * n + i];
        Elem<E>::store(y + i, s);
    }
}

}  // namespace moc
