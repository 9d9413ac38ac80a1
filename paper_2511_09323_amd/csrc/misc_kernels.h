// Small bandwidth-bound kernels around the GEMMs: the backward's pointwise/expansion step, the
// selection bit mask of its fallback, RMSNorm and the residual add.
#pragma once
#include "common.h"

namespace moc {

// From idx[T, K] (ascending per row) build the selection bit mask maskw[T, nw] (bit j % 32 of word
// j / 32) and pref[T, nw], the number of selected channels before each word.  One workgroup per
// row.  Entries of idx outside [0, F) are ignored.
static __global__ __launch_bounds__(256) void build_mask_kernel(const int32_t* __restrict__ idx, int K, int F, int nw,
                                                         uint32_t* __restrict__ maskw, uint16_t* __restrict__ pref) {
    extern __shared__ uint32_t mask_smem[];   // nw words + 4 ints
    uint32_t* words = mask_smem;
    int* red = reinterpret_cast<int*>(mask_smem + nw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t t = blockIdx.x;
    for (int i = tid; i < nw; i += 256) words[i] = 0;
    __syncthreads();
    for (int s = tid; s < K; s += 256) {
        int j = idx[t * K + s];
        if (j >= 0 && j < F) atomicOr(&words[j >> 5], 1u << (j & 31));
    }
    __syncthreads();
    const int per = (nw + 255) / 256;
    int local = 0;
    for (int q = 0; q < per; ++q) {
        int i = tid * per + q;
        if (i < nw) local += __popc(words[i]);
    }
    int inc = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int v = __shfl_up(inc, o, 64);
        if (lane >= o) inc += v;
    }
    if (lane == 63) red[wave] = inc;
    __syncthreads();
    int run = inc - local;
    for (int w = 0; w < wave; ++w) run += red[w];
    for (int q = 0; q < per; ++q) {
        int i = tid * per + q;
        if (i < nw) {
            uint32_t w = words[i];
            maskw[t * nw + i] = w;
            pref[t * nw + i] = (uint16_t)run;
            run += __popc(w);
        }
    }
}

// Backward pointwise step on the compact stored set, expanded to the dense operands of the
// weight-gradient and dX GEMMs.  One workgroup per token row t: for every stored slot s with channel
// j = idx[t, s] it takes dz' = dzd[t, j] (the dense dD W_down^T product), recomputes s = SiLU(g),
// z' = s u and forms du = s dz', dg = u dz' SiLU'(g) (Eqs. bp-1 ... bp-3, S' and Z' recomputed from
// the stored G.M as in MoC+GCP).  The three rows z', dg, du are assembled in LDS -- zero everywhere
// except at the K selected channels -- and streamed out with 16-byte stores, padding included.
template <class E>
__global__ __launch_bounds__(256) void bwd_expand_kernel(const int32_t* __restrict__ idx, const E* __restrict__ gvals,
                                                         const E* __restrict__ uvals, const E* __restrict__ dzd,
                                                         int K, int F, int64_t ldf, E* __restrict__ zd,
                                                         E* __restrict__ dgd, E* __restrict__ dud) {
    extern __shared__ __align__(16) unsigned char exp_smem[];
    E* rz = reinterpret_cast<E*>(exp_smem);
    E* rg = rz + ldf;
    E* ru = rg + ldf;
    const int tid = threadIdx.x;
    const int64_t t = blockIdx.x;
    constexpr int PER16 = 16 / sizeof(E);
    const int nvec = (int)(3 * ldf) / PER16;
    for (int i = tid; i < nvec; i += 256) reinterpret_cast<u32x4_t*>(exp_smem)[i] = u32x4_t{0, 0, 0, 0};
    __syncthreads();
    const E* dzrow = dzd + t * ldf;
    for (int s = tid; s < K; s += 256) {
        const int j = idx[t * K + s];
        if (j < 0 || j >= F) continue;
        const float g = Elem<E>::load(gvals + t * K + s);
        const float u = Elem<E>::load(uvals + t * K + s);
        const float dz = Elem<E>::load(dzrow + j);
        float z, dg, du;
        moc_bwd_pointwise(g, u, dz, z, dg, du);
        Elem<E>::store(rz + j, z);
        Elem<E>::store(rg + j, dg);
        Elem<E>::store(ru + j, du);
    }
    __syncthreads();
    const int rowvec = (int)ldf / PER16;
    u32x4_t* oz = reinterpret_cast<u32x4_t*>(zd + t * ldf);
    u32x4_t* og = reinterpret_cast<u32x4_t*>(dgd + t * ldf);
    u32x4_t* ou = reinterpret_cast<u32x4_t*>(dud + t * ldf);
    const u32x4_t* lz = reinterpret_cast<const u32x4_t*>(rz);
    const u32x4_t* lg = reinterpret_cast<const u32x4_t*>(rg);
    const u32x4_t* lu = reinterpret_cast<const u32x4_t*>(ru);
    for (int i = tid; i < rowvec; i += 256) {
        oz[i] = lz[i];
        og[i] = lg[i];
        ou[i] = lu[i];
    }
}

// 16 bytes of E as floats and back.
template <class E> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(u32x4_t t, float* v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(t[i]);
    }
    static __device__ __forceinline__ u32x4_t pack(const float* v) {
        return u32x4_t{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
    }
};
template <> struct Vec16<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(u32x4_t t, float* v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(t[i] << 16);
            v[2 * i + 1] = __uint_as_float(t[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ u32x4_t pack(const float* v) {
        return u32x4_t{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
    }
};

// RMSNorm of one row per workgroup: out = x / sqrt(mean(x^2) + eps) * gain.
// VEC: rows are read once with 16-byte loads and kept in registers (needs d a multiple of the
// 16-byte element count, d <= 256 * NV elements per 16 bytes, and 16-byte aligned pointers);
// otherwise element by element, reading the row twice.
template <class E, bool VEC, int NV>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const E* __restrict__ h, const E* __restrict__ gain, float eps,
                                                      int d, E* __restrict__ out) {
    __shared__ float red[4];
    const int64_t t = blockIdx.x;
    const E* x = h + t * d;
    float ss = 0.0f;
    constexpr int CN = Vec16<E>::N;
    u32x4_t raw[NV];
    if (VEC) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int i = (u * 256 + threadIdx.x) * CN;
            raw[u] = u32x4_t{0, 0, 0, 0};
            if (i < d) raw[u] = *reinterpret_cast<const u32x4_t*>(x + i);
            float v[CN];
            Vec16<E>::unpack(raw[u], v);
#pragma unroll
            for (int e = 0; e < CN; ++e) ss = fmaf(v[e], v[e], ss);
        }
    } else {
        for (int i = threadIdx.x; i < d; i += 256) {
            float v = Elem<E>::load(x + i);
            ss += v * v;
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    if (VEC) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int i = (u * 256 + threadIdx.x) * CN;
            if (i < d) {
                float v[CN], g[CN];
                Vec16<E>::unpack(raw[u], v);
                Vec16<E>::unpack(*reinterpret_cast<const u32x4_t*>(gain + i), g);
#pragma unroll
                for (int e = 0; e < CN; ++e) v[e] = v[e] * inv * g[e];
                *reinterpret_cast<u32x4_t*>(out + t * d + i) = Vec16<E>::pack(v);
            }
        }
    } else {
        for (int i = threadIdx.x; i < d; i += 256)
            Elem<E>::store(out + t * d + i, Elem<E>::load(x + i) * inv * Elem<E>::load(gain + i));
    }
}

// h <- h + y, element-wise.  VEC: 16 bytes per lane and step (n a multiple of the 16-byte element
// count, 16-byte aligned pointers).
template <class E, bool VEC> __global__ void residual_add_kernel(E* __restrict__ h, const E* __restrict__ y, int64_t n) {
    if (VEC) {
        constexpr int CN = Vec16<E>::N;
        const int64_t nv = n / CN;
        for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < nv; i += (int64_t)gridDim.x * blockDim.x) {
            float a[CN], b[CN];
            Vec16<E>::unpack(*reinterpret_cast<const u32x4_t*>(h + i * CN), a);
            Vec16<E>::unpack(*reinterpret_cast<const u32x4_t*>(y + i * CN), b);
#pragma unroll
            for (int e = 0; e < CN; ++e) a[e] += b[e];
            *reinterpret_cast<u32x4_t*>(h + i * CN) = Vec16<E>::pack(a);
        }
    } else {
        for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
            Elem<E>::store(h + i, Elem<E>::load(h + i) + Elem<E>::load(y + i));
    }
}

}  // namespace moc
