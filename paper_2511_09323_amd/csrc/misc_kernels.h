// Small bandwidth-bound kernels around the GEMMs: the selection bit mask for the backward,
// RMSNorm and the residual add.
#pragma once
#include "common.h"

namespace moc {

// From idx[T, K] (ascending per row) build the selection bit mask maskw[T, nw] (bit j % 32 of word
// j / 32) and pref[T, nw], the number of selected channels before each word.  One workgroup per
// row.  Entries of idx outside [0, F) are ignored.
__global__ __launch_bounds__(256) void build_mask_kernel(const int32_t* __restrict__ idx, int K, int F, int nw,
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

// RMSNorm of one row per workgroup: out = x / sqrt(mean(x^2) + eps) * gain.
template <class E>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const E* __restrict__ h, const E* __restrict__ gain, float eps,
                                                      int d, E* __restrict__ out) {
    __shared__ float red[4];
    const int64_t t = blockIdx.x;
    const E* x = h + t * d;
    float ss = 0.0f;
    for (int i = threadIdx.x; i < d; i += 256) {
        float v = Elem<E>::load(x + i);
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256)
        Elem<E>::store(out + t * d + i, Elem<E>::load(x + i) * inv * Elem<E>::load(gain + i));
}

template <class E> __global__ void residual_add_kernel(E* __restrict__ h, const E* __restrict__ y, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        Elem<E>::store(h + i, Elem<E>::load(h + i) + Elem<E>::load(y + i));
}

}  // namespace moc
