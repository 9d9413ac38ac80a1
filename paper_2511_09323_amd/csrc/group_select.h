// Grouped Top-K of MoC_{a:b} (paper item "MoC with structured 2:8 sparsity"; a:b as defined before
// Theorem 1): in every contiguous group of b channels the a largest signed gate values are kept,
// equal values ordered by channel index (lower first), -0.0 equal to +0.0.
//
// The decision is local to a group, so one thread owns one group: it loads the b fp32 gate values,
// ranks them by pairwise comparison and writes the kept channels to slots q*a .. q*a+a-1 of the
// row, which therefore ascends by channel.  Streaming, HBM-bound.
//
// FUSED = true is the training forward (same outputs as the row-wide kernel in topk.h): idx, the
// gate and up values at the kept channels, and the dense row Z' = SiLU(G) . M . U (Eq. MoC-2) with
// zeros on dropped channels and on the padding up to ldz.
#pragma once
#include "common.h"
#include "topk.h"

namespace moc {

// rank[i] = number of group members that precede member i in the order (value descending, channel
// ascending).  Member i is kept iff rank[i] < a.  Float comparison makes -0.0 equal +0.0.
template <int GB> __device__ __forceinline__ void group_ranks(const float (&v)[GB], int (&rank)[GB]) {
#pragma unroll
    for (int i = 0; i < GB; ++i) {
        int r = 0;
#pragma unroll
        for (int j = 0; j < GB; ++j) {
            if (j < i) r += (v[j] >= v[i]) ? 1 : 0;
            if (j > i) r += (v[j] > v[i]) ? 1 : 0;
        }
        rank[i] = r;
    }
}

template <class E> __device__ __forceinline__ void load_vec4_any(const E* p, float v[4]);
template <> __device__ __forceinline__ void load_vec4_any<float>(const float* p, float v[4]) {
    const f32x4_t t = *reinterpret_cast<const f32x4_t*>(p);
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
}
template <> __device__ __forceinline__ void load_vec4_any<bf16_t>(const bf16_t* p, float v[4]) {
    const u32x2_t t = *reinterpret_cast<const u32x2_t*>(p);
    v[0] = __uint_as_float(t[0] << 16); v[1] = __uint_as_float(t[0] & 0xFFFF0000u);
    v[2] = __uint_as_float(t[1] << 16); v[3] = __uint_as_float(t[1] & 0xFFFF0000u);
}

template <class E, int GB, bool FUSED>
__global__ __launch_bounds__(256) void group_select_kernel(TopkArgs<E> a, int T, int ga, int vec_ok) {
    static_assert(GB == 4 || GB == 8 || GB == 16, "group size");
    const int gpr = FUSED ? (int)(a.ldz / GB) : a.F / GB;               // groups per row, padding included
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= (int64_t)T * gpr) return;
    const int row = (int)(gid / gpr), q = (int)(gid - (int64_t)row * gpr);
    const int c0 = q * GB;
    if (FUSED && c0 >= a.F) {                                            // padding of the dense row
        const float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int i = 0; i < GB; i += 4) store_vec4_any<E>(a.zd + (int64_t)row * a.ldz + c0 + i, z);
        return;
    }
    float v[GB];
    const float* gp = a.g + (int64_t)row * a.ldg + c0;
    if (vec_ok) {
#pragma unroll
        for (int i = 0; i < GB; i += 4) {
            const f32x4_t t = *reinterpret_cast<const f32x4_t*>(gp + i);
            v[i] = t[0]; v[i + 1] = t[1]; v[i + 2] = t[2]; v[i + 3] = t[3];
        }
    } else {
#pragma unroll
        for (int i = 0; i < GB; ++i) v[i] = gp[i];
    }
    float u[GB];
    if (FUSED) {
#pragma unroll
        for (int i = 0; i < GB; i += 4) load_vec4_any<E>(a.u + (int64_t)row * a.ldu + c0 + i, u + i);   // ldu, ldz: multiples of 64
    }
    int rank[GB];
    group_ranks<GB>(v, rank);
    const int64_t out0 = (int64_t)row * a.K + (int64_t)q * ga;
    int r = 0;
    float z[GB];
#pragma unroll
    for (int i = 0; i < GB; ++i) {
        const bool keep = rank[i] < ga && r < ga;        // r < ga only matters for non-finite input
        if (FUSED) z[i] = keep ? silu_f32(v[i]) * u[i] : 0.0f;
        if (keep) {
            a.idx[out0 + r] = c0 + i;
            if (a.gsel_f32) a.gsel_f32[out0 + r] = v[i];
            if (a.gvals) Elem<E>::store(a.gvals + out0 + r, v[i]);
            if (FUSED) Elem<E>::store(a.uvals + out0 + r, u[i]);
            ++r;
        }
    }
    if (FUSED) {
#pragma unroll
        for (int i = 0; i < GB; i += 4) store_vec4_any<E>(a.zd + (int64_t)row * a.ldz + c0 + i, z + i);
    }
}

}  // namespace moc
