// GEMM problem description shared by both GEMM kernels, and the generic fp32-accumulate tiled
// kernel: any element type, any shape, any alignment -- the fp32 path of the layer and the
// fallback for bf16 problems the MFMA kernel does not take.
//
//   C[m, n] = sum_k A(m, k) B(n, k)  (+ the same over a second pointer pair: "segment 1")
//
// An operand is either k-contiguous (element (r, k) at p[r * ld + k]) or k-major (element (r, k)
// at p[k * ld + r]).
#pragma once
#include "common.h"

namespace moc {

template <class E> struct GemmOperand {
    const E* p;     // segment 0
    const E* p2;    // segment 1, or null
    int64_t ld;     // leading dimension in elements, both segments
    int ext;        // k-major only: number of readable columns r (>= rows used, multiple of 8 for MFMA)
    bool km;        // k-major layout
    __host__ __device__ const E* seg(int s) const { return s ? p2 : p; }
};

template <class E> struct GemmProblem {
    GemmOperand<E> A, B;
    int M, N;
    int Kc, Kc2;    // contraction lengths of segment 0 and 1 (Kc2 = 0: single segment)
    bool kc_zero_padded;   // the k-contiguous operand holds zeros from Kc up to the next multiple of 32
};

template <class E> inline GemmOperand<E> kc_operand(const E* p, int64_t ld, const E* p2 = nullptr) {
    return GemmOperand<E>{p, p2, ld, 0, false};
}
template <class E> inline GemmOperand<E> km_operand(const E* p, int64_t ld, int ext, const E* p2 = nullptr) {
    return GemmOperand<E>{p, p2, ld, ext, true};
}

template <class E>
__device__ __forceinline__ float gemm_element(const GemmOperand<E>& o, int seg, int r, int k) {
    const E* p = o.seg(seg);
    return Elem<E>::load(o.km ? p + (int64_t)k * o.ld + r : p + (int64_t)r * o.ld + k);
}

// 64x64 output tile per 256-thread workgroup, 16-deep k slices in LDS, 4x4 register block per thread.
template <class E, class Epi>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmProblem<E> pr, Epi epi) {
    constexpr int BT = 64, BK = 16;
    __shared__ float As[BK][BT + 4];
    __shared__ float Bs[BK][BT + 4];
    const int tid = threadIdx.x;
    const int M = pr.M, N = pr.N;
    const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    const int lrow = tid / 4, lk = (tid % 4) * 4;
    float acc[4][4] = {};
    for (int seg = 0; seg < 2; ++seg) {
        const int Kc = seg ? pr.Kc2 : pr.Kc;
        if (Kc == 0) continue;
        for (int k0 = 0; k0 < Kc; k0 += BK) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = k0 + lk + e;
                const int am = m0 + lrow, bn = n0 + lrow;
                As[lk + e][lrow] = (am < M && k < Kc) ? gemm_element(pr.A, seg, am, k) : 0.0f;
                Bs[lk + e][lrow] = (bn < N && k < Kc) ? gemm_element(pr.B, seg, bn, k) : 0.0f;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < BK; ++k) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) { a[i] = As[k][tm + i]; b[i] = Bs[k][tn + i]; }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + tm + i;
        if (m < M) epi.store4(m, n0 + tn, acc[i]);
    }
}

template <class E, class Epi>
inline void launch_gemm_generic(const GemmProblem<E>& pr, const Epi& epi, hipStream_t st) {
    dim3 grid((pr.N + 63) / 64, (pr.M + 63) / 64);
    hipLaunchKernelGGL((gemm_generic_kernel<E, Epi>), grid, dim3(256), 0, st, pr, epi);
}

}  // namespace moc
