// Generic fp32-accumulate tiled GEMM, any element type and any shape: the fp32 path of the layer
// and the fallback for bf16 shapes the MFMA kernel does not take.
//
//   C[m, n] = sum_k A[m, k] B[n, k]  (+ sum_k A2[m, k] B2[n, k])      "NT": both operands are
// row-major with the contraction index contiguous.  64x64 output tile per 256-thread workgroup,
// 16-deep k slices staged in LDS, a 4x4 register block per thread.
#pragma once
#include "common.h"

namespace moc {

template <class E> struct GemmOperands {
    const E* A;
    const E* B;
    int64_t lda, ldb;
    int Kc;
    const E* A2;
    const E* B2;
    int64_t lda2, ldb2;
    int Kc2;
};

template <class E, class Epi>
__global__ __launch_bounds__(256) void gemm_nt_generic_kernel(GemmOperands<E> op, int M, int N, Epi epi) {
    constexpr int BT = 64, BK = 16;
    __shared__ float As[BK][BT + 4];
    __shared__ float Bs[BK][BT + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    const int lrow = tid / 4, lk = (tid % 4) * 4;
    float acc[4][4] = {};
    for (int seg = 0; seg < 2; ++seg) {
        const E* A = seg ? op.A2 : op.A;
        const E* B = seg ? op.B2 : op.B;
        const int64_t lda = seg ? op.lda2 : op.lda, ldb = seg ? op.ldb2 : op.ldb;
        const int Kc = seg ? op.Kc2 : op.Kc;
        if (A == nullptr) continue;
        for (int k0 = 0; k0 < Kc; k0 += BK) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int k = k0 + lk + e;
                int am = m0 + lrow, bn = n0 + lrow;
                As[lk + e][lrow] = (am < M && k < Kc) ? Elem<E>::load(A + (int64_t)am * lda + k) : 0.0f;
                Bs[lk + e][lrow] = (bn < N && k < Kc) ? Elem<E>::load(B + (int64_t)bn * ldb + k) : 0.0f;
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
        int m = m0 + tm + i;
        if (m < M) epi.store4(m, n0 + tn, acc[i]);
    }
}

template <class E, class Epi>
inline void launch_gemm_nt_generic(const GemmOperands<E>& op, int M, int N, const Epi& epi, hipStream_t st) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL((gemm_nt_generic_kernel<E, Epi>), grid, dim3(256), 0, st, op, M, N, epi);
}

}  // namespace moc
