// Epilogue functors shared by the generic and the MFMA GEMM kernels.
//
// A GEMM kernel hands over accumulators as groups of four consecutive columns of one row:
//     epi.store4(m, n0, v)      with n0 % 4 == 0, m < M guaranteed by the caller,
// and the functor guards the column range itself.  For the MoC layer the GEMM row index m is
// always a token (or a weight row) and n the other dimension, as noted per functor.
#pragma once
#include "common.h"

namespace moc {

template <class T> __device__ __forceinline__ void store_vec4(T* p, const float v[4]);
template <> __device__ __forceinline__ void store_vec4<float>(float* p, const float v[4]) {
    *reinterpret_cast<f32x4_t*>(p) = f32x4_t{v[0], v[1], v[2], v[3]};
}
template <> __device__ __forceinline__ void store_vec4<bf16_t>(bf16_t* p, const float v[4]) {
    *reinterpret_cast<u32x2_t*>(p) = u32x2_t{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
}

// C[m, n] = acc, row-major with leading dimension ldc.  Columns n >= N are dropped unless
// pad_to > N, in which case columns in [N, pad_to) are written as zero (keeps the padding of a
// later contraction operand clean).
template <class OutT> struct EpiStore {
    OutT* C;
    int64_t ldc;
    int N;
    int pad_to;
    __device__ __forceinline__ void store4(int m, int n0, const float v[4]) const {
        OutT* row = C + (int64_t)m * ldc;
        if (n0 + 3 < N && (ldc & 3) == 0) {
            store_vec4<OutT>(row + n0, v);
        } else if (n0 < N || n0 < pad_to) {      // (a tile that hangs over the edge has whole wavefronts out here)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int n = n0 + r;
                if (n < N) Elem<OutT>::store(row + n, v[r]);
                else if (n < pad_to) Elem<OutT>::store(row + n, 0.0f);
            }
        }
    }
};

// Dense SwiGLU forward, second GEMM (m = token, n = channel): acc = U.  Reads the stored gate,
// writes u_save and the dense activation Z = SiLU(G) . U (Eq. FFN-2) padded with zeros to ldz.
template <class E> struct EpiSwigluAct {
    const E* g_save;  // [T, F]
    E* u_save;        // [T, F]
    E* zd;            // [T, ldz]
    int F;
    int64_t ldz;
    __device__ __forceinline__ void store4(int m, int n0, const float v[4]) const {
        float z[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int n = n0 + r;
            z[r] = 0.0f;
            if (n < F) {
                float u = Elem<E>::round(v[r]);
                float g = Elem<E>::load(g_save + (int64_t)m * F + n);
                Elem<E>::store(u_save + (int64_t)m * F + n, u);
                z[r] = silu_f32(g) * u;
            }
        }
        if (n0 < ldz) store_vec4<E>(zd + (int64_t)m * ldz + n0, z);
    }
};

// Backward, first GEMM (m = token t, n = channel j): acc = dz'[t, j] = dy_t . W_down[j, :]
// (Eq. bp-1).  On selected channels it recomputes s, z' from the stored g, u and forms du, dg
// (Eqs. bp-2, bp-3); elsewhere everything is zero.  It writes the dense [T, ldf] operands the
// remaining GEMMs contract over: z' (for dW_down), dg and du (for dW_gate, dW_up and dX), zero on
// unselected channels and on the padding columns [F, ldf).
//   MoC:   selection comes from a bit mask maskw[T, nw] (bit j%32 of word j/32) with the number
//          of selected channels before each word in pref[T, nw]; stored values are [T, K].
//   dense: every channel is selected and the stored values are [T, F].
template <class E, bool DENSE> struct EpiBwdPointwise {
    const uint32_t* maskw;
    const uint16_t* pref;
    int nw;
    const E* gvals;
    const E* uvals;
    int K;  // row length of gvals / uvals (F when DENSE)
    E* zd;
    E* dgd;
    E* dud;  // [T, ldf]
    int F;
    int64_t ldf;
    // Branch-free on purpose: the stored values of all four channels are loaded unconditionally
    // (clamped slot, always a valid address) and masked afterwards, so the loads of several calls
    // can be in flight together instead of forming a chain of dependent, predicated gathers.
    __device__ __forceinline__ void store4(int t, int j0, const float v[4]) const {
        if (j0 >= ldf) return;
        float z[4], dg[4], du[4];
        uint32_t bits;
        int slot;
        if (DENSE) {
            bits = 0xFu;
            slot = j0;
        } else {
            const int wi = j0 >> 5, sh = j0 & 31;
            const uint32_t w = maskw[(int64_t)t * nw + wi];
            bits = (w >> sh) & 0xFu;
            slot = (int)pref[(int64_t)t * nw + wi] + __popc(w & ((1u << sh) - 1u));
        }
        const E* grow = gvals + (int64_t)t * K;
        const E* urow = uvals + (int64_t)t * K;
        float g[4], u[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int sl = min(slot + __popc(bits & ((1u << r) - 1u)), K - 1);
            g[r] = Elem<E>::load(grow + sl);
            u[r] = Elem<E>::load(urow + sl);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool on = j0 + r < F && ((bits >> r) & 1u);
            float zz, gg, uu;
            moc_bwd_pointwise(g[r], u[r], v[r], zz, gg, uu);
            z[r] = on ? zz : 0.0f;
            dg[r] = on ? gg : 0.0f;
            du[r] = on ? uu : 0.0f;
        }
        store_vec4<E>(zd + (int64_t)t * ldf + j0, z);
        store_vec4<E>(dgd + (int64_t)t * ldf + j0, dg);
        store_vec4<E>(dud + (int64_t)t * ldf + j0, du);
    }
};

}  // namespace moc
