// Row-wise Top-K selection over the fp32 gate (the mask M = TopK(G) of the paper's section
// "Mixture-of-Channels architecture"): exactly K channels per row, the largest signed values,
// equal values ordered by channel index (lower first), -0.0 equal to +0.0.
//
// One workgroup per row.  The row's order-preserving 32-bit keys are parked in LDS while a
// most-significant-digit-first radix select (11 + 11 + 10 bits, LDS histograms) finds the key of
// the K-th largest element; a final ordered pass ranks the selected channels with wavefront
// ballots so that the output is ascending by channel without any sort.
//
// FUSED = true is the training forward: besides idx and the gate values it gathers U at the
// selected channels and writes the dense activation row Z' = SiLU(G) . M . U (Eq. MoC-2), zeros
// on unselected channels and on the padding up to ldz.
#pragma once
#include "common.h"

namespace moc {

constexpr int kTopkBins = 2048;

template <class E> struct TopkArgs {
    const float* g;     // [T, ldg] fp32 gate
    int64_t ldg;
    int F, K;
    int32_t* idx;       // [T, K]
    float* gsel_f32;    // [T, K] or null: selected gate values, fp32
    E* gvals;           // [T, K] or null: selected gate values, E
    // FUSED only:
    const E* u;         // [T, ldu] dense up projection
    int64_t ldu;
    E* uvals;           // [T, K]
    E* zd;              // [T, ldz] dense masked activation
    int64_t ldz;
};

// Exclusive scan of one value per thread across the workgroup, in thread order.
// red must hold NT/64 ints.  Returns the exclusive prefix; total goes to *total.
template <int NT> __device__ __forceinline__ int block_exclusive_scan(int v, int* red, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    if (lane == 63) red[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        int r = red[w];
        if (w < wave) base += r;
        tot += r;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

template <class E, int NT, int VEC, bool FUSED>
__global__ __launch_bounds__(NT) void topk_rows_kernel(TopkArgs<E> a) {
    constexpr int NW = NT / 64;
    constexpr int CHUNK = NT * VEC;
    extern __shared__ __align__(16) unsigned char topk_smem[];
    const int F = a.F, K = a.K;
    const int nchunk = (F + CHUNK - 1) / CHUNK;
    uint32_t* keys = reinterpret_cast<uint32_t*>(topk_smem);           // nchunk * CHUNK
    uint32_t* hist = keys + nchunk * CHUNK;                            // kTopkBins
    int* cnt_gt = reinterpret_cast<int*>(hist + kTopkBins);            // nchunk * NW
    int* cnt_eq = cnt_gt + nchunk * NW;                                // nchunk * NW
    int* red = cnt_eq + nchunk * NW;                                   // NW
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_need;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const float* grow = a.g + row * a.ldg;

    // ---- load the row, build keys
    for (int i = tid; i < kTopkBins; i += NT) hist[i] = 0;
    __syncthreads();
    for (int c = 0; c < nchunk; ++c) {
        const int j0 = c * CHUNK + tid * VEC;
        uint32_t k[VEC];
        if (VEC == 4 && j0 + 3 < F) {
            f32x4_t v = *reinterpret_cast<const f32x4_t*>(grow + j0);
#pragma unroll
            for (int e = 0; e < VEC; ++e) k[e] = float_key(v[e]);
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) k[e] = (j0 + e < F) ? float_key(grow[j0 + e]) : 0u;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            keys[j0 + e] = k[e];
            if (j0 + e < F) atomicAdd(&hist[k[e] >> 21], 1u);
        }
    }
    __syncthreads();

    // ---- three digit passes, most significant first.  After a pass: prefix = the digits fixed so
    //      far of the K-th largest key, need = how many elements are still wanted among those
    //      whose key starts with that prefix.
    uint32_t prefix = 0;
    int need = K;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const int nbins = pass == 2 ? 1024 : 2048;
        if (pass > 0) {
            for (int i = tid; i < kTopkBins; i += NT) hist[i] = 0;
            __syncthreads();
            const int pshift = pass == 1 ? 21 : 10;
            for (int c = 0; c < nchunk; ++c) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int j = c * CHUNK + tid * VEC + e;
                    const uint32_t k = keys[j];
                    if (j < F && (k >> pshift) == prefix) atomicAdd(&hist[(k >> shift) & (nbins - 1)], 1u);
                }
            }
            __syncthreads();
        }
        // descending scan over bins: thread t owns bins [nbins-1 - t*per - (per-1), nbins-1 - t*per]
        const int per = (nbins + NT - 1) / NT;
        int local = 0;
        for (int q = 0; q < per; ++q) {
            int b = nbins - 1 - (tid * per + q);
            if (b >= 0) local += (int)hist[b];
        }
        int total;
        int above = block_exclusive_scan<NT>(local, red, &total);
        if (above < need && above + local >= need) {   // the crossing bin is one of mine
            int run = above;
            for (int q = 0; q < per; ++q) {
                int b = nbins - 1 - (tid * per + q);
                if (b < 0) break;
                int h = (int)hist[b];
                if (run + h >= need) {
                    sh_prefix = (prefix << (pass == 0 ? 0 : (pass == 1 ? 11 : 10))) | (uint32_t)b;
                    sh_need = need - run;
                    break;
                }
                run += h;
            }
        }
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        __syncthreads();
    }
    const uint32_t tau = prefix;   // key of the K-th largest element; `need` of the keys equal to
                                   // tau are selected (lowest channels first), all keys above are.

    // ---- ordered pass 1: per (chunk, wave) counts of keys > tau and keys == tau
    for (int c = 0; c < nchunk; ++c) {
        int ngt = 0, neq = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const int j = c * CHUNK + tid * VEC + e;
            const uint32_t k = keys[j];
            const bool in = j < F;
            ngt += __popcll(__ballot(in && k > tau));
            neq += __popcll(__ballot(in && k == tau));
        }
        if (lane == 0) {
            cnt_gt[c * NW + wave] = ngt;
            cnt_eq[c * NW + wave] = neq;
        }
    }
    __syncthreads();
    // exclusive scan of the two small tables in (chunk, wave) order, by wave 0
    if (wave == 0) {
        const int n = nchunk * NW;
        const int per = (n + 63) / 64;
        int sg = 0, se = 0;
        for (int q = 0; q < per; ++q) {
            int i = lane * per + q;
            if (i < n) { sg += cnt_gt[i]; se += cnt_eq[i]; }
        }
        int ig = sg, ie = se;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            int tg = __shfl_up(ig, o, 64), te = __shfl_up(ie, o, 64);
            if (lane >= o) { ig += tg; ie += te; }
        }
        int rg = ig - sg, re = ie - se;
        for (int q = 0; q < per; ++q) {
            int i = lane * per + q;
            if (i < n) {
                int g0 = cnt_gt[i], e0 = cnt_eq[i];
                cnt_gt[i] = rg; cnt_eq[i] = re;
                rg += g0; re += e0;
            }
        }
    }
    __syncthreads();

    // ---- ordered pass 2: rank and write
    int32_t* idx_row = a.idx + row * K;
    const int64_t ldz_pad = FUSED ? a.ldz : 0;
    const int out_chunks = FUSED ? (int)((ldz_pad + CHUNK - 1) / CHUNK) : nchunk;
    for (int c = 0; c < out_chunks; ++c) {
        const int j0 = c * CHUNK + tid * VEC;
        int gt_before = 0, eq_before = 0;
        uint32_t k[VEC];
        bool isgt[VEC], iseq[VEC];
        if (c < nchunk) {
            gt_before = cnt_gt[c * NW + wave];
            eq_before = cnt_eq[c * NW + wave];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                k[e] = keys[j0 + e];
                const bool in = j0 + e < F;
                isgt[e] = in && k[e] > tau;
                iseq[e] = in && k[e] == tau;
                gt_before += mbcnt(__ballot(isgt[e]));
                eq_before += mbcnt(__ballot(iseq[e]));
            }
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) { isgt[e] = iseq[e] = false; k[e] = 0; }
        }
        float z[VEC];
        float uu[VEC];
        if (FUSED) {
            const E* urow = a.u + row * a.ldu;
#pragma unroll
            for (int e = 0; e < VEC; ++e) uu[e] = (j0 + e < F) ? Elem<E>::load(urow + j0 + e) : 0.0f;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const bool sel = isgt[e] || (iseq[e] && eq_before < need);
            z[e] = 0.0f;
            if (sel) {
                const int slot = gt_before + min(eq_before, need);
                const float g = key_float(k[e]);
                idx_row[slot] = j0 + e;
                if (a.gsel_f32) a.gsel_f32[row * K + slot] = g;
                if (a.gvals) Elem<E>::store(a.gvals + row * K + slot, g);
                if (FUSED) {
                    Elem<E>::store(a.uvals + row * K + slot, uu[e]);
                    z[e] = silu_f32(g) * uu[e];
                }
            }
            gt_before += isgt[e] ? 1 : 0;
            eq_before += iseq[e] ? 1 : 0;
        }
        if (FUSED) {
            E* zrow = a.zd + row * a.ldz;
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                if (j0 + e < ldz_pad) Elem<E>::store(zrow + j0 + e, z[e]);
        }
    }
}

inline size_t topk_lds_bytes(int F, int NT, int VEC) {
    const int chunk = NT * VEC;
    const int nchunk = (F + chunk - 1) / chunk;
    return (size_t)nchunk * chunk * 4 + kTopkBins * 4 + (size_t)2 * nchunk * (NT / 64) * 4 + (NT / 64) * 4;
}

}  // namespace moc
