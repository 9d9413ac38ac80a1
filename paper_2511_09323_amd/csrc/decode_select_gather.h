// Row-wide decode after the gate projection in one launch (paper section "Accelerated inference": the Top-K
// mask of a token, then only the selected columns of W_up and rows of W_down).
//
// Workgroup (p, b) serves token b and the p-th range of channels.  It reads the token's whole fp32 gate row
// (44 KB at d_ffn = 11008, from L2 or the Infinity Cache) and finds the row's exact Top-K threshold by itself --
// every workgroup of a token repeats that search, which costs each of them the same few microseconds one
// workgroup alone would need and saves a launch boundary plus the single-workgroup selection kernel.  Knowing the
// threshold (key, tie cut), it picks the selected channels of its own range, counts the selected channels below
// the range (their number is where its part of idx[b] starts, so idx comes out ascending without any exchange
// between workgroups), and gathers: a wavefront owns a channel at a time, has its W_up and W_down rows in flight
// together, forms z' = SiLU(g) (x . w_up) and accumulates z' w_down.  part[p, b, :] gets the workgroup's partial
// output; decode_reduce_kernel sums the P partials in a fixed order.
//
// Measured at the 7B shape (d 4096, d_ffn 11008, K 1376, cold weights): the launch takes 27 us where the selection
// kernel and the gather take 11 + 15 us, and the call 46 / 62 / 80 us against 43 / 58 / 81 us for 1 / 4 / 16 tokens: the
// search is a chain of dependent steps that eight wavefronts do no faster than the selection kernel's sixteen, and the
// saved launch boundary does not pay for it.  (The same search as a selection kernel of its own, 1024 threads per
// token, takes 14 us against 11 us for the digit passes of the training Top-K kernel.)  The library therefore uses
// this kernel only on request (MOC_DECODE_SELECT_GATHER=1).
//
// Same decision rule as everywhere in the library: fp32 gate values, larger first, ties to the lower channel,
// -0 = +0.  512 threads; needs d <= 64 * (16 / sizeof(E)) * NIT, F <= NCH * 2048 and ceil(F / P) <= 2048.
#pragma once
#include "common.h"
#include "decode_kernels.h"
#include "decode_persist.h"

namespace moc {

constexpr int kDsgMaxRange = 2048;     // channels per workgroup range: one wavefront scans its 64 bitmap words

// LDS: x [d] of E | union of (selection scratch, bitmap, gate values and list of the range) and (8 x d fp32 partials)
template <class E> inline size_t decode_select_gather_lds(int d) {
    const size_t sel = kDecSelLds + 64 * 4 + (size_t)kDsgMaxRange * 8;
    const size_t red = (size_t)8 * d * sizeof(float);
    return round_up_sz((size_t)d * sizeof(E), 16) + (sel > red ? sel : red);
}

template <class E, int NIT, int NCH>
__global__ __launch_bounds__(512) void decode_select_gather_kernel(const E* __restrict__ x, const E* __restrict__ wu,
                                                                   const E* __restrict__ wd, const float* __restrict__ g,
                                                                   int64_t ldg, int F, int d, int K, int P, int B,
                                                                   int32_t* __restrict__ idx, float* __restrict__ part) {
    constexpr int NT = 512, CN = Chunk<E>::N, NWV = 8, CHUNK = NT * 4;
    extern __shared__ __align__(16) unsigned char dec_smem[];
    E* xs = reinterpret_cast<E*>(dec_smem);
    unsigned char* area = dec_smem + (((size_t)d * sizeof(E) + 15) & ~(size_t)15);
    float* red = reinterpret_cast<float*>(area);                              // [NWV][d], used last
    uint32_t* bitmap = reinterpret_cast<uint32_t*>(area + kDecSelLds);        // [64]
    float* gl = reinterpret_cast<float*>(bitmap + 64);                        // [range] gate value by channel offset
    int* list = reinterpret_cast<int*>(gl + kDsgMaxRange);                    // [range] selected channels, ascending
    __shared__ int sh_below[NWV];
    __shared__ int sh_n;
    int p, b;
    if (B > 1 && P % 8 == 0) {          // the workgroups of one range on one XCD: rows that several tokens selected meet in its L2
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        p = xcd + 8 * (slot / B);
        b = slot % B;
    } else {
        p = blockIdx.x / B;
        b = blockIdx.x % B;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- the token's gate row as keys in registers (channels past F get keys below every finite key)
    const float* grow = g + (int64_t)b * ldg;
    const uint32_t pad_key = (uint32_t)(lane & 3) << 21;
    uint32_t key[NCH][4];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int j0 = c * CHUNK + tid * 4;
        if (j0 + 3 < F) {
            const f32x4_t v = *reinterpret_cast<const f32x4_t*>(grow + j0);
#pragma unroll
            for (int e = 0; e < 4; ++e) key[c][e] = float_key(v[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) key[c][e] = (j0 + e < F) ? float_key(grow[j0 + e]) : pad_key;
        }
    }
    for (int i = tid * CN; i < d; i += NT * CN)
        *reinterpret_cast<u32x4_t*>(xs + i) = *reinterpret_cast<const u32x4_t*>(x + (int64_t)b * d + i);
    if (tid < 64) bitmap[tid] = 0u;

    // ---- exact threshold of the row (the histogram search; rows with too many equal keys take the general one)
    bool ok = false;
    TopkThreshold thr = dec_select_keys<NT, NCH>(key, F, K, area, &ok);
    if (!ok) thr = topk_keys_general<NT, NCH>(key, F, K);

    // ---- my range: selected channels into a bitmap (ascending order falls out of it), their gate values beside
    const int per = (F + P - 1) / P;
    const int c0 = p * per, c1 = min(F, c0 + per);
    int below = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = c * CHUNK + tid * 4 + e;
            if (j < F && topk_member(key[c][e], j, thr)) {
                if (j < c0) ++below;
                else if (j < c1) {
                    atomicOr(&bitmap[(j - c0) >> 5], 1u << ((j - c0) & 31));
                    gl[j - c0] = key_float(key[c][e]);
                }
            }
        }
    below = (int)wave_sum((float)below);                   // exact: counts are far below 2^24
    if (lane == 0) sh_below[wave] = below;
    __syncthreads();
    if (wave == 0) {
        uint32_t w = bitmap[lane];
        const int cnt = __popc(w);
        int inc = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o, 64);
            if (lane >= o) inc += t;
        }
        int at = inc - cnt;
        while (w) {
            const int bit = __ffs(w) - 1;
            list[at++] = c0 + lane * 32 + bit;
            w &= w - 1;
        }
        if (lane == 63) sh_n = inc;
    }
    __syncthreads();
    const int n = sh_n;
    if (idx) {
        int off = 0;
#pragma unroll
        for (int w = 0; w < NWV; ++w) off += sh_below[w];
        for (int i = tid; i < n; i += NT)
            if (off + i < K) idx[(int64_t)b * K + off + i] = list[i];
    }

    // ---- gather
    float acc[NIT][CN];
#pragma unroll
    for (int i = 0; i < NIT; ++i)
#pragma unroll
        for (int e = 0; e < CN; ++e) acc[i][e] = 0.0f;
    u32x4_t ru[NIT], rd[NIT];
    float gj = 0.0f;
    auto fetch_rows = [&](int s) {
        const int j = list[s];
        gj = gl[j - c0];
        const E* urow = wu + (int64_t)j * d;
        const E* drow = wd + (int64_t)j * d;
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int k = i * 64 * CN + lane * CN;
            ru[i] = u32x4_t{0, 0, 0, 0};
            if (k < d) ru[i] = (B > 1) ? *reinterpret_cast<const u32x4_t*>(urow + k)
                                       : __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(urow + k));
        }
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int k = i * 64 * CN + lane * CN;
            rd[i] = u32x4_t{0, 0, 0, 0};
            if (k < d) rd[i] = (B > 1) ? *reinterpret_cast<const u32x4_t*>(drow + k)
                                       : __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(drow + k));
        }
    };
    int s = wave;
    if (s < n) fetch_rows(s);
    while (s < n) {
        float dot = 0.0f;
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int k = i * 64 * CN + lane * CN;
            if (k < d) dot = Chunk<E>::dot(ru[i], *reinterpret_cast<const u32x4_t*>(xs + k), dot);
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
        if (s < n) fetch_rows(s);
    }
    __syncthreads();                    // list and gl have been read by every wavefront; red takes their place
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
        const int k = i * 64 * CN + lane * CN;
        if (k < d) {
#pragma unroll
            for (int e = 0; e < CN; ++e) red[wave * d + k + e] = acc[i][e];
        }
    }
    __syncthreads();
    for (int c = tid; c < d; c += NT) {
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) sum += red[w * d + c];
        part[((int64_t)p * B + b) * d + c] = sum;
    }
}

}  // namespace moc
