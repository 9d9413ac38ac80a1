// Row-wise Top-K selection over the fp32 gate (the mask M = TopK(G) of the paper's section
// "Mixture-of-Channels architecture"): exactly K channels per row, the largest signed values,
// equal values ordered by channel index (lower first), -0.0 equal to +0.0.
//
// One workgroup per row.  A most-significant-digit-first radix select on order-preserving 32-bit
// keys finds the key of the K-th largest element: the sign bit is settled with ballots, then
// digits of 10, 11 and 10 bits with LDS histograms.  A final ordered pass ranks the selected
// channels with wavefront ballots, so the output ascends by channel without any sort.
//
// topk_rows_kernel keeps the whole row in registers (all global loads are issued before anything
// waits on them); topk_rows_lds_kernel parks the keys in LDS instead and serves rows that are too
// long for registers or not 16-byte aligned.
//
// FUSED = true is the training forward: besides idx and the gate values it gathers U at the
// selected channels and writes the dense activation row Z' = SiLU(G) . M . U (Eq. MoC-2), zeros
// on unselected channels and on the padding up to ldz.
#pragma once
#include "common.h"

namespace moc {

constexpr int kTopkBins = 2048;

template <class E> __device__ __forceinline__ void store_vec4_any(E* p, const float v[4]);
template <> __device__ __forceinline__ void store_vec4_any<float>(float* p, const float v[4]) {
    *reinterpret_cast<f32x4_t*>(p) = f32x4_t{v[0], v[1], v[2], v[3]};
}
template <> __device__ __forceinline__ void store_vec4_any<bf16_t>(bf16_t* p, const float v[4]) {
    *reinterpret_cast<u32x2_t*>(p) = u32x2_t{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
}

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
    // Keyed selection (Top-K position variants): g then holds the transformed keys the ranking is
    // done on, and the gate values themselves are fetched from here ([T, ldg] like g); null otherwise.
    const float* g_raw;
};

// Selection keys of the Top-K position variants: mode 1 ranks SiLU(g) (ablation row "After SiLU"),
// mode 2 ranks |SiLU(g)| (the selection of the proof of Theorem 1).  Element-wise, [T, ld] fp32.
static __global__ void topk_key_transform_kernel(const float* __restrict__ g, float* __restrict__ keys, int64_t n, int mode) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const float s = silu_f32(g[i]);
        keys[i] = mode == 2 ? fabsf(s) : s;
    }
}

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
__global__ __launch_bounds__(NT) void topk_rows_lds_kernel(TopkArgs<E> a) {
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
                const float g = a.g_raw ? a.g_raw[row * a.ldg + j0 + e] : key_float(k[e]);
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

// ---------------------------------------------------------------- register-resident variant
// Row of up to NCH * NT * 4 channels; thread t holds channels c*NT*4 + t*4 .. +3 of every chunk c.
// Per digit pass there are three barriers: after the histogram atomics, inside the workgroup-wide
// scan of the bins, and after the crossing bin has been published.  Channels are ranked
// with one ballot sweep whose per-lane prefixes stay in registers.  When all keys equal to the
// threshold are selected (the usual case) a single ">= threshold" predicate is ranked; ties that
// straddle the cut take the general path with a second predicate.  Selected channels are staged
// in LDS at their output slot, so that the compact outputs are written slot by slot (coalesced,
// SiLU evaluated K times instead of under divergence for every channel) and the dense Z' row is
// assembled in LDS and streamed out with 16-byte stores.  Dynamic LDS: topk_reg_dyn_lds().
//
// The work of one row is a device function: `row` selects the row, topk_dyn is the caller's LDS area
// of topk_reg_dyn_lds() bytes, `write_out` = false skips every global store (the caller only wants
// the threshold), and the return value describes the selected set without the index list: a channel j with key k belongs
// to it iff k > tau, or k == tau and j <= cut (cut = INT_MAX when every key equal to tau is in).
struct TopkThreshold {
    uint32_t tau;
    int cut;
};

__device__ __forceinline__ bool topk_member(uint32_t key, int j, TopkThreshold t) {
    return key > t.tau || (key == t.tau && j <= t.cut);
}

template <class E, int NT, int NCH, bool FUSED>
__device__ __forceinline__ TopkThreshold topk_row_body(const TopkArgs<E>& a, int64_t row, unsigned char* topk_dyn, bool write_out) {
    constexpr int NW = NT / 64;
    constexpr int CHUNK = NT * 4;
    uint32_t (*hist)[kTopkBins] = reinterpret_cast<uint32_t (*)[kTopkBins]>(topk_dyn);     // histograms, later slot lists + dense row
    __shared__ int tab_gt[NCH * NW], tab_eq[NCH * NW];
    __shared__ int red[NW];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_need, sh_cnt, sh_cut;
    const int F = a.F, K = a.K;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* grow = a.g + row * a.ldg;

    // ---- all loads of the row up front
    f32x4_t gv[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        // ldg is a multiple of 4, so the aligned 16-byte block that holds channel j0 < F lies inside
        // the row pitch; what it holds past F is masked out when the keys are made
        // Threads past the end of the row re-read its last block instead of branching.
        const int j0 = min(c * CHUNK + tid * 4, ((F + 3) & ~3) - 4);
        gv[c] = *reinterpret_cast<const f32x4_t*>(grow + j0);
    }
    u32x2_t uraw[NCH];     // FUSED, E = bf16: four packed values
    f32x4_t uf[NCH];       // FUSED, E = float
    if (FUSED) {
        const E* urow = a.u + row * a.ldu;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int j0 = min(c * CHUNK + tid * 4, (int)a.ldu - 4);      // ldu is a multiple of 64
            if (sizeof(E) == 2) uraw[c] = *reinterpret_cast<const u32x2_t*>(reinterpret_cast<const bf16_t*>(urow) + j0);
            else uf[c] = *reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(urow) + j0);
        }
    }
    for (int i = tid * 4; i < 2 * kTopkBins; i += NT * 4) *reinterpret_cast<u32x4_t*>(&hist[0][0] + i) = u32x4_t{0, 0, 0, 0};

    // Keys of channels past F: below 2^23, i.e. below the key of every finite value, so they are
    // never selected and need no range check later; spread over the four lowest bins of the first
    // digit so that their histogram updates do not pile up on one address.
    const uint32_t pad_key = (uint32_t)(lane & 3) << 21;
    uint32_t key[NCH][4];
    int npos = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
#pragma unroll
        for (int e = 0; e < 4; ++e) key[c][e] = float_key(gv[c][e]);
        if ((c + 1) * CHUNK > F) {                          // only the chunks that reach past the row (uniform)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c * CHUNK + tid * 4 + e >= F) key[c][e] = pad_key;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) npos += (int)(key[c][e] >> 31);
    }
    // ---- sign digit: keys with the top bit set are the non-negative values
    npos = (int)wave_sum((float)npos);                       // exact: counts are far below 2^24
    if (lane == 0) red[wave] = npos;
    __syncthreads();
    int total_pos = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) total_pos += red[w];
    uint32_t prefix = total_pos >= K ? 1u : 0u;              // leading bit of the K-th largest key
    int need = total_pos >= K ? K : K - total_pos;
    int cnt_eq = 0;

    // ---- three histogram passes over bits [30:21], [20:10], [9:0]
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const int nbits = pass == 1 ? 11 : 10;
        const int nbins = 1 << nbits;
        const int pshift = shift + nbits;
        uint32_t* cur = hist[pass & 1];
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t k = key[c][e];
                if ((k >> pshift) == prefix) atomicAdd(&cur[(k >> shift) & (nbins - 1)], 1u);
            }
        __syncthreads();
        {
            // Suffix scan over all kTopkBins counters by the whole workgroup (a 10-bit pass leaves the
            // upper half at zero): thread t owns the BPT bins below kTopkBins - BPT t, so thread order
            // is descending bin order; the thread whose range crosses `need` publishes the result.
            // (a workgroup size that does not divide the bins, 768, leaves its last threads without bins)
            constexpr int BPT = NT >= 1024 ? 2 : (NT >= 512 ? 4 : 8);
            static_assert(BPT * NT >= kTopkBins, "bins per thread");
            const bool owner = BPT * (tid + 1) <= kTopkBins;
            const int base = owner ? kTopkBins - BPT * (tid + 1) : 0;
            uint32_t hv[BPT];
            if (BPT == 2) {
                const u32x2_t t2 = *reinterpret_cast<const u32x2_t*>(cur + base);
                hv[0] = t2[0]; hv[1] = t2[1];
            } else {
#pragma unroll
                for (int q = 0; q < BPT; q += 4) {
                    const u32x4_t t4 = *reinterpret_cast<const u32x4_t*>(cur + base + q);
                    hv[q] = t4[0]; hv[q + 1] = t4[1]; hv[q + 2] = t4[2]; hv[q + 3] = t4[3];
                }
            }
            if (!owner) {
#pragma unroll
                for (int q = 0; q < BPT; ++q) hv[q] = 0;
            }
            int local = 0;
#pragma unroll
            for (int q = 0; q < BPT; ++q) local += (int)hv[q];
            int inc = local;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(inc, o, 64);
                if (lane >= o) inc += t;
            }
            if (lane == 63) red[wave] = inc;
            __syncthreads();
            int before = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) before += (w < wave) ? red[w] : 0;
            inc += before;
            const int above = inc - local;
            if (owner && above < need && inc >= need) {      // the crossing bin is one of mine
                int run = above, fb = -1, fneed = 0, fh = 0;
#pragma unroll
                for (int q = BPT - 1; q >= 0; --q) {         // descending bins
                    const int h = (int)hv[q];
                    if (fb < 0 && run + h >= need) { fb = base + q; fneed = need - run; fh = h; }
                    run += h;
                }
                sh_prefix = (prefix << nbits) | (uint32_t)fb;
                sh_need = fneed;
                sh_cnt = fh;
            }
            if (pass == 1) {                                  // buffer 0 was used by pass 0: clear it for pass 2
                uint32_t* nxt = hist[0];
                for (int i = tid * 4; i < kTopkBins; i += NT * 4) *reinterpret_cast<u32x4_t*>(nxt + i) = u32x4_t{0, 0, 0, 0};
            }
        }
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        cnt_eq = sh_cnt;
    }
    const uint32_t tau = prefix;
    const bool all_ties = cnt_eq == need;        // every key equal to tau is selected (the usual case)
    // "above" test as one unsigned compare: k >= thr (padding keys lie below every finite key).
    const uint32_t thr = tau + ((all_ties || tau == 0xFFFFFFFFu) ? 0u : 1u);

    // ---- one ballot sweep: per-lane prefixes in registers, per-wave totals to LDS
    int pg[NCH], pe[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        int lg = 0, ngt = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t bg = __ballot(key[c][e] >= thr);
            lg += mbcnt(bg);
            ngt += __popcll(bg);
        }
        pg[c] = lg;
        pe[c] = 0;
        if (lane == 0) {
            tab_gt[c * NW + wave] = ngt;
            tab_eq[c * NW + wave] = 0;
        }
    }
    if (!all_ties) {                               // ties straddle the cut: rank the equal keys too
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            int le = 0, neq = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint64_t be = __ballot(key[c][e] == tau);
                le += mbcnt(be);
                neq += __popcll(be);
            }
            pe[c] = le;
            if (lane == 0) tab_eq[c * NW + wave] = neq;
        }
    }
    __syncthreads();
    if (wave == 0) {
        constexpr int n = NCH * NW;
        constexpr int per = (n + 63) / 64;
        int sg = 0, se = 0;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            const int i = lane * per + q;
            if (i < n) { sg += tab_gt[i]; se += tab_eq[i]; }
        }
        int ig = sg, ie = se;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int tg = __shfl_up(ig, o, 64), te = __shfl_up(ie, o, 64);
            if (lane >= o) { ig += tg; ie += te; }
        }
        int rg = ig - sg, re = ie - se;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            const int i = lane * per + q;
            if (i < n) {
                const int g0 = tab_gt[i], e0 = tab_eq[i];
                tab_gt[i] = rg; tab_eq[i] = re;
                rg += g0; re += e0;
            }
        }
    }
    // ---- slot lists and the dense row take over the histogram memory (dead since the last pass)
    uint32_t* rec = reinterpret_cast<uint32_t*>(topk_dyn);            // [K] records {channel, key, up value}
    E* zrow = reinterpret_cast<E*>(topk_dyn + ((size_t)3 * K * 4 + 15) / 16 * 16);   // [ldz] (FUSED)
    const int ldz = FUSED ? (int)a.ldz : 0;
    if (FUSED) {
        constexpr int PER = 16 / (int)sizeof(E);
        for (int i = tid * PER; i < ldz; i += NT * PER) *reinterpret_cast<u32x4_t*>(zrow + i) = u32x4_t{0, 0, 0, 0};
    }
    if (tid == 0) sh_cut = 0x7FFFFFFF;
    __syncthreads();

    // ---- rank: every selected channel drops (channel, gate value, up value) into LDS at its
    //      output slot (number of selected channels before it)
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int j0 = c * CHUNK + tid * 4;
        float uu[4];
        if (FUSED) {
            if (sizeof(E) == 2) {
                uu[0] = __uint_as_float(uraw[c][0] << 16); uu[1] = __uint_as_float(uraw[c][0] & 0xFFFF0000u);
                uu[2] = __uint_as_float(uraw[c][1] << 16); uu[3] = __uint_as_float(uraw[c][1] & 0xFFFF0000u);
            } else {
                uu[0] = uf[c][0]; uu[1] = uf[c][1]; uu[2] = uf[c][2]; uu[3] = uf[c][3];
            }
        }
        int gt_before = tab_gt[c * NW + wave] + pg[c];
        if (all_ties) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t k = key[c][e];
                if (k >= thr) {
                    uint32_t* r = rec + 3 * min(gt_before, K - 1);
                    r[0] = (uint32_t)(j0 + e);
                    r[1] = k;
                    if (FUSED) r[2] = __float_as_uint(uu[e]);
                    ++gt_before;
                }
            }
        } else {
            int eq_before = tab_eq[c * NW + wave] + pe[c];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t k = key[c][e];
                const bool isgt = k >= thr, iseq = k == tau;
                if (isgt || (iseq && eq_before < need)) {
                    uint32_t* r = rec + 3 * min(gt_before + min(eq_before, need), K - 1);
                    r[0] = (uint32_t)(j0 + e);
                    r[1] = k;
                    if (FUSED) r[2] = __float_as_uint(uu[e]);
                    if (iseq && eq_before == need - 1) sh_cut = j0 + e;     // the last tie that is taken
                }
                gt_before += isgt ? 1 : 0;
                eq_before += iseq ? 1 : 0;
            }
        }
    }
    __syncthreads();
    const TopkThreshold result{tau, sh_cut};
    if (!write_out) return result;
    // ---- write the compact outputs slot by slot (coalesced) and scatter z' into the dense row
    for (int sl = tid; sl < K; sl += NT) {
        const int j = min((int)rec[3 * sl], F - 1);       // the clamp only matters for non-finite input
        const float g = a.g_raw ? a.g_raw[row * a.ldg + j] : key_float(rec[3 * sl + 1]);
        a.idx[row * K + sl] = j;
        if (a.gsel_f32) a.gsel_f32[row * K + sl] = g;
        if (a.gvals) Elem<E>::store(a.gvals + row * K + sl, g);
        if (FUSED) {
            const float u = __uint_as_float(rec[3 * sl + 2]);
            Elem<E>::store(a.uvals + row * K + sl, u);
            Elem<E>::store(zrow + j, silu_f32(g) * u);
        }
    }
    if (FUSED) {
        __syncthreads();
        constexpr int PER = 16 / (int)sizeof(E);
        E* zout = a.zd + row * a.ldz;
        for (int i = tid * PER; i < ldz; i += NT * PER)
            *reinterpret_cast<u32x4_t*>(zout + i) = *reinterpret_cast<const u32x4_t*>(zrow + i);
    }
    return result;
}

template <class E, int NT, int NCH, bool FUSED>
__global__ __launch_bounds__(NT) void topk_rows_kernel(TopkArgs<E> a) {
    extern __shared__ __align__(16) unsigned char topk_dyn[];
    topk_row_body<E, NT, NCH, FUSED>(a, blockIdx.x, topk_dyn, true);
}

// Dynamic LDS of topk_rows_kernel: two digit histograms, reused for the three slot lists and, in
// the fused forward, the dense row.
inline size_t topk_reg_dyn_lds(int K, int64_t ldz, size_t elem, bool fused) {
    size_t lists = (size_t)3 * K * 4;
    lists = (lists + 15) / 16 * 16;
    if (fused) lists += (size_t)ldz * elem;
    const size_t hists = (size_t)2 * kTopkBins * 4;
    return lists > hists ? lists : hists;
}

inline size_t topk_lds_bytes(int F, int NT, int VEC) {
    const int chunk = NT * VEC;
    const int nchunk = (F + chunk - 1) / chunk;
    return (size_t)nchunk * chunk * 4 + kTopkBins * 4 + (size_t)2 * nchunk * (NT / 64) * 4 + (NT / 64) * 4;
}

}  // namespace moc
