// Row-wide decode (paper section "Accelerated inference") as ONE persistent launch.
//
// One workgroup per compute unit; the four steps of the per-token recipe are phases of the same
// kernel, and data flows between workgroups through memory without launch boundaries:
//
//   G   gate:   g[b, j] = x[b] . wg[j] for every channel (all of W_gate streams once);
//               rows are dealt to wavefronts (B <= 4, fp32 FMA) or 48-row blocks to workgroups
//               (5..16 tokens, bf16, v_mfma_f32_16x16x32_bf16).  g goes to the workspace, and each
//               workgroup keeps the gate values of its own rows in LDS.
//   S   select: the exact row Top-K threshold of token b (tau, cut) is found by workgroup b from the
//               complete gate row, and published; with one token every workgroup finds it
//               redundantly and nobody waits for anybody's result.
//   U   up:     every workgroup looks at its OWN gate rows: channel j is in the union if some
//               token's gate value passes that token's threshold.  W_up[j] is read once per union
//               channel and dotted with every token that selected it:
//               z[j, b] = SiLU(g[b, j]) (x[b] . wu[j]); the channel's token mask is stored with it.
//   D   down:   y[b, :] = sum_j z[j, b] wd[j, :] over a P x C split: workgroup (p, c) covers the
//               p-th range of channels and the c-th slice of columns, reads each union row's
//               segment once for all tokens and writes one partial [B, d/C]; the last of the P
//               workgroups of a column slice to finish adds the P partials in a fixed order and
//               writes y (deterministic: no floating-point atomics).
//       The index lists idx[b, :] are written by the last B workgroups, which get no share of D.
//
// Synchronisation is by data, not by barriers.  A grid-wide barrier costs three to four memory round
// trips of about 1.5 us here (wait for the stores, set a flag, see everybody's flag, release), and an
// agent-scope fence another 2 us because it writes back and invalidates a whole L2.  Instead every
// 32-bit value that crosses workgroups travels in a 64-bit word whose upper half is the call's TAG,
// written and read with single device-coherent 64-bit accesses (relaxed atomics at agent scope: they
// go through to memory instead of staying in one XCD's L2).  A consumer that finds the tag has the
// value; otherwise it reads again.  No store has to be ordered against any other, so nothing waits
// for store acknowledgements, and stale contents of the workspace never match: the tag mixes a host
// call counter with the generation word of the workspace, which workgroup 0 advances once per call
// (replays of a captured graph repeat the host counter but not the generation), and is always odd (a
// zero-filled buffer holds no valid word).  Every retry loop is bounded: after kDecSpinLimit rounds
// a workgroup raises `abort_tag` and every workgroup leaves (y is then undefined); that can only
// happen if the workgroups are not all resident, which the host prevents by launching one per compute
// unit.
#pragma once
#include "common.h"
#include "decode_kernels.h"
#include "topk.h"

namespace moc {

constexpr int kDecMaxWG = 1024;
constexpr int kDecMaxB = 16;
constexpr unsigned kDecSpinLimit = 1u << 21;     // retry rounds of a microsecond or more each

struct DecodeSync {
    uint64_t gen;                      // generation: advanced by workgroup 0 once per call
    uint64_t abort_tag;                // tag of a call that gave up waiting
    uint64_t thr[kDecMaxB][2];         // tagged (tau, cut) of every token
    uint64_t hello[kDecMaxWG];         // tagged: workgroup w has read the generation word
    uint64_t dflag[kDecMaxWG];         // tagged: partial (c, p) of the down projection is written
};

// Development aid, compiled in only with -DMOC_DEC_TRACE: workgroups 0 and gridDim.x - 40 stamp the
// 100 MHz wall clock at phase boundaries into the tail of the 32 KB flag area of the workspace.
#ifdef MOC_DEC_TRACE
#define DEC_TRACE(sync, k)                                                                                   \
    do {                                                                                                     \
        if (threadIdx.x == 0 && (blockIdx.x == 0 || blockIdx.x == gridDim.x - 40))                           \
            reinterpret_cast<uint64_t*>(reinterpret_cast<unsigned char*>(sync) + 28 * 1024)[(blockIdx.x ? 32 : 0) + (k)] = wall_clock64(); \
    } while (0)
#define DEC_TRACE_END(sync)                                                                                  \
    do {                                                                                                     \
        if (threadIdx.x == 0)                                                                                \
            atomicMax(reinterpret_cast<unsigned long long*>(reinterpret_cast<unsigned char*>(sync) + 28 * 1024) + 63, (unsigned long long)wall_clock64()); \
    } while (0)
#else
#define DEC_TRACE(sync, k) do { } while (0)
#define DEC_TRACE_END(sync) do { } while (0)
#endif

template <class E> struct DecArgs {
    const E *x, *wg, *wu, *wd;
    E* y;
    int32_t* idx;                      // [B, K]
    int B, d, F, K;
    int64_t ldF;
    uint64_t* g2;                      // [B, ldF] tagged gate values
    uint64_t* zt;                      // [F, 1 + BT] tagged token mask and z' of every channel
    float* part;                       // [P, B, d] partial outputs
    DecodeSync* sync;
    uint32_t salt;                     // host call counter
    int P, C;                          // down projection: channel ranges x column slices (P * C <= gridDim.x)
    int rmax;                          // gate rows per wavefront (row-per-wavefront variant) or blocks per workgroup (MFMA variant)
    int off_own, off_over;             // LDS byte offsets: own gate values, phase-overlaid area
};

// ---------------------------------------------------------------- device-coherent accesses and tags
__device__ __forceinline__ uint64_t dec_ld(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void dec_st(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float dec_ldf(const float* p) {
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<const uint32_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void dec_stf(float* p, float v) {
    __hip_atomic_store(reinterpret_cast<uint32_t*>(p), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t dec_pack(uint32_t tag, uint32_t v) { return ((uint64_t)tag << 32) | v; }
__device__ __forceinline__ uint64_t dec_packf(uint32_t tag, float v) { return dec_pack(tag, __float_as_uint(v)); }
__device__ __forceinline__ bool dec_tagged(uint64_t w, uint32_t tag) { return (uint32_t)(w >> 32) == tag; }
// every store this wavefront has issued is acknowledged
__device__ __forceinline__ void dec_drain() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// 16-byte device-coherent load, issued without waiting; dec_ld16_wait makes the value usable.
__device__ __forceinline__ u32x4_t dec_ld16_issue(const void* p) {
    u32x4_t v;
    asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1" : "=v"(v) : "v"(p) : "memory");
    return v;
}
__device__ __forceinline__ void dec_ld16_wait(u32x4_t& v) { asm volatile("s_waitcnt vmcnt(0)" : "+v"(v) : : "memory"); }

// Tag of this call: mixes the host call counter with the generation the workspace is in; odd.
__device__ __forceinline__ uint32_t dec_make_tag(uint32_t salt, uint64_t gen) {
    return ((salt * 0x9E3779B1u) ^ ((uint32_t)gen * 0x85EBCA6Bu + 0x27D4EB2Fu)) | 1u;
}

// One retry round of a wait has failed: true if the call is to be given up (somebody raised the
// abort word, which is looked at every 64th round, or this wavefront has waited kDecSpinLimit rounds
// and raises it).
__device__ __forceinline__ bool dec_give_up(DecodeSync* sync, uint32_t tag, unsigned& spins) {
    ++spins;
    if ((spins & 63u) != 0 && spins <= kDecSpinLimit) {
        __builtin_amdgcn_s_sleep(8);
        return false;
    }
    const bool aborted = dec_tagged(dec_ld(&sync->abort_tag), tag);
    if (aborted || spins > kDecSpinLimit) {
        if (!aborted) {                                      // (every active lane stores the same values)
            dec_st(&sync->abort_tag, dec_pack(tag, 1u));
            dec_st(&sync->gen, dec_ld(&sync->gen) + 2);      // the next call must not meet this call's words
        }
        return true;
    }
    __builtin_amdgcn_s_sleep(16);
    return false;
}

// ----------------------------------------------------------------------------- phase S
constexpr int kDecSelBins = 4096;       // first digit: bits [30:19] of the keys
constexpr int kDecSelCap = 512;         // candidates the one-wavefront finish takes (8 per lane)
constexpr size_t kDecSelLds = (size_t)kDecSelBins * 4 + (size_t)kDecSelCap * 8;

// The keys of one tagged gate row in registers: thread t holds channels c * NT * 4 + t * 4 .. + 3 of
// every chunk c < NCH; channels past F get keys below every finite key.  Reads the row again until
// every word carries the tag.  Returns false if the call was given up.
template <int NT, int NCH>
__device__ __forceinline__ bool dec_row_keys(const uint64_t* grow, int F, uint32_t tag, DecodeSync* sync,
                                             uint32_t (&key)[NCH][4]) {
    constexpr int CHUNK = NT * 4;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t pad_key = (uint32_t)(lane & 3) << 21;
    unsigned spins = 0;
    bool have[NCH];                                   // chunk c of this thread has been read with all its tags
#pragma unroll
    for (int c = 0; c < NCH; ++c) have[c] = false;
    for (;;) {
        u32x4_t raw[NCH][2];
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            // the aligned block of four words that holds channel j0 < F lies inside the row pitch (a
            // multiple of 64 words); threads past the end of the row re-read its last block
            const int j0 = min(c * CHUNK + tid * 4, ((F + 3) & ~3) - 4);
            if (!have[c]) {
                raw[c][0] = dec_ld16_issue(grow + j0);
                raw[c][1] = dec_ld16_issue(grow + j0 + 2);
            }
        }
        bool valid = true;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if (!have[c]) {
                dec_ld16_wait(raw[c][0]);
                dec_ld16_wait(raw[c][1]);
                bool ok = true;
                uint32_t k[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t bits = raw[c][e >> 1][(e & 1) * 2], t = raw[c][e >> 1][(e & 1) * 2 + 1];
                    if (c * CHUNK + tid * 4 + e >= F) k[e] = pad_key;
                    else {
                        k[e] = float_key(__uint_as_float(bits));
                        ok = ok && t == tag;
                    }
                }
                if (ok) {
                    have[c] = true;
#pragma unroll
                    for (int e = 0; e < 4; ++e) key[c][e] = k[e];
                }
                valid = valid && ok;
            }
        }
        if (__syncthreads_and(valid)) return true;
        if (dec_give_up(sync, tag, spins)) return false;
    }
}

// Exact Top-K threshold of ONE row, tuned for the case that the row is all a compute unit has to
// do: sign by counting, bits [30:19] with one LDS histogram (4096 bins keep the bins near the
// threshold at a few hundred keys at most, so the atomics rarely collide), then the keys of the
// crossing bin are compacted and a single wavefront finds the exact key by bisection with ballot
// counts (and, if equal keys straddle the cut, the last channel taken).  *ok = false when the
// crossing bin holds more than kDecSelCap keys (heavily tied rows); the caller then runs
// topk_keys_general.  lds: kDecSelLds bytes.
template <int NT, int NCH>
__device__ __forceinline__ TopkThreshold dec_select_keys(const uint32_t (&key)[NCH][4], int F, int K, unsigned char* lds, bool* ok) {
    constexpr int NW = NT / 64, CHUNK = NT * 4;
    constexpr int BPT = NT >= 1024 ? 4 : 8;                  // bins per owning thread in the scan
    static_assert(BPT * NT >= kDecSelBins, "bins per thread");
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds);
    uint32_t* cand = hist + kDecSelBins;                     // [kDecSelCap][2]: key, channel
    __shared__ int red[NW];
    __shared__ int sh_bin, sh_need, sh_cnt, sh_ncand;
    __shared__ TopkThreshold sh_thr;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid * 4; i < kDecSelBins; i += NT * 4) *reinterpret_cast<u32x4_t*>(hist + i) = u32x4_t{0, 0, 0, 0};
    if (tid == 0) sh_ncand = 0;
    // ---- sign: keys with the top bit set are the non-negative values
    int npos = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) npos += (int)(key[c][e] >> 31);
    npos = (int)wave_sum((float)npos);                       // exact: counts are far below 2^24
    if (lane == 0) red[wave] = npos;
    __syncthreads();
    int total_pos = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) total_pos += red[w];
    const uint32_t sign = total_pos >= K ? 1u : 0u;
    int need = total_pos >= K ? K : K - total_pos;
    // ---- bits [30:19]
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t k = key[c][e];
            if ((k >> 31) == sign) atomicAdd(&hist[(k >> 19) & (kDecSelBins - 1)], 1u);
        }
    __syncthreads();
    {
        // suffix scan: thread t owns the BPT bins below kDecSelBins - BPT t (descending bin order)
        const bool owner = BPT * (tid + 1) <= kDecSelBins;
        const int base = owner ? kDecSelBins - BPT * (tid + 1) : 0;
        uint32_t hv[BPT];
#pragma unroll
        for (int q = 0; q < BPT; q += 4) {
            const u32x4_t t4 = *reinterpret_cast<const u32x4_t*>(hist + base + q);
            hv[q] = t4[0]; hv[q + 1] = t4[1]; hv[q + 2] = t4[2]; hv[q + 3] = t4[3];
        }
        int local = 0;
#pragma unroll
        for (int q = 0; q < BPT; ++q) {
            if (!owner) hv[q] = 0;
            local += (int)hv[q];
        }
        int inc = local;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o, 64);
            if (lane >= o) inc += t;
        }
        if (lane == 63) red[wave] = inc;       // (the reads of red above lie before the barrier after the atomics)
        __syncthreads();
        int before = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) before += (w < wave) ? red[w] : 0;
        inc += before;
        const int above = inc - local;
        if (owner && above < need && inc >= need) {           // the crossing bin is one of mine
            int run = above, fb = -1, fneed = 0, fh = 0;
#pragma unroll
            for (int q = BPT - 1; q >= 0; --q) {
                const int h = (int)hv[q];
                if (fb < 0 && run + h >= need) { fb = base + q; fneed = need - run; fh = h; }
                run += h;
            }
            sh_bin = fb;
            sh_need = fneed;
            sh_cnt = fh;
        }
    }
    __syncthreads();
    const uint32_t prefix = (sign << 12) | (uint32_t)sh_bin;  // bits [31:19] of the K-th largest key
    need = sh_need;
    const int cnt = sh_cnt;
    if (cnt > kDecSelCap) {
        *ok = false;
        return TopkThreshold{0u, 0};
    }
    *ok = true;
    // ---- the crossing bin's keys, in any order
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t k = key[c][e];
            if ((k >> 19) == prefix) {
                const int slot = min(atomicAdd(&sh_ncand, 1), kDecSelCap - 1);
                cand[2 * slot] = k;
                cand[2 * slot + 1] = (uint32_t)(c * CHUNK + tid * 4 + e);
            }
        }
    __syncthreads();
    if (wave == 0) {
        constexpr int PL = kDecSelCap / 64;
        uint32_t ck[PL];
        int cj[PL];
        bool cv[PL];
#pragma unroll
        for (int q = 0; q < PL; ++q) {
            const int i = q * 64 + lane;
            cv[q] = i < cnt;
            ck[q] = cv[q] ? cand[2 * i] : 0u;
            cj[q] = cv[q] ? (int)cand[2 * i + 1] : 0;
        }
        const int nq = (cnt + 63) >> 6;                       // slots per lane that hold candidates
        auto count = [&](auto pred) -> int {
            int n = 0;
#pragma unroll
            for (int q = 0; q < PL; ++q)
                if (q < nq) n += __popcll(__ballot(cv[q] && pred(q)));
            return n;
        };
        uint32_t p = prefix << 19;
#pragma unroll 1
        for (int bit = 18; bit >= 0; --bit) {
            const uint32_t cp = p | (1u << bit);
            if (count([&](int q) { return ck[q] >= cp; }) >= need) p = cp;
        }
        const uint32_t tau = p;
        const int ngt = count([&](int q) { return ck[q] > tau; });
        const int neq = count([&](int q) { return ck[q] == tau; });
        const int need_eq = need - ngt;                       // 1 <= need_eq <= neq
        int cut = 0x7FFFFFFF;
        if (need_eq < neq) {
            // equal keys straddle the cut: the lowest channels are taken; find the need_eq-th of them
            int lo = 0, hi = F - 1;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (count([&](int q) { return ck[q] == tau && cj[q] <= mid; }) >= need_eq) hi = mid;
                else lo = mid + 1;
            }
            cut = lo;
        }
        if (lane == 0) sh_thr = TopkThreshold{tau, cut};
    }
    __syncthreads();
    return sh_thr;
}

// The general (slow, any distribution) threshold search on keys in registers: bit by bit over all 32
// bits with ballot counts, then the tie cut by bisection over the channel index.
template <int NT, int NCH>
__device__ __forceinline__ TopkThreshold topk_keys_general(const uint32_t (&key)[NCH][4], int F, int K) {
    constexpr int NW = NT / 64, CHUNK = NT * 4;
    __shared__ int cnt_red[2][NW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int it = 0;
    auto count = [&](auto pred) -> int {
        int cw = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) cw += __popcll(__ballot(pred(key[c][e], c * CHUNK + tid * 4 + e)));
        if (lane == 0) cnt_red[it & 1][wave] = cw;
        __syncthreads();
        int tot = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += cnt_red[it & 1][w];
        ++it;
        return tot;
    };
    uint32_t p = 0;
#pragma unroll 1
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cp = p | (1u << bit);
        if (count([&](uint32_t k, int) { return k >= cp; }) >= K) p = cp;
    }
    const uint32_t tau = p;
    const int ngt = count([&](uint32_t k, int) { return k > tau; });
    const int neq = count([&](uint32_t k, int) { return k == tau; });
    const int need_eq = K - ngt;
    int cut = 0x7FFFFFFF;
    if (need_eq < neq) {
        int lo = 0, hi = F - 1;
#pragma unroll 1
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (count([&](uint32_t k, int j) { return k == tau && j <= mid; }) >= need_eq) hi = mid;
            else lo = mid + 1;
        }
        cut = lo;
    }
    return TopkThreshold{tau, cut};
}

// idx[0 .. K-1] of one row from its threshold: the selected channels in ascending order (one ballot
// sweep over the keys, per-wavefront totals scanned through LDS).
template <int NT, int NCH>
__device__ __forceinline__ void dec_write_idx(const uint32_t (&key)[NCH][4], int K, TopkThreshold thr, int32_t* idx_row) {
    constexpr int NW = NT / 64, CHUNK = NT * 4;
    __shared__ int tab[NCH * NW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int pre[NCH][4];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        int tot = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t m = __ballot(topk_member(key[c][e], c * CHUNK + tid * 4 + e, thr));
            pre[c][e] = mbcnt(m);
            tot += __popcll(m);
        }
        if (lane == 0) tab[c * NW + wave] = tot;
    }
    __syncthreads();
    if (wave == 0) {                                      // exclusive scan of the table in (chunk, wavefront) order
        constexpr int n = NCH * NW;
        constexpr int per = (n + 63) / 64;
        int sum = 0;
#pragma unroll
        for (int q = 0; q < per; ++q) sum += (lane * per + q < n) ? tab[lane * per + q] : 0;
        int inc = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o, 64);
            if (lane >= o) inc += t;
        }
        int run = inc - sum;
#pragma unroll
        for (int q = 0; q < per; ++q) {
            const int i = lane * per + q;
            if (i < n) {
                const int t = tab[i];
                tab[i] = run;
                run += t;
            }
        }
    }
    __syncthreads();
    // channel order is (chunk, thread, element): before a thread's element e come the earlier chunks,
    // the earlier wavefronts of the chunk, the lower lanes' four elements and its own lower elements
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int base = tab[c * NW + wave];
        int lower = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) lower += pre[c][e];
        int mine = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = c * CHUNK + tid * 4 + e;
            if (topk_member(key[c][e], j, thr)) {
                const int slot = base + lower + mine;
                if (slot < K) idx_row[slot] = j;
                ++mine;
            }
        }
    }
    __syncthreads();
}

// Phase S for all variants: the thresholds of all tokens into thr_lds[BT].  Returns false if the call
// was given up.  The last B workgroups also write the index lists here (token b by workgroup
// gridDim.x - 1 - b).
template <int BT, int NT, int NCH, class E>
__device__ __forceinline__ bool dec_phase_select(const DecArgs<E>& a, unsigned char* over, TopkThreshold* thr_lds, uint32_t tag) {
    DecodeSync* sync = a.sync;
    const int B = a.B, nwg = gridDim.x;
    const int tid = threadIdx.x;
    auto select = [&](const uint32_t (&key)[NCH][4]) -> TopkThreshold {
        bool ok;
        TopkThreshold t = dec_select_keys<NT, NCH>(key, a.F, a.K, over, &ok);
        if (!ok) t = topk_keys_general<NT, NCH>(key, a.F, a.K);      // heavily tied row
        return t;
    };
    const int tb = nwg - 1 - (int)blockIdx.x;             // token whose index list this workgroup writes, if < B
    if (B == 1) {
        uint32_t key[NCH][4];
        if (!dec_row_keys<NT, NCH>(a.g2, a.F, tag, sync, key)) return false;
        const TopkThreshold t = select(key);
        if (tid == 0) thr_lds[0] = t;
        __syncthreads();
        if (tb == 0) dec_write_idx<NT, NCH>(key, a.K, t, a.idx);
        return true;
    }
    if ((int)blockIdx.x < B) {
        uint32_t key[NCH][4];
        if (!dec_row_keys<NT, NCH>(a.g2 + (int64_t)blockIdx.x * a.ldF, a.F, tag, sync, key)) return false;
        const TopkThreshold t = select(key);
        if (tid == 0) {
            dec_st(&sync->thr[blockIdx.x][0], dec_pack(tag, t.tau));
            dec_st(&sync->thr[blockIdx.x][1], dec_pack(tag, (uint32_t)t.cut));
        }
    }
    // everybody: wait for the B published thresholds (first wavefront polls, two words per token)
    __shared__ int sh_ok;
    if (tid < 64) {
        unsigned spins = 0;
        bool ok = true;
        uint64_t w = 0;
        for (;;) {
            bool have = true;
            if (tid < 2 * B) {
                w = dec_ld(&sync->thr[tid >> 1][tid & 1]);
                have = dec_tagged(w, tag);
            }
            if (__all(have)) break;
            if (dec_give_up(sync, tag, spins)) { ok = false; break; }
        }
        if (ok && tid < 2 * B) {
            if (tid & 1) thr_lds[tid >> 1].cut = (int)(uint32_t)w;
            else thr_lds[tid >> 1].tau = (uint32_t)w;
        }
        if (tid == 0) sh_ok = ok ? 1 : 0;
    }
    __syncthreads();
    if (!sh_ok) return false;
    if (tb < B) {                                         // index list of token tb: read its row (complete by now)
        uint32_t key[NCH][4];
        if (!dec_row_keys<NT, NCH>(a.g2 + (int64_t)tb * a.ldF, a.F, tag, sync, key)) return false;
        dec_write_idx<NT, NCH>(key, a.K, thr_lds[tb], a.idx + (int64_t)tb * a.K);
    }
    return true;
}

// ----------------------------------------------------------------------------- phase U
// The wavefronts of a workgroup share out its own gate rows (own row i belongs to wavefront
// i % NWV); rows(i, j, gp) gives the channel and the LDS address of its BT gate values.
// x sits in LDS with a row pitch of xpitch bytes.  Every own channel gets its tagged token mask, and
// the tagged z' of the tokens that selected it.
template <class E, int BT, int NWV, class Rows>
__device__ __forceinline__ void dec_phase_up(const DecArgs<E>& a, const unsigned char* xs, int xpitch, int nown, Rows rows,
                                             const TopkThreshold* thr, uint32_t tag) {
    constexpr int CN = Chunk<E>::N, UN = 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d = a.d, B = a.B;
    u32x4_t cur[UN], nxt[UN];
    auto fetch = [&](u32x4_t (&r)[UN], int j) {
        const E* wrow = a.wu + (int64_t)j * d;
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = (u * 64 + lane) * CN;
            r[u] = u32x4_t{0, 0, 0, 0};
            if (k < d) r[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + k));
        }
    };
    // token mask of own row i (0 past the end); the mask word is stored at once
    auto mask_of = [&](int i, int& j, const float*& gp) -> unsigned {
        j = -1;
        gp = nullptr;
        if (i >= nown) return 0u;
        rows(i, j, gp);
        if (j < 0) return 0u;
        unsigned m = 0;
#pragma unroll
        for (int b = 0; b < BT; ++b)
            if (b < B && topk_member(float_key(gp[b]), j, thr[b])) m |= 1u << b;
        if (lane == 0) dec_st(a.zt + (int64_t)j * (1 + BT), dec_pack(tag, m));
        return m;
    };
    int i = wave, j = -1, jn = -1;
    const float *gp = nullptr, *gpn = nullptr;
    unsigned m = 0, mn = 0;
    while (i < nown && (m = mask_of(i, j, gp)) == 0) i += NWV;       // first selected row of this wavefront
    if (m) fetch(cur, j);
    while (m) {
        int in = i + NWV;
        mn = 0;
        while (in < nown && (mn = mask_of(in, jn, gpn)) == 0) in += NWV;
        if (mn) fetch(nxt, jn);
        float zmine = 0.0f;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            if (m & (1u << b)) {                                      // uniform over the wavefront
                float dot = 0.0f;
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int k = (u * 64 + lane) * CN;
                    if (k < d) dot = Chunk<E>::dot(cur[u], *reinterpret_cast<const u32x4_t*>(xs + b * xpitch + k * (int)sizeof(E)), dot);
                }
                dot = wave_sum(dot);
                const float z = silu_f32(gp[b]) * dot;
                if (lane == b) zmine = z;
            }
        }
        if (lane < BT && (m >> lane & 1u)) dec_st(a.zt + (int64_t)j * (1 + BT) + 1 + lane, dec_packf(tag, zmine));
        i = in; j = jn; gp = gpn; m = mn;
        if (m) {
#pragma unroll
            for (int u = 0; u < UN; ++u) cur[u] = nxt[u];
        }
    }
}

// ----------------------------------------------------------------------------- phase D
// LDS use (from `lds`, the start of the dynamic area): the union channels of the workgroup's range and
// their token masks (two ints each), then the cross-wavefront reduction area [NWV][TB][seg] floats.
template <class E, int BT, int NT>
__device__ __forceinline__ void dec_phase_down(const DecArgs<E>& a, unsigned char* lds, uint32_t tag) {
    constexpr int CN = Chunk<E>::N, NWV = NT / 64;
    constexpr int TB = BT > 8 ? 8 : BT;              // tokens per wavefront: above 8 the wavefronts split into two token halves
    constexpr int NH = BT > 8 ? 2 : 1;
    constexpr int NWH = NWV / NH;                    // wavefronts per token half
    constexpr int UNR = 4;                           // row groups in flight per wavefront
    constexpr int ZS = 1 + BT;                       // words per channel in zt
    static_assert(NWV % NH == 0, "wavefronts must split evenly over the token halves");
    DecodeSync* sync = a.sync;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int P = a.P, C = a.C, B = a.B, d = a.d, F = a.F;
    const int wgid = blockIdx.x;
    if (wgid >= P * C) return;
    const int p = wgid / C, c = wgid % C;
    const int seg = d / C;                            // columns of this slice
    const int jlo = (int)((int64_t)p * F / P), jhi = (int)((int64_t)(p + 1) * F / P);
    int* list = reinterpret_cast<int*>(lds);          // [n][2]: channel, token mask
    const int list_cap = (F + P - 1) / P + 1;
    float* red = reinterpret_cast<float*>(lds + ((size_t)list_cap * 8 + 15) / 16 * 16);
    __shared__ int scan_red[NWV];
    __shared__ int sh_last;

    // ---- union channels of the range, ascending, from the channels' mask words; this is also where the
    //      workgroup waits for the up phase of the workgroups that own those channels
    int n = 0;
    for (int j0 = jlo; j0 < jhi; j0 += NT) {
        const int j = j0 + tid;
        uint64_t w = 0;
        unsigned spins = 0;
        for (;;) {
            bool have = true;
            if (j < jhi) {
                w = dec_ld(a.zt + (int64_t)j * ZS);
                have = dec_tagged(w, tag);
            }
            if (__syncthreads_and(have)) break;
            if (dec_give_up(sync, tag, spins)) return;
        }
        const unsigned m = j < jhi ? (uint32_t)w : 0u;
        int total;
        const int pos = block_exclusive_scan<NT>(m != 0 ? 1 : 0, scan_red, &total);
        if (m != 0) {
            list[2 * (n + pos)] = j;
            list[2 * (n + pos) + 1] = (int)m;
        }
        n += total;
    }
    __syncthreads();
    DEC_TRACE(sync, 9);

    const int LPR = seg / CN;                        // lanes per row segment (a power of two <= 64)
    const int RPI = 64 / LPR;                        // rows per load instruction
    const int rr = lane / LPR, ch = lane % LPR;
    const int th = NH == 2 ? wave / NWH : 0, wv = NH == 2 ? wave % NWH : wave;
    const int ngroups = (n + RPI - 1) / RPI;
    const bool lead = LPR >= TB;                     // one lane per (row, token) fetches z' and the row's lanes share it
    float acc[TB][CN];
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int e = 0; e < CN; ++e) acc[t][e] = 0.0f;
    const E* wbase = a.wd + (int64_t)c * seg + ch * CN;
    for (int q0 = wv; q0 < ngroups; q0 += NWH * UNR) {
        u32x4_t w[UNR];
        uint64_t zw[UNR];
        const uint64_t* zaddr[UNR];
        int jrow[UNR];
        unsigned mrow[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int e = (q0 + u * NWH) * RPI + rr;
            const bool valid = (q0 + u * NWH) < ngroups && e < n;
            jrow[u] = valid ? list[2 * e] : 0;
            mrow[u] = valid ? ((unsigned)list[2 * e + 1] >> (th * TB)) & ((1u << TB) - 1u) : 0u;
            w[u] = u32x4_t{0, 0, 0, 0};
            if (valid) w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wbase + (int64_t)jrow[u] * d));
            // lane `ch` of a row fetches the z' of the row's token th * TB + ch
            zaddr[u] = a.zt + (int64_t)jrow[u] * ZS + 1 + th * TB + ch;
            zw[u] = 0;
            if (lead && ch < TB && (mrow[u] >> ch & 1u)) zw[u] = dec_ld(zaddr[u]);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            float z[TB];
            if (lead) {
                float zmine = 0.0f;
                if (ch < TB && (mrow[u] >> ch & 1u)) {
                    unsigned spins = 0;
                    while (!dec_tagged(zw[u], tag)) {         // the word follows its mask word closely; rarely taken
                        if (dec_give_up(sync, tag, spins)) break;
                        zw[u] = dec_ld(zaddr[u]);
                    }
                    zmine = __uint_as_float((uint32_t)zw[u]);
                }
#pragma unroll
                for (int t = 0; t < TB; ++t) z[t] = __shfl(zmine, rr * LPR + t, 64);
            } else {
                // narrow column slices (fewer lanes per row than tokens): every lane reads its row's words
#pragma unroll
                for (int t = 0; t < TB; ++t) {
                    z[t] = 0.0f;
                    if (mrow[u] >> t & 1u) {
                        const uint64_t* za = a.zt + (int64_t)jrow[u] * ZS + 1 + th * TB + t;
                        uint64_t v = dec_ld(za);
                        unsigned spins = 0;
                        while (!dec_tagged(v, tag)) {
                            if (dec_give_up(sync, tag, spins)) break;
                            v = dec_ld(za);
                        }
                        z[t] = __uint_as_float((uint32_t)v);
                    }
                }
            }
            float wf[CN];
            Chunk<E>::unpack(w[u], wf);
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (TB == 1 || __ballot(mrow[u] >> t & 1u) != 0ull) {      // skip tokens none of the rows of this group feeds
#pragma unroll
                    for (int e = 0; e < CN; ++e) acc[t][e] = fmaf(z[t], wf[e], acc[t][e]);
                }
            }
        }
    }
    DEC_TRACE(sync, 10);
    // ---- rows of one instruction sit in different lane groups: add them up (lanes < LPR keep the sums)
    for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int e = 0; e < CN; ++e) acc[t][e] += __shfl_xor(acc[t][e], o, 64);
    }
    if (lane < LPR) {
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int e = 0; e < CN; ++e) red[((size_t)wave * TB + t) * seg + ch * CN + e] = acc[t][e];
    }
    __syncthreads();
    // ---- wavefronts of a token half in a fixed order
    const bool direct = P == 1;
    for (int i = tid; i < B * seg; i += NT) {
        const int b = i / seg, col = i - b * seg;
        const int h = NH == 2 ? b / TB : 0, t = NH == 2 ? b % TB : b;
        float s = 0.0f;
#pragma unroll
        for (int w2 = 0; w2 < NWH; ++w2) s += red[((size_t)(h * NWH + w2) * TB + t) * seg + col];
        if (direct) Elem<E>::store(a.y + (int64_t)b * d + c * seg + col, s);
        else dec_stf(a.part + ((int64_t)p * B + b) * d + c * seg + col, s);
    }
    DEC_TRACE(sync, 11);
    if (direct) return;
    // ---- the last workgroup of this column slice to get here adds the P partials (two workgroups may
    //      both find all flags set; they then write the same values).  The partials are plain
    //      coherent stores, so here the workgroup does wait for their acknowledgement before it
    //      raises its flag.
    dec_drain();
    __syncthreads();
    if (tid < 64) {
        // The flag is set with an exchange and the wavefront waits for its result before it reads the
        // other flags: the exchanges of the P workgroups are ordered at the memory, and the workgroup
        // whose exchange comes last finds every flag set.
        if (tid == 0) {
            const uint64_t old = __hip_atomic_exchange(&sync->dflag[c * P + p], dec_pack(tag, 1u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0)" :: "v"(old) : "memory");
        }
        bool all = true;
        for (int i = lane; i < P; i += 64) all &= dec_tagged(dec_ld(&sync->dflag[c * P + i]), tag);
        const int mine = __all(all) ? 1 : 0;
        if (lane == 0) sh_last = mine;
    }
    __syncthreads();
    if (!sh_last) return;
    for (int i = tid; i < B * seg; i += NT) {
        const int b = i / seg, col = i - b * seg;
        const float* src = a.part + (int64_t)b * d + c * seg + col;
        const int64_t pstride = (int64_t)B * d;
        float s = 0.0f;
        for (int q = 0; q < P; q += 32) {                     // up to 32 loads in flight, added in order
            float v[32];
#pragma unroll
            for (int r = 0; r < 32; ++r) v[r] = q + r < P ? dec_ldf(src + (q + r) * pstride) : 0.0f;
#pragma unroll
            for (int r = 0; r < 32; ++r)
                if (q + r < P) s += v[r];
        }
        Elem<E>::store(a.y + (int64_t)b * d + c * seg + col, s);
    }
}

// End of the call for workgroup 0: once every workgroup has read the generation word (their hello
// words say so), advance it.
__device__ __forceinline__ void dec_finish(DecodeSync* sync, uint32_t tag, uint64_t gen, int nwg) {
    if (blockIdx.x != 0 || threadIdx.x >= 64) return;
    const int lane = threadIdx.x;
    unsigned spins = 0;
    for (;;) {
        bool all = true;
        for (int i = lane; i < nwg; i += 64) all &= dec_tagged(dec_ld(&sync->hello[i]), tag);
        if (__all(all)) break;
        if (dec_give_up(sync, tag, spins)) return;
    }
    if (lane == 0) dec_st(&sync->gen, gen + 1);
}

// ------------------------------------------------------------------ row-per-wavefront variant (B <= 4)
// NT threads, one workgroup per compute unit.  LDS: x [BT, d] of E at 0; own gate values
// [NWV][rmax][BT] floats at off_own; the phase-overlaid area at off_over.
template <class E, int BT, int NT, int NCH>
__global__ __launch_bounds__(NT) void decode_persistent_kernel(DecArgs<E> a) {
    constexpr int CN = Chunk<E>::N, UN = 8, NWV = NT / 64;
    extern __shared__ __align__(16) unsigned char dec_smem[];
    E* xs = reinterpret_cast<E*>(dec_smem);
    float* gown = reinterpret_cast<float*>(dec_smem + a.off_own);
    unsigned char* over = dec_smem + a.off_over;
    __shared__ TopkThreshold thr[BT];
    __shared__ uint64_t sh_gen;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwg = gridDim.x, B = a.B, d = a.d, F = a.F;
    // Channel j belongs to workgroup j % nwg, and the l-th channel of a workgroup (l = j / nwg) to its
    // wavefront l % NWV: every compute unit streams the same number of rows (+-1).
    const int gw = blockIdx.x + wave * nwg, nwt = nwg * NWV;

    // ---- phase G
    u32x4_t cur[UN], nxt[UN];
    auto fetch = [&](u32x4_t (&r)[UN], int j) {
        const E* wrow = a.wg + (int64_t)j * d;
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = (u * 64 + lane) * CN;
            r[u] = u32x4_t{0, 0, 0, 0};
            if (k < d) r[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + k));
        }
    };
    DEC_TRACE(a.sync, 0);
    if (gw < F) fetch(cur, gw);                       // in flight while x is staged
    {
        // all loads of the start-up (first gate row, x, the generation word) are issued before any is used
        constexpr int XI = (BT * 64 * 8 + NT - 1) / NT;          // 16-byte chunks of x per thread (d <= 64 CN 8)
        u32x4_t xv[XI];
#pragma unroll
        for (int q = 0; q < XI; ++q) {
            const int i = (q * NT + tid) * CN;
            xv[q] = u32x4_t{0, 0, 0, 0};
            if (i < BT * d && i / d < B) xv[q] = *reinterpret_cast<const u32x4_t*>(a.x + i);
        }
        uint64_t gen = 0;
        if (tid == 0) gen = dec_ld(&a.sync->gen);
#pragma unroll
        for (int q = 0; q < XI; ++q) {
            const int i = (q * NT + tid) * CN;
            if (i < BT * d) *reinterpret_cast<u32x4_t*>(xs + i) = xv[q];
        }
        if (tid == 0) sh_gen = gen;
    }
    __syncthreads();
    const uint64_t gen = sh_gen;
    const uint32_t tag = dec_make_tag(a.salt, gen);
    if (tid == 0) dec_st(&a.sync->hello[blockIdx.x], dec_pack(tag, 1u));
    DEC_TRACE(a.sync, 1);
    {
        int r = 0;
        for (int j = gw; j < F; j += nwt, ++r) {
            const bool more = j + nwt < F;
            if (more) fetch(nxt, j + nwt);
            float acc[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) acc[b] = 0.0f;
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int k = (u * 64 + lane) * CN;
                if (k < d) {
#pragma unroll
                    for (int b = 0; b < BT; ++b)
                        acc[b] = Chunk<E>::dot(cur[u], *reinterpret_cast<const u32x4_t*>(xs + b * d + k), acc[b]);
                }
            }
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const float s = wave_sum(acc[b]);
                if (lane == 0) {
                    if (b < B) dec_st(a.g2 + (int64_t)b * a.ldF + j, dec_packf(tag, s));
                    gown[(wave * a.rmax + r) * BT + b] = s;
                }
            }
            if (more) {
#pragma unroll
                for (int u = 0; u < UN; ++u) cur[u] = nxt[u];
            }
        }
    }
    __syncthreads();                                   // own gate values visible to the whole workgroup
    DEC_TRACE(a.sync, 2);

    // ---- phase S
    if (!dec_phase_select<BT, NT, NCH>(a, over, thr, tag)) return;
    DEC_TRACE(a.sync, 5);

    // ---- phase U: own row i = r * NWV + wave is channel gw + r * nwt
    const int rmax = a.rmax;
    auto rows = [&](int i, int& j, const float*& gp) {
        const int r = i / NWV;
        j = gw + r * nwt;
        gp = gown + (wave * rmax + r) * BT;
        if (j >= F) j = -1;
    };
    dec_phase_up<E, BT, NWV>(a, dec_smem, d * (int)sizeof(E), rmax * NWV, rows, thr, tag);
    __syncthreads();                                   // x and the own gate values are dead from here
    DEC_TRACE(a.sync, 6);

    // ---- phase D (its LDS area starts at 0)
    dec_phase_down<E, BT, NT>(a, dec_smem, tag);
    DEC_TRACE(a.sync, 12);
    dec_finish(a.sync, tag, gen, nwg);
    DEC_TRACE_END(a.sync);
}

// ------------------------------------------------------------------------- MFMA variant (5..16 tokens)
// bf16, 768 threads = 3 row groups x 4 shares of the contraction (the gate phase is that of
// decode_gate_mfma_kernel<0, 3, 4, 16, 4>); a workgroup owns blocks of 48 consecutive channels.
// LDS: x [16, d] with rows padded by 16 bytes at 0; own gate tiles [rmax][48][17] floats at off_own;
// the phase-overlaid area (MFMA partial tiles, selection) at off_over.
template <int NCH>
__global__ __launch_bounds__(768) void decode_persistent_mfma_kernel(DecArgs<bf16_t> a) {
    constexpr int RG = 3, KS = 4, BTOK = 16, UN = 4, NT = 768, NWV = 12, ROWS = 48, BT = 16;
    extern __shared__ __align__(16) unsigned char dec_smem[];
    float* gown = reinterpret_cast<float*>(dec_smem + a.off_own);
    unsigned char* over = dec_smem + a.off_over;
    float* red = reinterpret_cast<float*>(over);                       // [RG][KS][256]
    __shared__ TopkThreshold thr[BT];
    __shared__ uint64_t sh_gen;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwg = gridDim.x, B = a.B, d = a.d, F = a.F;
    const int xpitch = d * 2 + 16;
    const int rg = wave / KS, ks = wave % KS;
    const int kq = d / KS, q = lane >> 4;
    const int nblk = (F + ROWS - 1) / ROWS;

    // ---- phase G
    DEC_TRACE(a.sync, 0);
    if (tid == 0) sh_gen = dec_ld(&a.sync->gen);
    for (int i = tid * 8; i < BTOK * d; i += NT * 8) {
        const int b = i / d, k = i - b * d;
        u32x4_t v = {0, 0, 0, 0};
        if (b < B) v = *reinterpret_cast<const u32x4_t*>(a.x + i);
        *reinterpret_cast<u32x4_t*>(dec_smem + b * xpitch + k * 2) = v;
    }
    __syncthreads();
    const uint64_t gen = sh_gen;
    const uint32_t tag = dec_make_tag(a.salt, gen);
    if (tid == 0) dec_st(&a.sync->hello[blockIdx.x], dec_pack(tag, 1u));
    DEC_TRACE(a.sync, 1);
    const unsigned char* xl = dec_smem + (lane & 15) * xpitch + (ks * kq + q * 16) * 2;
    const int nstep = kq / 64;
    int it = 0;
    for (int blk = blockIdx.x; blk < nblk; blk += nwg, ++it) {
        const int row0 = blk * ROWS + rg * 16;
        const bf16_t* wrow = a.wg + (int64_t)min(row0 + (lane & 15), F - 1) * d + ks * kq + q * 16;
        u32x4_t w0[UN], w1[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            w0[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + u * 64));
            w1[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + u * 64 + 8));
        }
        f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int s0 = 0; s0 < nstep; s0 += UN) {
            u32x4_t c0[UN], c1[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) { c0[u] = w0[u]; c1[u] = w1[u]; }
            if (s0 + UN < nstep) {
                const int nx = min(s0 + UN, nstep - UN);
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    w0[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + (nx + u) * 64));
                    w1[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow + (nx + u) * 64 + 8));
                }
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                if (s0 + u < nstep) {
                    const u32x4_t x0 = *reinterpret_cast<const u32x4_t*>(xl + (s0 + u) * 128);
                    const u32x4_t x1 = *reinterpret_cast<const u32x4_t*>(xl + (s0 + u) * 128 + 16);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dec_bf16x8_t, c0[u]),
                                                                  __builtin_bit_cast(dec_bf16x8_t, x0), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dec_bf16x8_t, c1[u]),
                                                                  __builtin_bit_cast(dec_bf16x8_t, x1), acc, 0, 0, 0);
                }
            }
        }
        // acc[r] = D[row 4*(lane/16) + r][token lane % 16] over this wavefront's share of k
        *reinterpret_cast<f32x4_t*>(red + ((rg * KS + ks) * 64 + lane) * 4) = acc;
        __syncthreads();
        if (ks == 0) {
            f32x4_t s = acc;
#pragma unroll
            for (int o = 1; o < KS; ++o) s += *reinterpret_cast<const f32x4_t*>(red + ((rg * KS + o) * 64 + lane) * 4);
            const int b = lane & 15, r = row0 + 4 * (lane >> 4);
            if (b < B) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (r + e < F) dec_st(a.g2 + (int64_t)b * a.ldF + r + e, dec_packf(tag, s[e]));
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) gown[((it * ROWS) + rg * 16 + 4 * (lane >> 4) + e) * 17 + b] = s[e];
        }
        __syncthreads();
    }
    DEC_TRACE(a.sync, 2);

    // ---- phase S
    if (!dec_phase_select<BT, NT, NCH>(a, over, thr, tag)) return;
    DEC_TRACE(a.sync, 5);

    // ---- phase U: own row i = it * 48 + local row
    const int nown = it * ROWS;
    auto rows = [&](int i, int& j, const float*& gp) {
        const int t = i / ROWS, lr = i - t * ROWS;
        j = (blockIdx.x + t * nwg) * ROWS + lr;
        gp = gown + (size_t)i * 17;
        if (j >= F) j = -1;
    };
    dec_phase_up<bf16_t, BT, NWV>(a, dec_smem, xpitch, nown, rows, thr, tag);
    __syncthreads();                                   // x and the own gate values are dead from here
    DEC_TRACE(a.sync, 6);

    // ---- phase D (its LDS area starts at 0)
    dec_phase_down<bf16_t, BT, NT>(a, dec_smem, tag);
    DEC_TRACE(a.sync, 12);
    dec_finish(a.sync, tag, gen, nwg);
    DEC_TRACE_END(a.sync);
}

}  // namespace moc
