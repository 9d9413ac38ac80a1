// bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16).
//
//   C[m, n] = sum_k A(m, k) B(n, k)   (+ a second operand pair accumulated into the same tile)
//
// Each operand is read in the layout it already has in memory:
//   k-contiguous ("KC"): element (r, k) at P[r * ld + k]   -- x, dy, the weights for X W^T products
//   k-major      ("KM"): element (r, k) at P[k * ld + r]   -- the same arrays when the contraction
//                                                             runs over their row index
// so no transposed copies are ever made.  KC tiles are staged in LDS as [row][k] and fragments are
// plain 16-byte reads; KM tiles are staged as [k][row] exactly as they lie in memory and fragments
// come from two ds_read_b64_tr_b16 transposing reads (each gives a lane 4 consecutive k of one row).
//
// One workgroup of NWV wavefronts (4 or 8) computes a BM x BN tile; its 2 x (NWV/2) wavefronts each
// own a (BM/2) x (BN/(NWV/2)) sub-tile of 32x32 MFMA blocks.  k-slices of 32 are staged global -> registers
// -> LDS through three LDS stages: while slice t is multiplied, slice t+1 is already visible in
// LDS, slice t+2 is being written and slices t+3 .. t+2+NSETS are in flight from global memory.  One barrier per
// slice.  Fragment registers are double-buffered so LDS reads overlap the MFMAs of the previous
// half-slice; sched_group_barrier pins that interleaving.
//
// Operand roles: the B rows (n) feed the MFMA "A" input and the A rows (m) the MFMA "B" input, so
// a lane ends up with four consecutive n for one m -- the shape the epilogues want.
//
// Requirements checked by the host: 16-byte aligned bases, leading dimensions multiples of 8,
// contraction lengths >= 32; a KM operand must be readable up to `ext` columns (multiple of 8).
// Contraction lengths that are not multiples of 32 take one of two tail modes:
//   TAILMODE 2 ("padded"): one operand is KC, readable and zero up to the next multiple of 32
//     (the library's own dense intermediates are), the other is KM: the KM k-rows past the end
//     are clamped to the last row and meet those zeros.  Nearly free.
//   TAILMODE 1 (general): the last slice re-reads the final 32-wide window (8-aligned, so a KC
//     operand must be readable and zero up to the next multiple of 8) and zeroes what lies
//     before the part still to be accumulated or past the end; KM rows are clamped as well.
#pragma once
#include <type_traits>

#include "common.h"
#include "gemm_generic.h"
#include "kernel_attrs.h"

namespace moc {

typedef GemmProblem<bf16_t> MfmaProblem;

constexpr int kMfmaBK = 32;
constexpr int kMfmaStages = 3;

// LDS byte offset of the 16-byte chunk `ch` (8 k) of row `row` in a k-contiguous tile: rows of 64
// bytes, chunk position XORed with bits 2..3 of the row.  Both the staging writes (16 lanes = 4
// rows x 4 chunks) and the fragment reads (16 lanes = 16 rows, one chunk) then hit 16 different
// 16-byte bank groups.
__device__ __forceinline__ int kc_lds_offset(int row, int ch) {
    return row * 64 + ((ch ^ ((row >> 2) & 3)) << 4);
}

template <int ROWS, bool KM> struct OperandTile {
    static constexpr int kPitch = KM ? (ROWS * 2 + 64) : kMfmaBK * 2;   // bytes
    static constexpr int kBytes = KM ? kMfmaBK * kPitch : ROWS * kPitch;
    static constexpr int kChunks64 = ROWS * kMfmaBK / 8 / 64;                   // 16-byte chunks per lane of one wavefront
};

template <int BM, int BN, bool AKM, bool BKM> struct MfmaCfg {
    using TA = OperandTile<BM, AKM>;
    using TB = OperandTile<BN, BKM>;
    static constexpr int kStage = TA::kBytes + TB::kBytes;
    static constexpr int kLds = kMfmaStages * kStage;
};

typedef short s16x4_t __attribute__((ext_vector_type(4)));

// Fragment of 32 rows x 16 k for one MFMA input: lane l gets row (l % 32), k = 8 * (l / 32) .. + 8.
template <bool KM, int PITCH>
__device__ __forceinline__ bf16x8_t read_fragment(const unsigned char* tile, int row0, int kk, int lane) {
    if (!KM) {
        return *reinterpret_cast<const bf16x8_t*>(tile + kc_lds_offset(row0 + (lane & 31), kk * 2 + (lane >> 5)));
    } else {
        // 16-lane groups: lanes 4q..4q+3 of a group address k-row q (4 x 8 bytes = 16 rows); the
        // transposing read hands lane i of the group the 4 k-values of row i.
        const int krow = kk * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
        const int col = row0 + 16 * ((lane >> 4) & 1) + (lane & 3) * 4;
        const unsigned char* p = tile + krow * PITCH + col * 2;
        typedef s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
        s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
        s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * PITCH));
        typedef short s16x8_t __attribute__((ext_vector_type(8)));
        s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8_t, v);
    }
}

// Emits a sched_group_barrier sequence for N MFMAs: after MFMA number R come the share of `n`
// instructions of one class (mask) whose window is MFMA slots [a, b).
template <int R, int A, int B, int N_> struct SchedShare {
    static constexpr int value = (R >= A && R < B) ? ((R - A + 1) * N_ / (B - A) - (R - A) * N_ / (B - A)) : 0;
};
template <int R, int N, int RA, int RB, int NR, int WA, int WB, int NW, int VA, int VB, int NV> struct SchedSeq {
    static __device__ __forceinline__ void apply() {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                   // one MFMA
        constexpr int r = SchedShare<R, RA, RB, NR>::value;
        constexpr int w = SchedShare<R, WA, WB, NW>::value;
        constexpr int v = SchedShare<R, VA, VB, NV>::value;
        if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);             // LDS reads
        if constexpr (w > 0) __builtin_amdgcn_sched_group_barrier(0x200, w, 0);             // LDS writes
        if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);             // global loads
        if constexpr (R + 1 < N) SchedSeq<R + 1, N, RA, RB, NR, WA, WB, NW, VA, VB, NV>::apply();
    }
};

// Workgroup g of `total` runs on XCD g % 8.  Gives every XCD a contiguous range of the logical work
// items 0 .. total-1, so that neighbouring items (tiles that share operand panels) meet in one L2.
__device__ __forceinline__ int xcd_contiguous_index(int g, int total) {
    const int xcd = g & 7, local = g >> 3;
    return xcd * (total >> 3) + min(xcd, total & 7) + local;
}

// What a workgroup needs to know about the tile it works on (all uniform except the two offset arrays).
// [ks, ke) is the range of k-slices of the tile that this workgroup multiplies (all of them unless the
// work is split along k, see StreamKArgs).
template <int LA, int LB> struct MfmaTileCtx {
    const bf16_t *ap, *ap2, *bp, *bp2;
    int lda, ldb, Kc, Kc2, nk0, nk, ks, ke;
    int M, N, m0, n0;
    int a_off[LA], b_off[LB];
};

// Splitting the work along k ("stream-K").  The k-slices of all tiles, tile after tile, form one sequence
// of units; workgroup rank r (ranks are contiguous per XCD) takes the units [start(r), start(r + 1)), so every
// workgroup gets the same amount of work whatever the number of tiles, and the workgroups reach their
// epilogues at different times instead of all at once.  A tile whose slices fall to several workgroups is
// summed along a chain that runs from its last slices to its first: a workgroup whose share does not reach the
// end of the tile starts from the accumulators that rank r + 1 left in its slot of `part` (announced by
// `tag` in its word of `flag`, which the reader sets back to zero) instead of from zero, and a workgroup whose
// share does not start the tile writes its accumulators to its own slot instead of running the epilogue.  The
// order of the additions is fixed, so results do not depend on timing.  Rank r + 1's share is the first thing it
// does and rank r's share of the same tile the last, so in normal operation nobody waits; should the word not
// arrive within spin_limit polls (a workgroup that the hardware has not started yet), the reader multiplies
// the rest of the tile itself, which gives the same sum up to the order of additions.  `tag` is nonzero and
// differs from launch to launch, and the words are left at zero, so `flag` needs no initialisation (a stale word
// equals a fresh tag with probability 2^-64) and a captured launch can be replayed.
struct StreamKArgs {
    float* part;                 // one BM x BN fp32 slot per workgroup
    unsigned long long* flag;    // one word per workgroup
    unsigned long long tag;
    int snap;                    // a boundary closer than this many slices to a tile boundary moves onto it
    int spin_limit;
};

// Slot traffic goes past the caches that are not coherent across workgroups (the compute unit's L1 and,
// between XCDs, the L2): stores are written through and loads fetched at device scope.  Fences would do as
// well but cost far more here: a device-scope release writes back the whole L2 (which is full of freshly
// written output tiles) and an acquire drops every clean line of the operand panels the XCD is sharing.
// The loads are issued without waiting: a "s_waitcnt vmcnt(0)" must follow before their values are used.
__device__ __forceinline__ void streamk_store16(unsigned char* base, uint32_t lane_off, f32x4_t v) {
    asm volatile("global_store_dwordx4 %0, %1, %2 sc0 sc1" : : "v"(lane_off), "a"(v), "s"(base) : "memory");
}
__device__ __forceinline__ f32x4_t streamk_load16(const unsigned char* base, uint32_t lane_off) {
    f32x4_t v;
    asm volatile("global_load_dwordx4 %0, %1, %2 sc0 sc1" : "=a"(v) : "v"(lane_off), "s"(base) : "memory");
    return v;
}
// First unit of rank r when `units` units (nk per tile) are dealt to `ranks` workgroups.
__device__ __forceinline__ int streamk_start(int r, int ranks, int units, int nk, int snap) {
    if (r >= ranks) return units;
    int s = (int)((long long)r * units / ranks);
    const int off = s % nk;
    if (off < snap) s -= off;
    else if (off > nk - snap) s += nk - off;
    return s;
}

// Output tiles item_first, item_first + item_stride, ... < item_total of the problems prs[0 .. ] (all of
// one shape: tiles_m x tiles_n tiles each, problem z owning items z * tiles_m * tiles_n ...), workgroup-wide.
// With xcd_map the item numbers are first sent through xcd_contiguous_index (item_stride must then be a
// multiple of 8, or the workgroup has a single item).  A workgroup that has several tiles issues the
// global loads of the next tile's first two k-slices before it writes the current tile out, so that the
// epilogue and the next prologue overlap; one barrier separates the epilogue's use of the stage memory
// from the next tile's staging.
template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NWV, int NSETS, bool SK = false, bool MULTI = true>
__device__ __forceinline__ void gemm_bf16_mfma_tiles(const MfmaProblem* prs, const Epi* epis, int tiles_m, int tiles_n,
                                                     int item_first, int item_stride, int item_total, bool xcd_map,
                                                     const StreamKArgs* sk = nullptr) {
    using Cfg = MfmaCfg<BM, BN, AKM, BKM>;
    using TA = typename Cfg::TA;
    using TB = typename Cfg::TB;
    constexpr int BK = kMfmaBK;
    constexpr int NT = NWV * 64;
    constexpr int WAVES_N = NWV / 2;                   // wavefronts form a 2 x (NWV/2) grid over the tile
    constexpr int WM = BM / 2, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must consist of 32x32 blocks");
    constexpr int LA = TA::kChunks64 / NWV, LB = TB::kChunks64 / NWV;
    static_assert(LA >= 1 && LB >= 1, "tile too small for this many threads");
    using Ctx = MfmaTileCtx<LA, LB>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int nblk = tiles_m * tiles_n;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

    // ---- staging assignment (the same for every tile).  KC: chunk c -> (row c / 4, k chunk c % 4); rows
    //      past the edge are clamped.  KM: chunk c -> (k row c / (ROWS/8), column chunk c % (ROWS/8));
    //      columns past the readable extent are clamped.
    int a_lds[LA], a_k[LA], b_lds[LB], b_k[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int c = tid + i * NT;
        if (!AKM) {
            a_lds[i] = kc_lds_offset(c >> 2, c & 3);
            a_k[i] = (c & 3) * 8;
        } else {
            a_lds[i] = (c / (BM / 8)) * TA::kPitch + (c % (BM / 8)) * 16;
            a_k[i] = c / (BM / 8);
        }
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int c = tid + i * NT;
        if (!BKM) {
            b_lds[i] = TA::kBytes + kc_lds_offset(c >> 2, c & 3);
            b_k[i] = (c & 3) * 8;
        } else {
            b_lds[i] = TA::kBytes + (c / (BN / 8)) * TB::kPitch + (c % (BN / 8)) * 16;
            b_k[i] = c / (BN / 8);
        }
    }

    // ---- tile order inside a problem: bands of GROUP tile-rows, column by column inside a band, so that a
    //      contiguous range of tiles (one XCD's share) touches few distinct operand panels.
    auto setup = [&](Ctx& t, int item, int& z) {
        const int mapped = (xcd_map && !SK) ? xcd_contiguous_index(item, item_total) : item;
        z = mapped / nblk;
        const int logical = mapped - z * nblk;
        const MfmaProblem& pr = prs[z];
        // band height, measured: at the 1B shape (22 tile columns) heights 2 / 4 / 6 / 8 / 16 give 1.591 / 1.596 / 1.599 / 1.605 /
        // 1.619 ms per layer step and 425 / 280 / 312 / 291 / 463 MB beyond L2 for the gate product; at the 7B shape (43 tile
        // columns) 8 is ahead of 4 and 2 (gate + up 1.285 / 1.294 / 1.299 ms)
        const int GROUP = tiles_n >= 32 ? 8 : 4;
        const int band = logical / (GROUP * tiles_n);
        const int first_m = band * GROUP;
        const int gsz = min(tiles_m - first_m, GROUP);
        const int in_band = logical - band * GROUP * tiles_n;
        t.M = pr.M; t.N = pr.N;
        t.m0 = (first_m + in_band % gsz) * BM;
        t.n0 = (in_band / gsz) * BN;
        t.ap = pr.A.p; t.ap2 = pr.A.p2; t.bp = pr.B.p; t.bp2 = pr.B.p2;
        t.lda = (int)pr.A.ld; t.ldb = (int)pr.B.ld;
        t.Kc = pr.Kc; t.Kc2 = pr.Kc2;
        t.nk0 = (pr.Kc + BK - 1) / BK;
        t.nk = t.nk0 + (pr.Kc2 + BK - 1) / BK;
        t.ks = 0;
        t.ke = t.nk;
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int c = tid + i * NT;
            if (!AKM) t.a_off[i] = min(t.m0 + (c >> 2), t.M - 1) * t.lda + (c & 3) * 8;
            else t.a_off[i] = min(t.m0 + (c % (BM / 8)) * 8, pr.A.ext - 8);
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int c = tid + i * NT;
            if (!BKM) t.b_off[i] = min(t.n0 + (c >> 2), t.N - 1) * t.ldb + (c & 3) * 8;
            else t.b_off[i] = min(t.n0 + (c % (BN / 8)) * 8, pr.B.ext - 8);
        }
    };

    u32x4_t ga[NSETS][LA], gb[NSETS][LB];   // NSETS slices in flight from global memory
    [[maybe_unused]] uint32_t gz[NSETS];    // TAILMODE 1: which of a set's chunks are to be zeroed (A chunks in bits 0 .. LA-1, then B)
    // global -> registers for the kt-th k-slice of this workgroup's share of tile t (clamped to the last one so
    // the loop body has no branch)
    auto fetch = [&](const Ctx& t, int buf, int kt) {
        kt = min(t.ks + kt, t.ke - 1);
        const bool seg = kt >= t.nk0;
        const int klen = seg ? t.Kc2 : t.Kc;
        const int kwant = (seg ? kt - t.nk0 : kt) * BK;                                  // first k still to accumulate
        const int kfrom = TAILMODE == 1 ? min(kwant, ((klen + 7) & ~7) - BK) : kwant;   // first k read
        const int klast = klen - 1 - kfrom;                                              // last valid k row of this slice
        // TAILMODE 1: the chunks of this slice that lie before the part still to accumulate or past the end are
        // zeroed when the slice goes to LDS, not here: a select on a value just loaded would make the wavefront
        // wait for the load at once and undo the prefetch
        [[maybe_unused]] uint32_t zero = 0;
        const bf16_t* ap = (seg ? t.ap2 : t.ap) + (AKM ? (int64_t)kfrom * t.lda : (int64_t)kfrom);
        const bf16_t* bp = (seg ? t.bp2 : t.bp) + (BKM ? (int64_t)kfrom * t.ldb : (int64_t)kfrom);
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            int off = t.a_off[i];
            if (AKM) off += (TAILMODE ? min(a_k[i] * t.lda, klast * t.lda) : a_k[i] * t.lda);
            // uniform base + unsigned 32-bit byte offset: the load takes the base from scalar registers
            ga[buf][i] = *reinterpret_cast<const u32x4_t*>(reinterpret_cast<const unsigned char*>(ap) + (uint32_t)off * 2u);
            if (TAILMODE == 1) {
                const int k = kfrom + a_k[i];
                if (k < kwant || k >= klen) zero |= 1u << i;
            }
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            int off = t.b_off[i];
            if (BKM) off += (TAILMODE ? min(b_k[i] * t.ldb, klast * t.ldb) : b_k[i] * t.ldb);
            gb[buf][i] = *reinterpret_cast<const u32x4_t*>(reinterpret_cast<const unsigned char*>(bp) + (uint32_t)off * 2u);
            if (TAILMODE == 1) {
                const int k = kfrom + b_k[i];
                if (k < kwant || k >= klen) zero |= 1u << (LA + i);
            }
        }
        if (TAILMODE == 1) gz[buf] = zero;
    };
    auto stash = [&](int buf, int stage) {
        unsigned char* base = smem + stage * Cfg::kStage;
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            u32x4_t v = ga[buf][i];
            if (TAILMODE == 1 && ((gz[buf] >> i) & 1u)) v = u32x4_t{0, 0, 0, 0};
            *reinterpret_cast<u32x4_t*>(base + a_lds[i]) = v;
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            u32x4_t v = gb[buf][i];
            if (TAILMODE == 1 && ((gz[buf] >> (LA + i)) & 1u)) v = u32x4_t{0, 0, 0, 0};
            *reinterpret_cast<u32x4_t*>(base + b_lds[i]) = v;
        }
    };

    f32x16_t acc[TM][TN];
    constexpr int NREAD = TN * (BKM ? 2 : 1) + TM * (AKM ? 2 : 1);    // LDS reads per half slice
    bf16x8_t fm[2][TM], fn[2][TN];
    auto load_frags = [&](int buf, int stage, int kk) {
        const unsigned char* base = smem + stage * Cfg::kStage;
        // order of use by mma(): fm[0] with every fn[j] first, then fm[1], ...
        fm[buf][0] = read_fragment<AKM, TA::kPitch>(base, wm0, kk, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fn[buf][j] = read_fragment<BKM, TB::kPitch>(base + TA::kBytes, wn0 + j * 32, kk, lane);
#pragma unroll
        for (int i = 1; i < TM; ++i) fm[buf][i] = read_fragment<AKM, TA::kPitch>(base, wm0 + i * 32, kk, lane);
    };
    auto mma = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fn[buf][j], fm[buf][i], acc[i][j], 0, 0, 0);
    };

    Ctx cur, nxt;
    int zc = 0, zn = 0;
    int item = item_first;
    // split along k: item_first is the workgroup's number and item_stride the number of workgroups; the
    // workgroup owns the units [u, u_end)
    [[maybe_unused]] int rank = 0, ranks = 0, units = 0, nk_all = 0, u = 0, u_end = 0;
    __shared__ int sk_ok;
    auto sk_start = [&](int r) { return streamk_start(r, ranks, units, nk_all, sk->snap); };
    // Slot of rank r.  Piece p (16 bytes per lane) of a slot lies at p * NT * 16 + tid * 16: a uniform base, which
    // is kept opaque so that the 64 piece addresses are formed where they are used (scalar adds) rather than
    // all ahead of the tile loop, plus one per-lane offset.
    auto sk_slot = [&](int r) {
        unsigned char* q = reinterpret_cast<unsigned char*>(sk->part) + (size_t)r * (BM * BN * sizeof(float));
        asm volatile("" : "+s"(q));
        return q;
    };
    auto sk_advance = [&](unsigned char*& q) {      // next piece; opaque for the same reason
        q += NT * 16;
        asm volatile("" : "+s"(q));
    };
    [[maybe_unused]] const uint32_t sk_lane = (uint32_t)tid * 16u;
    if constexpr (SK) {
        nk_all = (prs[0].Kc + BK - 1) / BK + (prs[0].Kc2 + BK - 1) / BK;
        ranks = item_stride;
        rank = xcd_contiguous_index(item_first, ranks);
        units = item_total * nk_all;
        u = sk_start(rank);
        u_end = sk_start(rank + 1);
        if (u >= u_end) return;
        item = u / nk_all;
        setup(cur, item, zc);
        cur.ks = u - item * nk_all;
        cur.ke = min(nk_all, cur.ks + (u_end - u));
    } else {
        if (item >= item_total) return;
        setup(cur, item, zc);
    }
    fetch(cur, 0, 0);
    fetch(cur, 1, 1);
    for (;;) {
        [[maybe_unused]] bool from_slot = false;
        if constexpr (SK) {
            if (cur.ke < cur.nk) {
                // the rest of this tile is rank + 1's: start from the accumulators it left (its share and whatever
                // followed it), or take the rest over if they do not arrive
                if (tid == 0) {
                    int ok = 0;
                    for (int it = 0; it < sk->spin_limit; ++it) {
                        if (__hip_atomic_load(sk->flag + rank + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == sk->tag) {
                            ok = 1;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(4);
                    }
                    sk_ok = ok;
                }
                __syncthreads();
                from_slot = sk_ok != 0;
                if (from_slot) {
                    // all 64 loads of a lane go out before the one wait; the values are handed on only after it
                    unsigned char* src = sk_slot(rank + 1);
                    f32x4_t t[TM * TN * 4];
#pragma unroll
                    for (int p = 0; p < TM * TN * 4; ++p) {
                        t[p] = streamk_load16(src, sk_lane);
                        sk_advance(src);
                    }
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
#pragma unroll
                            for (int ii = 0; ii < 4; ++ii) {
                                f32x4_t v = t[(i * TN + j) * 4 + ii];
                                asm volatile("" : "+a"(v));
#pragma unroll
                                for (int e = 0; e < 4; ++e) acc[i][j][4 * ii + e] = v[e];
                            }
                } else {
                    cur.ke = cur.nk;
                }
                __syncthreads();           // sk_ok and the slot have been read by every wavefront
                if (from_slot && tid == 0) __hip_atomic_store(sk->flag + rank + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (!from_slot) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
        }

        // ---- prologue: slices 0 and 1 (already on their way) into LDS, slices 2 .. NSETS+1 into registers
        stash(0, 0);
        stash(1, 1);
#pragma unroll
        for (int i = 0; i < NSETS; ++i) fetch(cur, i, 2 + i);
        __syncthreads();
        load_frags(0, 0, 0);

        int st_cur = 0, st_next = 1, st_fill = 2;
        // One k-slice.  On entry fragment buffer 0 holds the first half of slice kt; register set
        // `buf` holds slice kt+2.  LDS reads are issued ahead of the LDS writes in program order (the
        // compiler cannot tell the stages apart) and everything is spread between the MFMAs.
        auto slice = [&](auto buf_c, int kt) {
            constexpr int buf = decltype(buf_c)::value;
            load_frags(1, st_cur, 1);       // second half of slice kt
            stash(buf, st_fill);            // slice kt+2 -> LDS (its stage was last read in slice kt-1)
            mma(0);
            fetch(cur, buf, kt + 2 + NSETS);     // slice kt+2+NSETS -> registers
            load_frags(0, st_next, 0);      // first half of slice kt+1 (visible since the last barrier)
            mma(1);
            // first half: the fragment reads go out with the first quarter of the MFMAs, the LDS writes
            // with the rest; second half: fragment reads with the first half of the MFMAs, global loads
            // spread over all of them (measured best of several spreads).
            constexpr int NM = TM * TN;
            SchedSeq<0, NM, 0, NM / 4, NREAD, NM / 4, NM, LA + LB, 0, 0, 0>::apply();
            SchedSeq<0, NM, 0, NM / 2, NREAD, 0, 0, 0, 0, NM, LA + LB>::apply();
            __syncthreads();
            const int t = st_cur;
            st_cur = st_next;
            st_next = st_fill;
            st_fill = t;
        };
        const int nk = cur.ke - cur.ks;
        int kt = 0;
        for (; kt + NSETS <= nk; kt += NSETS) {
            slice(std::integral_constant<int, 0>{}, kt);
            slice(std::integral_constant<int, 1>{}, kt + 1);
            if constexpr (NSETS > 2) slice(std::integral_constant<int, 2>{}, kt + 2);
            if constexpr (NSETS > 3) slice(std::integral_constant<int, 3>{}, kt + 3);
        }
        if (kt < nk) slice(std::integral_constant<int, 0>{}, kt++);
        if (kt < nk) slice(std::integral_constant<int, 1>{}, kt++);
        if constexpr (NSETS > 3)
            if (kt < nk) slice(std::integral_constant<int, 2>{}, kt++);

        // ---- the next tile's first two slices go out before this tile is written
        int next_item = item + item_stride;
        bool more = MULTI && next_item < item_total;      // (MULTI = false: a single tile, the walk over tiles compiled out)
        [[maybe_unused]] bool contributed = false;
        if constexpr (SK) {
            u += nk;
            next_item = item + 1;
            more = u < u_end;
            if (cur.ks > 0) {
                // a share that does not start the tile: the accumulators go to this workgroup's slot, 1 KB per
                // store instruction, in the layout they are read back in
                unsigned char* dst = sk_slot(rank);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int ii = 0; ii < 4; ++ii) {
                            streamk_store16(dst, sk_lane, f32x4_t{acc[i][j][4 * ii], acc[i][j][4 * ii + 1], acc[i][j][4 * ii + 2],
                                                                  acc[i][j][4 * ii + 3]});
                            sk_advance(dst);
                        }
                // every wavefront waits until its stores have been written through, then one thread publishes
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                if (tid == 0) __hip_atomic_store(sk->flag + rank, sk->tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                contributed = true;
            }
        }
        if (more) {
            setup(nxt, next_item, zn);
            if constexpr (SK) nxt.ke = min(nk_all, u_end - u);
            fetch(nxt, 0, 0);
            fetch(nxt, 1, 1);
        }

        // ---- epilogue.  acc[i][j][4*ii + r] is C[m, n] with m = .. + lane % 32 and n = .. + 8*ii +
        //      4*(lane/32) + r: a lane owns 4 consecutive n of 32 different rows, which would make
        //      scattered 8/16-byte global stores.  Each wave therefore turns its 32-row blocks around
        //      in a private LDS area (the stages are free after the last barrier) and hands the
        //      epilogue functor whole row segments: 32 lanes x 4 columns = 128 consecutive columns.
        //      Wave tiles whose row segments do not divide the 64 lanes (96 columns: 24 lanes per row,
        //      16 lanes idle) store straight from the accumulator layout instead, which measured faster
        //      for them: 16 or 32 contiguous bytes per row and store instruction.
        const Epi& epi = epis[zc];
        const int M = cur.M, m0 = cur.m0, n0 = cur.n0;
        constexpr bool kDirectStores = 64 % (WN / 4) != 0;
        if (SK && contributed) {
            // nothing to write: the finisher of this tile does
        } else if constexpr (kDirectStores) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int ii = 0; ii < 4; ++ii) {
                        const int m = m0 + wm0 + i * 32 + (lane & 31);
                        const int n = n0 + wn0 + j * 32 + 8 * ii + 4 * (lane >> 5);
                        const float v[4] = {acc[i][j][4 * ii], acc[i][j][4 * ii + 1], acc[i][j][4 * ii + 2], acc[i][j][4 * ii + 3]};
                        if (m < M) epi.store4(m, n, v);
                    }
        } else {
            constexpr int EPITCH = WN * 4 + 16;                       // bytes per staged row (fp32)
            static_assert(NWV * 32 * EPITCH <= Cfg::kLds, "epilogue staging must fit in the stage memory");
            unsigned char* area = smem + wave * (32 * EPITCH);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int ii = 0; ii < 4; ++ii) {
                        const int col = j * 32 + 8 * ii + 4 * (lane >> 5);
                        *reinterpret_cast<f32x4_t*>(area + (lane & 31) * EPITCH + col * 4) =
                            f32x4_t{acc[i][j][4 * ii], acc[i][j][4 * ii + 1], acc[i][j][4 * ii + 2], acc[i][j][4 * ii + 3]};
                    }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                constexpr int LPR = WN / 4;                            // lanes per staged row
                constexpr int RPI = 64 / LPR;                          // rows per instruction
#pragma unroll 4
                for (int it = 0; it < 32 / RPI; ++it) {
                    const int row = it * RPI + lane / LPR, c4 = lane % LPR;
                    if (64 % LPR != 0 && lane >= RPI * LPR) continue;    // lanes beyond the last whole row
                    const f32x4_t t = *reinterpret_cast<const f32x4_t*>(area + row * EPITCH + c4 * 16);
                    const int m = m0 + wm0 + i * 32 + row;
                    const float v[4] = {t[0], t[1], t[2], t[3]};
                    if (m < M) epi.store4(m, n0 + wn0 + c4 * 4, v);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
        if (!more) break;
        __syncthreads();                   // every wavefront is done with the stage memory
        cur = nxt;
        zc = zn;
        item = next_item;
    }
}

// One output tile of one problem (`logical` is its position in the band order).
template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NWV, int NSETS>
__device__ __forceinline__ void gemm_bf16_mfma_tile(const MfmaProblem& pr, int tiles_m, int tiles_n, const Epi& epi,
                                                    int logical) {
    gemm_bf16_mfma_tiles<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS, false, false>(&pr, &epi, tiles_m, tiles_n, logical, 1 << 30,
                                                                                    tiles_m * tiles_n, false);
}

// The grid is either one workgroup per tile or, when there are more tiles than the chip holds workgroups,
// a multiple of 8 workgroups that each walk over several tiles (persistent).
template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NWV = 4, int NSETS = 2>
__global__ __launch_bounds__(NWV * 64) void gemm_bf16_mfma_kernel(MfmaProblem pr, int tiles_m, int tiles_n, Epi epi) {
    gemm_bf16_mfma_tiles<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS>(&pr, &epi, tiles_m, tiles_n, blockIdx.x, gridDim.x,
                                                                      tiles_m * tiles_n, true);
}

// The same with the work split along k (see StreamKArgs); the grid is a multiple of 8 workgroups, all resident.
template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NWV = 4, int NSETS = 2>
__global__ __launch_bounds__(NWV * 64) void gemm_bf16_mfma_streamk_kernel(MfmaProblem pr, int tiles_m, int tiles_n, Epi epi,
                                                                          StreamKArgs sk) {
    gemm_bf16_mfma_tiles<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS, true>(&pr, &epi, tiles_m, tiles_n, blockIdx.x, gridDim.x,
                                                                            tiles_m * tiles_n, true, &sk);
}

// NB independent problems of one shape and layout in one launch (the three weight-gradient products
// of the backward): the work items are the tiles of all problems, problem after problem.  Small
// problems fill the chip together where each alone would not, and two launches are saved.
template <class Epi, int NB> struct MfmaBatch {
    MfmaProblem pr[NB];
    Epi epi[NB];
};

template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NB, int NWV = 4, int NSETS = 2>
__global__ __launch_bounds__(NWV * 64) void gemm_bf16_mfma_batch_kernel(MfmaBatch<Epi, NB> b, int tiles_m, int tiles_n) {
    gemm_bf16_mfma_tiles<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS>(b.pr, b.epi, tiles_m, tiles_n, blockIdx.x, gridDim.x,
                                                                      NB * tiles_m * tiles_n, true);
}

template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NB, int NWV = 4, int NSETS = 2>
__global__ __launch_bounds__(NWV * 64) void gemm_bf16_mfma_batch_streamk_kernel(MfmaBatch<Epi, NB> b, int tiles_m, int tiles_n,
                                                                                StreamKArgs sk) {
    gemm_bf16_mfma_tiles<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS, true>(b.pr, b.epi, tiles_m, tiles_n, blockIdx.x, gridDim.x,
                                                                            NB * tiles_m * tiles_n, true, &sk);
}

// Up to NB independent problems that share the output width, the contraction lengths and the layouts
// but not the number of rows (one product per expert of an MoE layer, or the weight-gradient products
// of all experts, whose contraction runs over each expert's own rows) in one launch.  cum[z] is the
// number of tiles before problem z; the work items are the tiles of all problems, problem after
// problem, dealt to the XCDs as contiguous ranges.
template <class Epi, int NB> struct MfmaGroup {
    MfmaProblem pr[NB];
    Epi epi[NB];
    int cum[NB + 1];
};

template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NB, int NWV = 4, int NSETS = 2>
__global__ __launch_bounds__(NWV * 64) void gemm_bf16_mfma_group_kernel(MfmaGroup<Epi, NB> g, int nprob, int tiles_n) {
    const int item = xcd_contiguous_index(blockIdx.x, g.cum[nprob]);
    int z = 0;
    while (z + 1 < nprob && item >= g.cum[z + 1]) ++z;
    const int tiles_m = (g.cum[z + 1] - g.cum[z]) / tiles_n;
    gemm_bf16_mfma_tile<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS>(g.pr[z], tiles_m, tiles_n, g.epi[z], item - g.cum[z]);
}

// Two independent problems of one shape and layout with different epilogues in one launch (gate and
// up projection of the forward): the work items are the tiles of the first problem, then of the second.
template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class EpiA, class EpiB, int NWV = 4, int NSETS = 2>
__global__ __launch_bounds__(NWV * 64) void gemm_bf16_mfma_pair_kernel(MfmaProblem pa, EpiA ea, MfmaProblem pb, EpiB eb,
                                                                        int tiles_m, int tiles_n) {
    const int nblk = tiles_m * tiles_n;
    const int item = xcd_contiguous_index(blockIdx.x, 2 * nblk);
    if (item < nblk)
        gemm_bf16_mfma_tile<BM, BN, AKM, BKM, TAILMODE, EpiA, NWV, NSETS>(pa, tiles_m, tiles_n, ea, item);
    else
        gemm_bf16_mfma_tile<BM, BN, AKM, BKM, TAILMODE, EpiB, NWV, NSETS>(pb, tiles_m, tiles_n, eb, item - nblk);
}

// Host-side check of the kernel's layout assumptions (the caller vouches for the zero padding of
// k-contiguous operands past a contraction length that is not a multiple of 8).
inline bool mfma_problem_ok(const MfmaProblem& p) {
    auto al16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
    auto operand_ok = [&](const GemmOperand<bf16_t>& o, int rows, bool two) {
        bool ok = o.p && al16(o.p) && o.ld % 8 == 0 && (!two || (o.p2 && al16(o.p2)));
        if (o.km) ok = ok && o.ext % 8 == 0 && o.ext >= 8 && o.ext <= o.ld && rows <= o.ext;
        // element offsets inside a tile are kept in 32 bits
        ok = ok && (int64_t)(o.km ? kMfmaBK : rows) * o.ld < (1ll << 31);
        return ok;
    };
    const bool two = p.Kc2 != 0;
    bool ok = p.M >= 1 && p.N >= 1 && p.Kc >= kMfmaBK && (!two || p.Kc2 >= kMfmaBK);
    return ok && operand_ok(p.A, p.M, two) && operand_ok(p.B, p.N, two);
}

// Workgroups to launch for `tiles` tiles: one per tile, or `persistent_wgs` (rounded down to a multiple of
// 8, the number of XCDs) workgroups that walk over the tiles when there are more tiles than that.
inline int mfma_grid(int tiles, int persistent_wgs) {
    const int p = persistent_wgs / 8 * 8;
    return (p >= 8 && tiles > p) ? p : tiles;
}

template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NWV = 4, int NSETS = 2>
inline hipError_t launch_gemm_bf16_mfma(const MfmaProblem& p, const Epi& epi, hipStream_t st, int persistent_wgs = 0) {
    static_assert(NSETS >= 2 && NSETS <= 4, "two to four slices in flight");
    using Cfg = MfmaCfg<BM, BN, AKM, BKM>;
    auto kern = gemm_bf16_mfma_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS>;
    LdsAttr<gemm_bf16_mfma_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS>, Cfg::kLds>::use();      // attribute set at library set-up
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(mfma_grid(tiles_m * tiles_n, persistent_wgs)), dim3(NWV * 64), Cfg::kLds, st, p, tiles_m,
                       tiles_n, epi);
    return hipGetLastError();
}

// Whether splitting along k pays for `tiles` tiles of `nk` slices on `wgs` resident workgroups: there is at
// least one tile per workgroup and the last round of whole tiles would leave more than 7 % of the chip idle.
inline bool streamk_pays(int64_t tiles, int nk, int wgs) {
    if (wgs < 8 || tiles < wgs || nk < 16 || tiles * nk >= (1ll << 30)) return false;
    const int64_t rounds = (tiles + wgs - 1) / wgs;
    return (double)tiles / (double)(rounds * wgs) < 0.93;
}

template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NWV = 4, int NSETS = 2>
inline hipError_t launch_gemm_bf16_mfma_streamk(const MfmaProblem& p, const Epi& epi, const StreamKArgs& sk, int wgs,
                                                hipStream_t st) {
    using Cfg = MfmaCfg<BM, BN, AKM, BKM>;
    auto kern = gemm_bf16_mfma_streamk_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS>;
    LdsAttr<gemm_bf16_mfma_streamk_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NWV, NSETS>, Cfg::kLds>::use();
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(wgs / 8 * 8), dim3(NWV * 64), Cfg::kLds, st, p, tiles_m, tiles_n, epi, sk);
    return hipGetLastError();
}

template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NB, int NWV = 4, int NSETS = 2>
inline hipError_t launch_gemm_bf16_mfma_batch_streamk(const MfmaBatch<Epi, NB>& b, const StreamKArgs& sk, int wgs,
                                                      hipStream_t st) {
    using Cfg = MfmaCfg<BM, BN, AKM, BKM>;
    auto kern = gemm_bf16_mfma_batch_streamk_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NB, NWV, NSETS>;
    LdsAttr<gemm_bf16_mfma_batch_streamk_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NB, NWV, NSETS>, Cfg::kLds>::use();
    const int tiles_m = (b.pr[0].M + BM - 1) / BM, tiles_n = (b.pr[0].N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(wgs / 8 * 8), dim3(NWV * 64), Cfg::kLds, st, b, tiles_m, tiles_n, sk);
    return hipGetLastError();
}

template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NB, int NWV = 4, int NSETS = 2>
inline hipError_t launch_gemm_bf16_mfma_batch(const MfmaBatch<Epi, NB>& b, hipStream_t st, int persistent_wgs = 0) {
    using Cfg = MfmaCfg<BM, BN, AKM, BKM>;
    auto kern = gemm_bf16_mfma_batch_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NB, NWV, NSETS>;
    LdsAttr<gemm_bf16_mfma_batch_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NB, NWV, NSETS>, Cfg::kLds>::use();      // attribute set at library set-up
    const int tiles_m = (b.pr[0].M + BM - 1) / BM, tiles_n = (b.pr[0].N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(mfma_grid(NB * tiles_m * tiles_n, persistent_wgs)), dim3(NWV * 64), Cfg::kLds, st, b, tiles_m,
                       tiles_n);
    return hipGetLastError();
}

// Fills g.cum from the problems' row counts (problems with M = 0 get no tiles) and launches.
template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class Epi, int NB, int NWV = 4, int NSETS = 2>
inline hipError_t launch_gemm_bf16_mfma_group(MfmaGroup<Epi, NB>& g, int nprob, hipStream_t st) {
    using Cfg = MfmaCfg<BM, BN, AKM, BKM>;
    auto kern = gemm_bf16_mfma_group_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NB, NWV, NSETS>;
    LdsAttr<gemm_bf16_mfma_group_kernel<BM, BN, AKM, BKM, TAILMODE, Epi, NB, NWV, NSETS>, Cfg::kLds>::use();      // attribute set at library set-up
    const int tiles_n = (g.pr[0].N + BN - 1) / BN;
    g.cum[0] = 0;
    for (int z = 0; z < nprob; ++z) g.cum[z + 1] = g.cum[z] + (g.pr[z].M + BM - 1) / BM * tiles_n;
    for (int z = nprob; z < NB; ++z) g.cum[z + 1] = g.cum[nprob];
    if (g.cum[nprob] == 0) return hipSuccess;
    hipLaunchKernelGGL(kern, dim3(g.cum[nprob]), dim3(NWV * 64), Cfg::kLds, st, g, nprob, tiles_n);
    return hipGetLastError();
}

template <int BM, int BN, bool AKM, bool BKM, int TAILMODE, class EpiA, class EpiB, int NWV = 4, int NSETS = 2>
inline hipError_t launch_gemm_bf16_mfma_pair(const MfmaProblem& pa, const EpiA& ea, const MfmaProblem& pb, const EpiB& eb,
                                             hipStream_t st) {
    using Cfg = MfmaCfg<BM, BN, AKM, BKM>;
    auto kern = gemm_bf16_mfma_pair_kernel<BM, BN, AKM, BKM, TAILMODE, EpiA, EpiB, NWV, NSETS>;
    LdsAttr<gemm_bf16_mfma_pair_kernel<BM, BN, AKM, BKM, TAILMODE, EpiA, EpiB, NWV, NSETS>, Cfg::kLds>::use();      // attribute set at library set-up
    const int tiles_m = (pa.M + BM - 1) / BM, tiles_n = (pa.N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(2 * tiles_m * tiles_n), dim3(NWV * 64), Cfg::kLds, st, pa, ea, pb, eb, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace moc
