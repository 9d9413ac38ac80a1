// Shared by the entry-point files of the library (moc_api.hip, moc_fwd.hip, moc_bwd.hip,
// moc_decode.hip): error reporting, per-kernel timing spans, options from the environment, the
// per-device set-up, argument checks and the workspace layouts.  Host code only.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "../../include/moc.h"
#include "common.h"

namespace mocapi {
using namespace moc;

// ------------------------------------------------------------------------------- errors
extern thread_local char g_err[512];

inline moc_status fail(moc_status s, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return s;
}

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail(MOC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// ---------------------------------------------------------------------- per-kernel timing
// (state and bookkeeping live in moc_api.hip)
extern bool g_timing_on;
hipEvent_t timing_take_event();
int timing_entry_index(const char* name);
void timing_push(int entry, hipEvent_t start, hipEvent_t stop);

// Brackets the launches made during its lifetime with two events on the stream.
struct Span {
    hipStream_t st;
    hipEvent_t start = nullptr, stop = nullptr;
    int entry = -1;
    Span(const char* name, hipStream_t s) : st(s) {
        if (!g_timing_on) return;
        start = timing_take_event();
        stop = timing_take_event();
        if (!start || !stop) return;
        entry = timing_entry_index(name);
        (void)hipEventRecord(start, st);
    }
    ~Span() {
        if (entry < 0) return;
        (void)hipEventRecord(stop, st);
        timing_push(entry, start, stop);
    }
};

// ------------------------------------------------------------------------ small helpers
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

struct Carver {   // hands out 256-byte aligned pieces of the workspace
    unsigned char* base;
    size_t off = 0;
    explicit Carver(void* p) : base(static_cast<unsigned char*>(p)) {}
    template <class T> T* take(size_t count) {
        T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += round_up_sz(count * sizeof(T), 256);
        return r;
    }
};

struct Options {          // environment, read once when the library is loaded
    int force_generic;    // MOC_FORCE_GENERIC=1: never use the MFMA GEMM
    int tile;             // MOC_GEMM_TILE=256|192|128 forces a tile shape, 0 = choose by problem size
    int decode_fused;     // MOC_DECODE_FUSED=0: grouped decode of one token as separate launches
    int decode_fused_p;   // MOC_DECODE_FUSED_P=n: workgroups of the single-launch grouped decode kernel, 0 = choose
    int bwd_epilogue;     // MOC_BWD_EPILOGUE=1: backward pointwise step inside the dZ' GEMM's epilogue (mask + prefix tables) instead of the expansion kernel
    int decode_select_gather;  // MOC_DECODE_SELECT_GATHER=1: row-wide decode with the selection repeated inside every gather workgroup instead of a launch of its own (not faster as measured)
    int grouped_sparse;   // MOC_GROUPED_SPARSE=1: down projection of MoC_{a:b}, a <= 2, on the structured-sparse matrix instruction (not faster as measured)
    int gemm_streamk_spin;  // MOC_GEMM_STREAMK_SPIN=n: polls before a workgroup of a split product stops waiting for its neighbour's share and multiplies it itself (0 in a test of that path)
    int gemm_streamk;     // MOC_GEMM_STREAMK=1: split GEMM work along the contraction where whole tiles leave part of the chip idle (measured slower)
    int gemm_persistent;  // MOC_GEMM_PERSISTENT=0: one workgroup per GEMM tile instead of one per compute unit walking over tiles
    int decode_persistent;  // MOC_DECODE_PERSISTENT=1: row-wide decode as one persistent launch (measured slower than the separate launches)
    Options();
};
const Options& options();

// Per-device set-up (kernel attributes, address of the static scratch); see moc_api.hip.
// scratch_out, if given, receives the current device's address of the static scratch array.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
moc_status ensure_init(void** scratch_out = nullptr);
int device_cu_count();          // compute units of the current device (after ensure_init)

#define MOC_SETUP()                                  \
    do {                                             \
        moc_status si_ = mocapi::ensure_init();      \
        if (si_ != MOC_OK) return si_;               \
    } while (0)

moc_status check_shape(const moc_shape* s, bool decode);
moc_status check_group(int F, int K, int ga, int gb);
moc_status check_key_mode(int32_t key_mode);
moc_status check_offsets(const moc_shape* shape, int32_t n_experts, const int32_t* off);

#define CHECK_PTR(p)                                                                   \
    do {                                                                               \
        if ((p) == nullptr) return fail(MOC_ERR_BAD_ARG, "%s is NULL", #p);            \
        if (!aligned16(p)) return fail(MOC_ERR_BAD_ARG, "%s is not 16-byte aligned", #p); \
    } while (0)

#define CHECK_WS(op)                                                                                  \
    do {                                                                                              \
        CHECK_PTR(ws);                                                                                \
        size_t need_ = moc_workspace_bytes(shape, op);                                                \
        if (ws_bytes < need_) return fail(MOC_ERR_WORKSPACE, "workspace: %zu bytes given, %zu needed", ws_bytes, need_); \
    } while (0)

// ------------------------------------------------------------------- workspace layouts
struct Dims {
    int T, d, F, K;
    int ldF, nw;
    explicit Dims(const moc_shape& s) : T(s.T), d(s.d), F(s.F), K(s.K) {
        ldF = round_up(F, 64);
        nw = ldF / 32;
    }
};

// Memory for GEMMs whose work is split along the contraction: one 256 x 256 fp32 accumulator slot and one
// word per workgroup.  Carved out of the training workspaces when the layer is large enough for such a split
// to be chosen at all (MOC_GEMM_STREAMK=1, bf16, at least one 256 x 256 tile per workgroup in the [T, F] or
// the 3 x [F, d] products).  The words need no initialisation.
constexpr int kStreamKSlots = 256;
struct StreamKArea {
    float* part = nullptr;
    unsigned long long* flag = nullptr;
    template <class E> static bool wanted(const Dims& D) {
        if (!std::is_same<E, uint16_t>::value || !options().gemm_streamk) return false;
        const int64_t tf = (int64_t)((D.T + 255) / 256) * ((D.F + 255) / 256);
        const int64_t fd = 3 * (int64_t)((D.F + 255) / 256) * ((D.d + 255) / 256);
        return tf >= kStreamKSlots || fd >= kStreamKSlots;
    }
    template <class E> void carve(Carver& c, const Dims& D) {
        if (!wanted<E>(D)) return;
        part = c.take<float>((size_t)kStreamKSlots * 256 * 256);
        flag = c.take<unsigned long long>(kStreamKSlots);
    }
};
unsigned long long next_streamk_tag();

template <class E> struct FwdWs {      // dense scratch of the forward: fp32 gate, U, masked Z'
    float *G, *keys;                   // keys: transformed selection keys (Top-K position variants only)
    E *U, *Zd;
    uint16_t* zc;                      // compressed Z' of the structured-sparse down projection (MOC_GROUPED_SPARSE=1, bf16)
    uint32_t* zi;
    StreamKArea sk;
    size_t bytes;
    FwdWs(void* ws, const Dims& D, bool dense, bool keyed = false) {
        Carver c(ws);
        G = dense ? nullptr : c.take<float>((size_t)D.T * D.ldF);
        U = dense ? nullptr : c.take<E>((size_t)D.T * D.ldF);
        Zd = c.take<E>((size_t)D.T * D.ldF);
        keys = keyed ? c.take<float>((size_t)D.T * D.ldF) : nullptr;
        const bool sparse = !dense && std::is_same<E, uint16_t>::value && options().grouped_sparse;
        zc = sparse ? c.take<uint16_t>((size_t)D.T * (D.ldF / 2)) : nullptr;
        zi = sparse ? c.take<uint32_t>((size_t)D.T * (D.ldF / 32)) : nullptr;
        sk.carve<E>(c, D);
        bytes = c.off;
    }
};

template <class E> struct BwdWs {      // dense [T, ldF] operands (+ the bit mask of the fallback path)
    uint32_t* maskw;
    uint16_t* pref;
    E *dZd, *Zd, *dGd, *dUd;
    StreamKArea sk;
    size_t bytes;
    BwdWs(void* ws, const Dims& D, bool dense) {
        Carver c(ws);
        maskw = dense ? nullptr : c.take<uint32_t>((size_t)D.T * D.nw);
        pref = dense ? nullptr : c.take<uint16_t>((size_t)D.T * D.nw);
        dZd = dense ? nullptr : c.take<E>((size_t)D.T * D.ldF);
        Zd = c.take<E>((size_t)D.T * D.ldF);
        dGd = c.take<E>((size_t)D.T * D.ldF);
        dUd = c.take<E>((size_t)D.T * D.ldF);
        sk.carve<E>(c, D);
        bytes = c.off;
    }
};

// Channel shares per token in the gather stage: shares x tokens fills the 256 CUs once (one
// 512-thread workgroup per CU), and a multiple of 8 shares lets the kernel keep each share on one XCD.
inline int decode_splits(int B, int K) {
    const int by_batch = std::max(8, 256 / B / 8 * 8);
    const int by_k = (K + 7) / 8;
    return std::max(1, std::min(by_batch, by_k));
}

constexpr int kDecodeFusedMaxP = 512;

constexpr size_t kDecodeSyncBytes = 32 * 1024;          // >= sizeof(moc::DecodeSync), checked where that type is known
constexpr size_t kDecodePartBudget = (size_t)4 << 20;   // partial outputs of the persistent kernel's down projection

struct DecodeWs {
    float *g, *gkeys, *gsel, *z, *part;
    int32_t* idx;
    // persistent single-launch kernel: tagged gate values [T, ldF], tagged token mask and z' of every
    // channel [F, 1 + token slots], partial outputs of its down projection, its flag words
    uint64_t *g2, *zt;
    float* part2;
    void* sync;
    size_t bytes;
    DecodeWs(void* ws, const Dims& D) {
        Carver c(ws);
        g = c.take<float>((size_t)D.T * D.ldF);
        gkeys = c.take<float>((size_t)D.T * D.ldF);
        gsel = c.take<float>((size_t)D.T * D.K);
        z = c.take<float>((size_t)D.T * D.K);
        idx = c.take<int32_t>((size_t)D.T * D.K);
        // partial outputs: one per channel share, or one per workgroup of the single-launch grouped kernel
        const int shares = std::max(decode_splits(D.T, D.K), D.T == 1 ? kDecodeFusedMaxP : 0);
        part = c.take<float>((size_t)shares * D.T * D.d);
        const int slots = D.T == 1 ? 1 : (D.T <= 4 ? 4 : 16);
        g2 = c.take<uint64_t>((size_t)D.T * D.ldF);
        zt = c.take<uint64_t>((size_t)D.F * (1 + slots));
        part2 = c.take<float>(kDecodePartBudget / sizeof(float));
        sync = c.take<unsigned char>(kDecodeSyncBytes);
        bytes = c.off;
    }
};

template <class E> size_t workspace_for(const Dims& D, int op) {
    switch (op) {
        case MOC_OP_FWD: return FwdWs<E>(nullptr, D, false).bytes;
        case MOC_OP_BWD: return BwdWs<E>(nullptr, D, false).bytes;
        case MOC_OP_DECODE: return DecodeWs(nullptr, D).bytes;
        case MOC_OP_SWIGLU_FWD: return FwdWs<E>(nullptr, D, true).bytes;
        case MOC_OP_SWIGLU_BWD: return BwdWs<E>(nullptr, D, true).bytes;
        case MOC_OP_FWD_KEYED: return FwdWs<E>(nullptr, D, false, true).bytes;
    }
    return 0;
}


constexpr int kMaxExperts = 8;

}  // namespace mocapi
