// C ABI of the MoC FFN library (see include/moc.h): the state shared by the entry-point files
// (error text, timing records, options, per-device set-up), argument checks, workspace sizes and
// the small entry points.  The kernel sequences of the forward, backward and decode entry points
// are in moc_fwd.hip, moc_bwd.hip and moc_decode.hip.  No device memory is allocated anywhere.
#include <atomic>
#include <mutex>
#include <random>
#include <string>
#include <vector>

#include "api_common.h"
#include "kernel_attrs.h"
#include "misc_kernels.h"

using namespace moc;

// Scratch of moc_ffn_decode_static, the entry point for callers that cannot hand over a workspace.
// Every GPU the library runs on holds its own copy until the process ends.  In host code the name
// below is only a handle for hipGetSymbolAddress: ensure_init() asks for the device address once
// per device, and everything else (kernel arguments) uses that address.
static __device__ __align__(256) unsigned char scratch[mocapi::kStaticScratchBytes];

namespace mocapi {

thread_local char g_err[512] = "";

// ---------------------------------------------------------------------- per-kernel timing
struct TimingEntry {
    std::string name;
    double ms = 0.0;
    int64_t launches = 0;
};
struct PendingSpan {
    int entry;
    hipEvent_t start, stop;
};
bool g_timing_on = false;
std::vector<TimingEntry> g_entries;
std::vector<PendingSpan> g_pending;
std::vector<hipEvent_t> g_event_pool;

hipEvent_t timing_take_event() {
    if (!g_event_pool.empty()) {
        hipEvent_t e = g_event_pool.back();
        g_event_pool.pop_back();
        return e;
    }
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

int timing_entry_index(const char* name) {
    for (size_t i = 0; i < g_entries.size(); ++i)
        if (g_entries[i].name == name) return (int)i;
    g_entries.push_back(TimingEntry{name, 0.0, 0});
    return (int)g_entries.size() - 1;
}

void timing_push(int entry, hipEvent_t start, hipEvent_t stop) { g_pending.push_back(PendingSpan{entry, start, stop}); }

static int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    return v ? atoi(v) : dflt;
}
Options::Options()
    : force_generic(env_int("MOC_FORCE_GENERIC", 0)), tile(env_int("MOC_GEMM_TILE", 0)),
      decode_fused(env_int("MOC_DECODE_FUSED", 1)), decode_fused_p(env_int("MOC_DECODE_FUSED_P", 0)),
      bwd_epilogue(env_int("MOC_BWD_EPILOGUE", 0)), decode_select_gather(env_int("MOC_DECODE_SELECT_GATHER", 0)), grouped_sparse(env_int("MOC_GROUPED_SPARSE", 0)), gemm_streamk_spin(env_int("MOC_GEMM_STREAMK_SPIN", 1 << 20)), gemm_streamk(env_int("MOC_GEMM_STREAMK", 0)), gemm_persistent(env_int("MOC_GEMM_PERSISTENT", 1)), decode_persistent(env_int("MOC_DECODE_PERSISTENT", 0)) {}
static const Options g_options;
const Options& options() { return g_options; }

// Tags of the split GEMM launches: a counter from a random start, scrambled (splitmix64), never zero.
unsigned long long next_streamk_tag() {
    static std::atomic<unsigned long long> counter{((unsigned long long)std::random_device{}() << 32) ^ std::random_device{}()};
    unsigned long long z = counter.fetch_add(0x9E3779B97F4A7C15ull, std::memory_order_relaxed) + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z | 1ull;
}

// ------------------------------------------------------------------- per-device set-up
// Done once per device, by the first entry point called with that device current (or by moc_init):
// the dynamic-LDS limit of every kernel that registered one, and the address of this device's copy
// of the static scratch array.  Nothing else is kept between calls.
constexpr int kMaxDevices = 64;
struct DeviceState {
    std::atomic<int> ready{0};
    void* scratch_ptr = nullptr;      // device address of this device's copy of `scratch`
    int num_cu = 0;
};
DeviceState g_dev[kMaxDevices];
std::mutex g_init_mu;

moc_status ensure_init(void** scratch_out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(MOC_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    DeviceState& D = g_dev[dev];
    if (!D.ready.load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lk(g_init_mu);
        if (!D.ready.load(std::memory_order_relaxed)) {
            for (const KernelAttr& a : kernel_attr_list())
                HIP_TRY(hipFuncSetAttribute(a.fn, hipFuncAttributeMaxDynamicSharedMemorySize, a.lds_bytes));
            void* p = nullptr;
            HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p) return fail(MOC_ERR_HIP, "hipGetSymbolAddress gave no address for the static scratch");
            D.scratch_ptr = p;
            HIP_TRY(hipDeviceGetAttribute(&D.num_cu, hipDeviceAttributeMultiprocessorCount, dev));
            D.ready.store(1, std::memory_order_release);
        }
    }
    if (scratch_out) *scratch_out = D.scratch_ptr;
    return MOC_OK;
}

int device_cu_count() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    return g_dev[dev].num_cu;
}

moc_status check_shape(const moc_shape* s, bool decode) {
    if (!s) return fail(MOC_ERR_BAD_ARG, "shape is NULL");
    if (s->dtype != MOC_F32 && s->dtype != MOC_BF16) return fail(MOC_ERR_BAD_ARG, "unknown dtype %d", s->dtype);
    if (s->T < 1 || s->d < 1 || s->F < 1) return fail(MOC_ERR_BAD_ARG, "T, d, F must be >= 1 (got %d, %d, %d)", s->T, s->d, s->F);
    if (s->K < 1 || s->K > s->F) return fail(MOC_ERR_BAD_ARG, "K must satisfy 1 <= K <= F (got K=%d, F=%d)", s->K, s->F);
    if (s->F > 32768) return fail(MOC_ERR_UNSUPPORTED, "F = %d exceeds 32768", s->F);
    if (s->dtype == MOC_BF16 && s->d % 8 != 0) return fail(MOC_ERR_BAD_ARG, "bf16 needs d %% 8 == 0 (got %d)", s->d);
    if (s->dtype == MOC_F32 && s->d % 4 != 0 && decode) return fail(MOC_ERR_BAD_ARG, "fp32 decode needs d %% 4 == 0 (got %d)", s->d);
    if ((int64_t)s->T * s->F >= (1ll << 40)) return fail(MOC_ERR_UNSUPPORTED, "T*F too large");
    if (decode && s->T > 16) return fail(MOC_ERR_BAD_ARG, "decode batch must be <= 16 (got %d)", s->T);
    return MOC_OK;
}

moc_status check_group(int F, int K, int ga, int gb) {
    if (gb != 4 && gb != 8 && gb != 16) return fail(MOC_ERR_BAD_ARG, "group size b must be 4, 8 or 16 (got %d)", gb);
    if (ga < 1 || ga > gb) return fail(MOC_ERR_BAD_ARG, "a must satisfy 1 <= a <= b (got a=%d, b=%d)", ga, gb);
    if (F % gb != 0) return fail(MOC_ERR_BAD_ARG, "b = %d must divide F = %d", gb, F);
    if (K != F / gb * ga) return fail(MOC_ERR_BAD_ARG, "K = %d must equal a*F/b = %d", K, F / gb * ga);
    return MOC_OK;
}

moc_status check_key_mode(int32_t key_mode) {
    if (key_mode < MOC_KEY_GATE || key_mode > MOC_KEY_ABS_SILU) return fail(MOC_ERR_BAD_ARG, "unknown selection key %d", key_mode);
    return MOC_OK;
}

moc_status check_offsets(const moc_shape* shape, int32_t n_experts, const int32_t* off) {
    if (n_experts < 1 || n_experts > kMaxExperts) return fail(MOC_ERR_UNSUPPORTED, "n_experts must be 1..%d (got %d)", kMaxExperts, n_experts);
    if (!off) return fail(MOC_ERR_BAD_ARG, "expert_offsets is NULL");
    if (off[0] != 0 || off[n_experts] != shape->T) return fail(MOC_ERR_BAD_ARG, "expert_offsets must run from 0 to T");
    for (int e = 0; e < n_experts; ++e)
        if (off[e + 1] < off[e]) return fail(MOC_ERR_BAD_ARG, "expert_offsets must ascend");
    return MOC_OK;
}

}  // namespace mocapi

using namespace mocapi;

// =============================================================================== C ABI
extern "C" {

size_t moc_workspace_bytes(const moc_shape* shape, int op) {
    if (check_shape(shape, op == MOC_OP_DECODE) != MOC_OK) return 0;
    if (op < MOC_OP_FWD || op > MOC_OP_FWD_KEYED) return 0;
    Dims D(*shape);
    return shape->dtype == MOC_BF16 ? workspace_for<bf16_t>(D, op) : workspace_for<float>(D, op);
}

moc_status moc_init(void) { return ensure_init(); }

size_t moc_static_scratch_bytes(void) { return kStaticScratchBytes; }

moc_status moc_rmsnorm(int32_t T, int32_t d, int32_t dtype, const void* h, const void* gain, float eps, void* out,
                       void* hip_stream) {
    if (T < 1 || d < 1) return fail(MOC_ERR_BAD_ARG, "T and d must be >= 1");
    if (dtype != MOC_F32 && dtype != MOC_BF16) return fail(MOC_ERR_BAD_ARG, "unknown dtype %d", dtype);
    CHECK_PTR(h); CHECK_PTR(gain); CHECK_PTR(out);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Span span("rmsnorm", st);
    if (dtype == MOC_BF16) {
        const bf16_t *hp = (const bf16_t*)h, *gp = (const bf16_t*)gain;
        bf16_t* op = (bf16_t*)out;
        if (d % 8 == 0 && d <= 256 * 8 * 2)
            hipLaunchKernelGGL((rmsnorm_kernel<bf16_t, true, 2>), dim3(T), dim3(256), 0, st, hp, gp, eps, d, op);
        else
            hipLaunchKernelGGL((rmsnorm_kernel<bf16_t, false, 1>), dim3(T), dim3(256), 0, st, hp, gp, eps, d, op);
    } else {
        const float *hp = (const float*)h, *gp = (const float*)gain;
        float* op = (float*)out;
        if (d % 4 == 0 && d <= 256 * 4 * 4)
            hipLaunchKernelGGL((rmsnorm_kernel<float, true, 4>), dim3(T), dim3(256), 0, st, hp, gp, eps, d, op);
        else
            hipLaunchKernelGGL((rmsnorm_kernel<float, false, 1>), dim3(T), dim3(256), 0, st, hp, gp, eps, d, op);
    }
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

moc_status moc_residual_add(int32_t T, int32_t d, int32_t dtype, void* h_inout, const void* y, void* hip_stream) {
    if (T < 1 || d < 1) return fail(MOC_ERR_BAD_ARG, "T and d must be >= 1");
    if (dtype != MOC_F32 && dtype != MOC_BF16) return fail(MOC_ERR_BAD_ARG, "unknown dtype %d", dtype);
    CHECK_PTR(h_inout); CHECK_PTR(y);
    MOC_SETUP();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Span span("residual_add", st);
    const int64_t n = (int64_t)T * d;
    if (dtype == MOC_BF16) {
        const bool vec = n % 8 == 0;
        const int64_t work = vec ? n / 8 : n;
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((work + 255) / 256, 16384));
        if (vec) hipLaunchKernelGGL((residual_add_kernel<bf16_t, true>), dim3(grid), dim3(256), 0, st, (bf16_t*)h_inout, (const bf16_t*)y, n);
        else hipLaunchKernelGGL((residual_add_kernel<bf16_t, false>), dim3(grid), dim3(256), 0, st, (bf16_t*)h_inout, (const bf16_t*)y, n);
    } else {
        const bool vec = n % 4 == 0;
        const int64_t work = vec ? n / 4 : n;
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((work + 255) / 256, 16384));
        if (vec) hipLaunchKernelGGL((residual_add_kernel<float, true>), dim3(grid), dim3(256), 0, st, (float*)h_inout, (const float*)y, n);
        else hipLaunchKernelGGL((residual_add_kernel<float, false>), dim3(grid), dim3(256), 0, st, (float*)h_inout, (const float*)y, n);
    }
    HIP_TRY(hipGetLastError());
    return MOC_OK;
}

void moc_timing_enable(int on) { g_timing_on = on != 0; }

int32_t moc_timing_collect(void) {
    for (const PendingSpan& p : g_pending) {
        float ms = 0.0f;
        if (hipEventSynchronize(p.stop) == hipSuccess && hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
            g_entries[p.entry].ms += ms;
            g_entries[p.entry].launches += 1;
        }
        g_event_pool.push_back(p.start);
        g_event_pool.push_back(p.stop);
    }
    g_pending.clear();
    return (int32_t)g_entries.size();
}

moc_status moc_timing_get(int32_t i, char* name, int32_t name_cap, double* total_ms, int64_t* launches) {
    if (i < 0 || i >= (int32_t)g_entries.size()) return fail(MOC_ERR_BAD_ARG, "timing entry %d out of range", i);
    if (name && name_cap > 0) {
        strncpy(name, g_entries[i].name.c_str(), name_cap - 1);
        name[name_cap - 1] = 0;
    }
    if (total_ms) *total_ms = g_entries[i].ms;
    if (launches) *launches = g_entries[i].launches;
    return MOC_OK;
}

void moc_timing_reset(void) {
    moc_timing_collect();
    g_entries.clear();
}

const char* moc_status_string(int status) {
    switch (status) {
        case MOC_OK: return "MOC_OK";
        case MOC_ERR_BAD_ARG: return "MOC_ERR_BAD_ARG";
        case MOC_ERR_WORKSPACE: return "MOC_ERR_WORKSPACE";
        case MOC_ERR_UNSUPPORTED: return "MOC_ERR_UNSUPPORTED";
        case MOC_ERR_HIP: return "MOC_ERR_HIP";
    }
    return "MOC_ERR_UNKNOWN";
}

const char* moc_last_error(void) { return g_err; }

#ifndef MOC_SOURCE_HASH
#define MOC_SOURCE_HASH "unknown"
#endif
const char* moc_version(void) { return "moc-ffn 0.2 gfx950 src:" MOC_SOURCE_HASH; }

}  // extern "C"
