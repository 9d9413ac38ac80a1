/*
 * moc.h -- C ABI of the Mixture-of-Channels (MoC) feed-forward layer for AMD MI355X (gfx950).
 *
 * The layer (paper section "Mixture-of-Channels architecture", Eqs. (MoC-1), (MoC-2)):
 *     G = X W_gate,  U = X W_up,  M = TopK(G) row-wise on the signed, pre-SiLU gate,
 *     S' = SiLU(G) . M,  Z' = S' . U,  D = Z' W_down.
 * Backward: section "Activation-efficient pre-training", Eqs. (bp-1)...(bp-5), with the
 * MoC+GCP stored set of Table 1 (G.M, U.M and M; S' and Z' are recomputed).
 * Decode: section "Accelerated inference", the per-token recipe that touches only K columns of
 * W_up and K rows of W_down.
 *
 * Conventions shared by every entry point
 *  - Every data pointer is DEVICE memory owned by the caller, 16-byte aligned, valid on the
 *    device that is current when the call is made.  The shape struct is HOST memory.
 *  - Layouts (row-major, tight): x, y, dy, dx are [T, d].  The three weights and their gradients
 *    are channel-major [F, d]: row j of wg / wu is column j of the paper's W_gate / W_up, row j of
 *    wd is row j of W_down.  idx, gvals, uvals are [T, K]; within a row idx ascends by channel and
 *    gvals / uvals hold G and U at those channels (the paper's G.M, U.M and M in compact form).
 *  - dtype is the element type of x, the weights, y, the saved values and all gradients
 *    (MOC_F32 or MOC_BF16).  All accumulation is fp32.  The Top-K decision is taken on the fp32
 *    gate accumulator before any rounding; equal values are ordered by channel, lower first,
 *    and -0.0 equals +0.0.  Non-finite inputs are not detected.
 *  - The library allocates no device memory; scratch lives in the caller's workspace `ws` of at
 *    least moc_workspace_bytes(shape, op) bytes (256-byte aligned).  Two calls that overlap in
 *    time must not share a workspace.  The only state kept between calls is a per-device set-up
 *    done once, by moc_init() or by the first entry point called with that device current: the
 *    dynamic-LDS limit of every kernel (hipFuncSetAttribute) and the device address of the static
 *    scratch array of moc_ffn_decode_static.  It is guarded by a mutex and makes no stream operation, so a first call may be
 *    made from any thread and under stream capture; a caller that wants the set-up outside its
 *    capture or timing calls moc_init() beforehand.
 *  - Calls validate their arguments on the host, enqueue kernels on `hip_stream` (a hipStream_t,
 *    NULL = the default stream) and return without synchronising; outputs are valid in stream
 *    order.  Gradients are overwritten, not accumulated.
 *  - Errors: a negative moc_status is returned and moc_last_error() describes it (thread-local
 *    text).  Argument errors are found before anything is launched and leave outputs untouched.
 *  - Limits: 1 <= K <= F <= 32768, T >= 1 (T <= 16 for decode), d >= 1; MOC_BF16 needs d % 8 == 0.
 *    Tighter limits, all refused with MOC_ERR_UNSUPPORTED before anything is launched:
 *    moc_ffn_bwd_experts stages three rows of F_pad elements in LDS, so it needs
 *    3 * F_pad * sizeof(element) <= 160 KiB - 64 (F <= ~27k for bf16, ~13.6k for fp32; plain
 *    moc_ffn_bwd has no such limit).  The decode entry points stage the tokens' inputs in LDS:
 *    Bt * d * sizeof(element) <= 160 KiB - 64 with Bt = 1, 4 or 16 for T = 1, 2..4, 5..16
 *    (fp32 with T > 4: d <= 2559; bf16 with T > 4 and d not a multiple of 1024: d <= 5119), and
 *    d * sizeof(element) <= 64 KiB for the gather stage.
 *  - Environment variables for testing and tuning (none is needed in normal use):
 *    MOC_FORCE_GENERIC=1 sends every GEMM to the generic fp32-FMA kernel and decode to
 *    its non-MFMA kernels; MOC_GEMM_TILE=256|192|128 forces an MFMA tile shape;
 *    MOC_DECODE_FUSED=0 and MOC_DECODE_FUSED_P=n switch off, or set the workgroup count of, the
 *    single-launch grouped decode kernel; MOC_DECODE_SELECT_GATHER=1 repeats the selection of row-wide
 *    decode inside every gather workgroup instead of giving it a launch of its own (not faster as
 *    measured); MOC_DECODE_PERSISTENT=1 runs row-wide decode (moc_ffn_decode,
 *    moc_ffn_decode_static) as one persistent launch instead of four launches (slower on the
 *    measured shapes, kept for study); MOC_GEMM_PERSISTENT=0 launches one workgroup per GEMM tile
 *    instead of one per compute unit looping over tiles; MOC_GEMM_STREAMK=1 lets the training products
 *    whose whole tiles leave part of the chip idle split their work along the contraction (needs a
 *    larger workspace; slower as measured; MOC_GEMM_STREAMK_SPIN=n bounds the polls a workgroup spends
 *    waiting for a neighbour's share before it multiplies that share itself); MOC_BWD_EPILOGUE=1 applies the backward's
 *    pointwise step in the dZ' product's epilogue instead of a kernel of its own (slower as measured);
 *    MOC_GROUPED_SPARSE=1 runs the down projection of moc_ffn_fwd_grouped with a <= 2 on the
 *    structured-sparse matrix instruction (bf16; needs a larger workspace; not faster as measured).
 *    All are read once, when the library is loaded.
 */
#ifndef MOC_H
#define MOC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOC_OK = 0,
    MOC_ERR_BAD_ARG = -1,      /* null / misaligned pointer, K or shape out of range, unknown dtype */
    MOC_ERR_WORKSPACE = -2,    /* ws_bytes smaller than moc_workspace_bytes() */
    MOC_ERR_UNSUPPORTED = -3,  /* valid request this build cannot run (e.g. F too large for LDS) */
    MOC_ERR_HIP = -4           /* a HIP runtime call failed; text holds hipGetErrorString */
} moc_status;

typedef enum { MOC_F32 = 0, MOC_BF16 = 1 } moc_dtype;

typedef enum {
    MOC_OP_FWD = 0,
    MOC_OP_BWD = 1,
    MOC_OP_DECODE = 2,
    MOC_OP_SWIGLU_FWD = 3,
    MOC_OP_SWIGLU_BWD = 4,
    MOC_OP_FWD_KEYED = 5       /* moc_ffn_fwd_keyed: the forward workspace plus one fp32 [T, F] key array */
} moc_op;

/* What the row Top-K ranks (ablation "Effect of top-K's position" and the remark after the proof
 * of Theorem 1): the raw gate (the paper's choice and the default everywhere else), the SiLU
 * output, or its absolute value. */
typedef enum { MOC_KEY_GATE = 0, MOC_KEY_SILU = 1, MOC_KEY_ABS_SILU = 2 } moc_key;

/* T tokens (batch for decode), d = d_model, F = d_ffn, K selected channels per token. */
typedef struct {
    int32_t T, d, F, K;
    int32_t dtype; /* moc_dtype */
} moc_shape;

/* Bytes of workspace `op` needs for `shape`; 0 if the shape is invalid. */
size_t moc_workspace_bytes(const moc_shape* shape, int op);

/* Per-device set-up for the device that is current (see the conventions above).  Optional: every
 * entry point does the same on its first call on a device.  Returns MOC_ERR_HIP without a GPU. */
moc_status moc_init(void);

/* Training forward, Eqs. (MoC-1), (MoC-2).  Writes y[T,d] and the stored set idx[T,K] (int32),
 * gvals[T,K], uvals[T,K] (dtype).  Steps: gate projection (fp32), row Top-K, up projection,
 * SiLU(g).u on the selected channels, down projection. */
moc_status moc_ffn_fwd(const moc_shape* shape, const void* x, const void* wg, const void* wu,
                       const void* wd, void* y, int32_t* idx, void* gvals, void* uvals,
                       void* ws, size_t ws_bytes, void* hip_stream);

/* Training backward, Eqs. (bp-1)...(bp-5), from the stored set and dy[T,d].  Writes dx[T,d] and
 * dwg, dwu, dwd [F,d].  idx rows must ascend strictly and lie in [0, F). */
moc_status moc_ffn_bwd(const moc_shape* shape, const void* x, const void* wg, const void* wu,
                       const void* wd, const int32_t* idx, const void* gvals, const void* uvals,
                       const void* dy, void* dx, void* dwg, void* dwu, void* dwd,
                       void* ws, size_t ws_bytes, void* hip_stream);

/* Decode, section "Accelerated inference": shape->T is the batch B (1..16).  Reads all of wg and
 * only the rows of wu and wd that some token selected.  Writes y[B,d]; if idx_or_null is not
 * NULL also the selected channels idx[B,K] (ascending). */
moc_status moc_ffn_decode(const moc_shape* shape, const void* x, const void* wg, const void* wu,
                          const void* wd, void* y, int32_t* idx_or_null,
                          void* ws, size_t ws_bytes, void* hip_stream);

/* moc_ffn_decode for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and
 * kernels as moc_ffn_decode, but the scratch is a static device array inside the library
 * (moc_static_scratch_bytes() = 16 MiB per GPU, held until the process ends); the call allocates
 * nothing.  Shapes whose moc_workspace_bytes(shape, MOC_OP_DECODE) exceeds that size are refused
 * with MOC_ERR_UNSUPPORTED before anything is launched (the 7B shape with 16 tokens needs about
 * 6 MiB).  All calls on one GPU share the array: the kernels overwrite what they read, nothing has
 * to be cleared between calls, but two calls that overlap in time on one GPU (different streams)
 * race; order them on one stream or with events. */
moc_status moc_ffn_decode_static(const moc_shape* shape, const void* x, const void* wg, const void* wu,
                                 const void* wd, void* y, int32_t* idx_or_null, void* hip_stream);
size_t moc_static_scratch_bytes(void);

/* Dense SwiGLU FFN, Eqs. (FFN-1), (FFN-2): the K = F reference.  shape->K is ignored.
 * g_save, u_save are [T,F] in dtype (the dense stored set G and U). */
moc_status moc_swiglu_fwd(const moc_shape* shape, const void* x, const void* wg, const void* wu,
                          const void* wd, void* y, void* g_save, void* u_save,
                          void* ws, size_t ws_bytes, void* hip_stream);

moc_status moc_swiglu_bwd(const moc_shape* shape, const void* x, const void* wg, const void* wu,
                          const void* wd, const void* g_save, const void* u_save, const void* dy,
                          void* dx, void* dwg, void* dwu, void* dwd,
                          void* ws, size_t ws_bytes, void* hip_stream);

/* Row-wise Top-K alone (the mask definition of section "Mixture-of-Channels architecture"):
 * g[T, ldg] fp32 (ldg >= F elements) -> idx[T,K] ascending by channel and gsel[T,K] fp32, the gate
 * values there.  Needs no workspace.  When ldg is a multiple of 4 and g is 16-byte aligned, the
 * aligned 16-byte block that holds the last element of a row is read whole. */
moc_status moc_topk_rows(int32_t T, int32_t F, int32_t K, const float* g, int64_t ldg,
                         int32_t* idx, float* gsel, void* hip_stream);

/* Top-K position variants: as moc_ffn_fwd / moc_ffn_decode / moc_topk_rows, but the K channels of
 * a row are those with the largest key_mode(g) (moc_key); gvals / gsel still hold the gate values
 * themselves, so moc_ffn_bwd takes the stored set unchanged.  key_mode = MOC_KEY_GATE is the plain
 * call.  moc_ffn_fwd_keyed needs moc_workspace_bytes(shape, MOC_OP_FWD_KEYED); moc_topk_rows_keyed
 * needs key_scratch, caller-owned fp32 [T, ldg] (unused, may be NULL, for MOC_KEY_GATE).  The
 * keys are computed in fp32 from the fp32 gate; ties and signed zeros as everywhere else. */
moc_status moc_ffn_fwd_keyed(const moc_shape* shape, int32_t key_mode, const void* x, const void* wg,
                             const void* wu, const void* wd, void* y, int32_t* idx, void* gvals,
                             void* uvals, void* ws, size_t ws_bytes, void* hip_stream);

moc_status moc_ffn_decode_keyed(const moc_shape* shape, int32_t key_mode, const void* x,
                                const void* wg, const void* wu, const void* wd, void* y,
                                int32_t* idx_or_null, void* ws, size_t ws_bytes, void* hip_stream);

moc_status moc_topk_rows_keyed(int32_t T, int32_t F, int32_t K, int32_t key_mode, const float* g,
                               int64_t ldg, float* key_scratch, int32_t* idx, float* gsel,
                               void* hip_stream);

/* MoC as the MLP of every expert of an MoE layer (section "Compatibility with MoE architectures").
 * The rows of x are the routed token copies, sorted by expert: rows expert_offsets[e] ..
 * expert_offsets[e+1]-1 belong to expert e (HOST array of n_experts + 1 ascending int32, first 0,
 * last shape->T; an expert may have no rows).  wg, wu, wd and their gradients hold the experts'
 * channel-major matrices one after the other, [n_experts, F, d].  Routing and the weighted
 * combination of the experts' outputs belong to the surrounding MoE layer and are the caller's.
 * Everything else -- outputs, stored set, workspace (MOC_OP_FWD / MOC_OP_BWD for shape) -- as
 * moc_ffn_fwd / moc_ffn_bwd; each projection runs as one launch over all experts.  Weight
 * gradients of an expert without rows are set to zero.  n_experts <= 8. */
moc_status moc_ffn_fwd_experts(const moc_shape* shape, int32_t n_experts, const int32_t* expert_offsets,
                               const void* x, const void* wg, const void* wu, const void* wd, void* y,
                               int32_t* idx, void* gvals, void* uvals,
                               void* ws, size_t ws_bytes, void* hip_stream);

moc_status moc_ffn_bwd_experts(const moc_shape* shape, int32_t n_experts, const int32_t* expert_offsets,
                               const void* x, const void* wg, const void* wu, const void* wd,
                               const int32_t* idx, const void* gvals, const void* uvals, const void* dy,
                               void* dx, void* dwg, void* dwu, void* dwd,
                               void* ws, size_t ws_bytes, void* hip_stream);

/* MoC_{a:b}, the grouped Top-K variant (item "MoC with structured 2:8 sparsity" of section
 * "Mixture-of-Channels architecture"; a:b defined before Theorem 1): the mask keeps the a largest
 * signed gate values of every contiguous group of b channels (channels q*b .. q*b+b-1), ties to
 * the lower channel.  b must be 4, 8 or 16 and divide F, 1 <= a <= b, and shape->K must equal
 * a*F/b; otherwise MOC_ERR_BAD_ARG.  Arguments, layouts, workspace (moc_workspace_bytes with
 * MOC_OP_FWD / MOC_OP_DECODE and the same shape) and ownership are those of moc_ffn_fwd /
 * moc_ffn_decode / moc_topk_rows; idx rows ascend, slot q*a + r holds the r-th kept channel of
 * group q.  The stored set feeds moc_ffn_bwd unchanged. */
moc_status moc_ffn_fwd_grouped(const moc_shape* shape, int32_t a, int32_t b, const void* x,
                               const void* wg, const void* wu, const void* wd, void* y,
                               int32_t* idx, void* gvals, void* uvals,
                               void* ws, size_t ws_bytes, void* hip_stream);

moc_status moc_ffn_decode_grouped(const moc_shape* shape, int32_t a, int32_t b, const void* x,
                                  const void* wg, const void* wu, const void* wd, void* y,
                                  int32_t* idx_or_null, void* ws, size_t ws_bytes, void* hip_stream);

moc_status moc_topk_grouped_rows(int32_t T, int32_t F, int32_t a, int32_t b, const float* g,
                                 int64_t ldg, int32_t* idx, float* gsel, void* hip_stream);

/* RMSNorm of each row, y = x / sqrt(mean(x^2) + eps) . gain (section "Activation memory
 * profiling", RMSNorm item); h, out are [T,d] in dtype, gain is [d] in dtype. */
moc_status moc_rmsnorm(int32_t T, int32_t d, int32_t dtype, const void* h, const void* gain,
                       float eps, void* out, void* hip_stream);

/* Residual connection h <- h + y on [T,d] (same section, residual item). */
moc_status moc_residual_add(int32_t T, int32_t d, int32_t dtype, void* h_inout, const void* y,
                            void* hip_stream);

/* Per-kernel timing for benchmarks.  moc_timing_enable(1) makes every later call bracket each
 * kernel launch with HIP events on the call's stream; moc_timing_collect synchronises those
 * events, adds their durations to the per-kernel totals and returns the number of distinct
 * kernel names seen so far.  moc_timing_get copies entry i (name up to name_cap-1 chars, total
 * milliseconds, launch count).  moc_timing_enable(0) stops recording; moc_timing_reset clears
 * the totals.  HOST pointers.  Not thread-safe. */
void moc_timing_enable(int on);
int32_t moc_timing_collect(void);
moc_status moc_timing_get(int32_t i, char* name, int32_t name_cap, double* total_ms, int64_t* launches);
void moc_timing_reset(void);

const char* moc_status_string(int status);
const char* moc_last_error(void);
/* Library version string, e.g. "moc-ffn 0.2 gfx950 src:0123456789abcdef": the last field is a hash of
 * the sources the library was built from. */
const char* moc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOC_H */
