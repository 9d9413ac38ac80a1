"""MI355X-native Mixture-of-Channels FFN: hand-written HIP kernels behind a C ABI (include/moc.h).

The Python names mirror the C entry points and only marshal arguments; importing this package
does not load the library (binding.load_library() does, and raises if it is not built).
"""
from .binding import (  # noqa: F401
    MocError, init, load_library, moc_ffn_bwd, moc_ffn_decode, moc_ffn_decode_static, static_scratch_bytes,
    moc_ffn_decode_grouped, moc_ffn_fwd, moc_ffn_fwd_grouped,
    moc_ffn_fwd_keyed, moc_ffn_decode_keyed, moc_topk_rows_keyed, moc_ffn_fwd_experts, moc_ffn_bwd_experts,
    moc_residual_add, moc_rmsnorm, moc_topk_grouped_rows,
    moc_swiglu_bwd, moc_swiglu_fwd, moc_topk_rows, timing_enable, timing_read, timing_reset, version,
    workspace_bytes,
)
