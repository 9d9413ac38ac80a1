"""ctypes binding of libmoc_ffn.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their data pointers and
the current torch stream through the C ABI declared in include/moc.h, and raises MocError when the
library returns a negative status.  There is no fallback: without the built library (or without a
GPU tensor) the call fails.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoc_ffn.so")

MOC_F32, MOC_BF16 = 0, 1
OP_FWD, OP_BWD, OP_DECODE, OP_SWIGLU_FWD, OP_SWIGLU_BWD = range(5)

EXPORTS = (
    "moc_workspace_bytes", "moc_init", "moc_ffn_fwd", "moc_ffn_bwd", "moc_ffn_decode", "moc_ffn_decode_static", "moc_static_scratch_bytes", "moc_swiglu_fwd",
    "moc_swiglu_bwd", "moc_topk_rows", "moc_ffn_fwd_experts", "moc_ffn_bwd_experts", "moc_ffn_fwd_keyed", "moc_ffn_decode_keyed", "moc_topk_rows_keyed", "moc_ffn_fwd_grouped", "moc_ffn_decode_grouped", "moc_topk_grouped_rows", "moc_rmsnorm", "moc_residual_add", "moc_timing_enable",
    "moc_timing_collect", "moc_timing_get", "moc_timing_reset", "moc_status_string",
    "moc_last_error", "moc_version",
)


class MocError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("%s: %s" % (status, text))
        self.status = status


class MocShape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("F", ctypes.c_int32),
                ("K", ctypes.c_int32), ("dtype", ctypes.c_int32)]


_lib = None


def load_library():
    """Loads the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MocError("MOC_ERR_NOT_BUILT", "%s is missing: run `python -m paper_2511_09323_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    shp = ctypes.POINTER(MocShape)
    lib.moc_workspace_bytes.restype = sz
    lib.moc_workspace_bytes.argtypes = [shp, ctypes.c_int]
    lib.moc_init.restype = ctypes.c_int
    lib.moc_init.argtypes = []
    lib.moc_ffn_fwd.restype = ctypes.c_int
    lib.moc_ffn_fwd.argtypes = [shp] + [vp] * 9 + [sz, vp]
    lib.moc_ffn_bwd.restype = ctypes.c_int
    lib.moc_ffn_bwd.argtypes = [shp] + [vp] * 13 + [sz, vp]
    lib.moc_ffn_decode.restype = ctypes.c_int
    lib.moc_ffn_decode.argtypes = [shp] + [vp] * 7 + [sz, vp]
    lib.moc_ffn_decode_static.restype = ctypes.c_int
    lib.moc_ffn_decode_static.argtypes = [shp] + [vp] * 6 + [vp]
    lib.moc_static_scratch_bytes.restype = sz
    lib.moc_static_scratch_bytes.argtypes = []
    lib.moc_swiglu_fwd.restype = ctypes.c_int
    lib.moc_swiglu_fwd.argtypes = [shp] + [vp] * 8 + [sz, vp]
    lib.moc_swiglu_bwd.restype = ctypes.c_int
    lib.moc_swiglu_bwd.argtypes = [shp] + [vp] * 12 + [sz, vp]
    lib.moc_topk_rows.restype = ctypes.c_int
    lib.moc_topk_rows.argtypes = [i32, i32, i32, vp, i64, vp, vp, vp]
    lib.moc_ffn_fwd_experts.restype = ctypes.c_int
    lib.moc_ffn_fwd_experts.argtypes = [shp, i32, ctypes.POINTER(i32)] + [vp] * 9 + [sz, vp]
    lib.moc_ffn_bwd_experts.restype = ctypes.c_int
    lib.moc_ffn_bwd_experts.argtypes = [shp, i32, ctypes.POINTER(i32)] + [vp] * 13 + [sz, vp]
    lib.moc_ffn_fwd_keyed.restype = ctypes.c_int
    lib.moc_ffn_fwd_keyed.argtypes = [shp, i32] + [vp] * 9 + [sz, vp]
    lib.moc_ffn_decode_keyed.restype = ctypes.c_int
    lib.moc_ffn_decode_keyed.argtypes = [shp, i32] + [vp] * 7 + [sz, vp]
    lib.moc_topk_rows_keyed.restype = ctypes.c_int
    lib.moc_topk_rows_keyed.argtypes = [i32, i32, i32, i32, vp, i64, vp, vp, vp, vp]
    lib.moc_ffn_fwd_grouped.restype = ctypes.c_int
    lib.moc_ffn_fwd_grouped.argtypes = [shp, i32, i32] + [vp] * 9 + [sz, vp]
    lib.moc_ffn_decode_grouped.restype = ctypes.c_int
    lib.moc_ffn_decode_grouped.argtypes = [shp, i32, i32] + [vp] * 7 + [sz, vp]
    lib.moc_topk_grouped_rows.restype = ctypes.c_int
    lib.moc_topk_grouped_rows.argtypes = [i32, i32, i32, i32, vp, i64, vp, vp, vp]
    lib.moc_rmsnorm.restype = ctypes.c_int
    lib.moc_rmsnorm.argtypes = [i32, i32, i32, vp, vp, ctypes.c_float, vp, vp]
    lib.moc_residual_add.restype = ctypes.c_int
    lib.moc_residual_add.argtypes = [i32, i32, i32, vp, vp, vp]
    lib.moc_timing_enable.restype = None
    lib.moc_timing_enable.argtypes = [ctypes.c_int]
    lib.moc_timing_collect.restype = i32
    lib.moc_timing_collect.argtypes = []
    lib.moc_timing_get.restype = ctypes.c_int
    lib.moc_timing_get.argtypes = [i32, ctypes.c_char_p, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    lib.moc_timing_reset.restype = None
    lib.moc_timing_reset.argtypes = []
    lib.moc_status_string.restype = ctypes.c_char_p
    lib.moc_status_string.argtypes = [ctypes.c_int]
    lib.moc_last_error.restype = ctypes.c_char_p
    lib.moc_last_error.argtypes = []
    lib.moc_version.restype = ctypes.c_char_p
    lib.moc_version.argtypes = []
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        lib = load_library()
        raise MocError(lib.moc_status_string(status).decode(), lib.moc_last_error().decode())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return MOC_F32
    if t.dtype == torch.bfloat16:
        return MOC_BF16
    raise MocError("MOC_ERR_BAD_ARG", "unsupported torch dtype %s" % t.dtype)


def _ptr(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise MocError("MOC_ERR_BAD_ARG", "%s must be a GPU tensor" % name)
    if not t.is_contiguous():
        raise MocError("MOC_ERR_BAD_ARG", "%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise MocError("MOC_ERR_BAD_ARG", "%s has dtype %s, expected %s" % (name, t.dtype, dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise MocError("MOC_ERR_BAD_ARG", "%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _shape(T, d, F, K, code):
    return MocShape(int(T), int(d), int(F), int(K), int(code))


def init():
    """Per-device set-up for the current device (optional; every call does it on first use)."""
    _check(load_library().moc_init())


def workspace_bytes(T, d, F, K, dtype, op):
    code = {torch.float32: MOC_F32, torch.bfloat16: MOC_BF16}[dtype]
    shp = _shape(T, d, F, K, code)
    return int(load_library().moc_workspace_bytes(ctypes.byref(shp), op))


def _workspace(ws, T, d, F, K, dtype, op, device):
    need = workspace_bytes(T, d, F, K, dtype, op)
    if need == 0:
        # let the entry point produce the precise error text
        return torch.empty(256, dtype=torch.uint8, device=device), 256
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws, ws.numel() * ws.element_size()


def moc_ffn_fwd(x, wg, wu, wd, K, ws=None, out=None):
    """Returns (y, idx, gvals, uvals).  x [T,d]; wg, wu, wd channel-major [F,d]."""
    lib = load_library()
    T, d = x.shape
    F = wg.shape[0]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((T, d), dtype=dt, device=x.device)
        idx = torch.empty((T, K), dtype=torch.int32, device=x.device)
        gvals = torch.empty((T, K), dtype=dt, device=x.device)
        uvals = torch.empty((T, K), dtype=dt, device=x.device)
    else:
        y, idx, gvals, uvals = out
    ws, ws_bytes = _workspace(ws, T, d, F, K, dt, OP_FWD, x.device)
    shp = _shape(T, d, F, K, code)
    _check(lib.moc_ffn_fwd(ctypes.byref(shp), _ptr(x, dt, (T, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                           _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"), _ptr(y, dt, (T, d), "y"),
                           _ptr(idx, torch.int32, (T, K), "idx"), _ptr(gvals, dt, (T, K), "gvals"),
                           _ptr(uvals, dt, (T, K), "uvals"), _ptr(ws, name="ws"), ws_bytes, _stream()))
    return y, idx, gvals, uvals


def moc_ffn_bwd(x, wg, wu, wd, idx, gvals, uvals, dy, ws=None, out=None):
    """Returns (dx, dwg, dwu, dwd) from the stored set and the upstream gradient."""
    lib = load_library()
    T, d = x.shape
    F = wg.shape[0]
    K = idx.shape[1]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        dx = torch.empty((T, d), dtype=dt, device=x.device)
        dwg = torch.empty((F, d), dtype=dt, device=x.device)
        dwu = torch.empty((F, d), dtype=dt, device=x.device)
        dwd = torch.empty((F, d), dtype=dt, device=x.device)
    else:
        dx, dwg, dwu, dwd = out
    ws, ws_bytes = _workspace(ws, T, d, F, K, dt, OP_BWD, x.device)
    shp = _shape(T, d, F, K, code)
    _check(lib.moc_ffn_bwd(ctypes.byref(shp), _ptr(x, dt, (T, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                           _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"),
                           _ptr(idx, torch.int32, (T, K), "idx"), _ptr(gvals, dt, (T, K), "gvals"),
                           _ptr(uvals, dt, (T, K), "uvals"), _ptr(dy, dt, (T, d), "dy"),
                           _ptr(dx, dt, (T, d), "dx"), _ptr(dwg, dt, (F, d), "dwg"), _ptr(dwu, dt, (F, d), "dwu"),
                           _ptr(dwd, dt, (F, d), "dwd"), _ptr(ws, name="ws"), ws_bytes, _stream()))
    return dx, dwg, dwu, dwd


def moc_ffn_decode(x, wg, wu, wd, K, ws=None, want_idx=True, out=None):
    """Returns (y, idx or None) for a decode batch x [B,d], B <= 16."""
    lib = load_library()
    B, d = x.shape
    F = wg.shape[0]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((B, d), dtype=dt, device=x.device)
        idx = torch.empty((B, K), dtype=torch.int32, device=x.device) if want_idx else None
    else:
        y, idx = out
    ws, ws_bytes = _workspace(ws, B, d, F, K, dt, OP_DECODE, x.device)
    shp = _shape(B, d, F, K, code)
    _check(lib.moc_ffn_decode(ctypes.byref(shp), _ptr(x, dt, (B, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                              _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"), _ptr(y, dt, (B, d), "y"),
                              _ptr(idx, torch.int32, (B, K), "idx") if idx is not None else None,
                              _ptr(ws, name="ws"), ws_bytes, _stream()))
    return y, idx


def moc_ffn_decode_static(x, wg, wu, wd, K, want_idx=True, out=None):
    """moc_ffn_decode on the library's static scratch array: no workspace argument, no allocation
    inside the call when `out` is given.  Returns (y, idx or None)."""
    lib = load_library()
    B, d = x.shape
    F = wg.shape[0]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((B, d), dtype=dt, device=x.device)
        idx = torch.empty((B, K), dtype=torch.int32, device=x.device) if want_idx else None
    else:
        y, idx = out
    shp = _shape(B, d, F, K, code)
    _check(lib.moc_ffn_decode_static(ctypes.byref(shp), _ptr(x, dt, (B, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                                     _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"), _ptr(y, dt, (B, d), "y"),
                                     _ptr(idx, torch.int32, (B, K), "idx") if idx is not None else None, _stream()))
    return y, idx


def static_scratch_bytes():
    return int(load_library().moc_static_scratch_bytes())


def moc_swiglu_fwd(x, wg, wu, wd, ws=None, out=None):
    """Dense SwiGLU forward.  Returns (y, g_save, u_save)."""
    lib = load_library()
    T, d = x.shape
    F = wg.shape[0]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((T, d), dtype=dt, device=x.device)
        g_save = torch.empty((T, F), dtype=dt, device=x.device)
        u_save = torch.empty((T, F), dtype=dt, device=x.device)
    else:
        y, g_save, u_save = out
    ws, ws_bytes = _workspace(ws, T, d, F, F, dt, OP_SWIGLU_FWD, x.device)
    shp = _shape(T, d, F, F, code)
    _check(lib.moc_swiglu_fwd(ctypes.byref(shp), _ptr(x, dt, (T, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                              _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"), _ptr(y, dt, (T, d), "y"),
                              _ptr(g_save, dt, (T, F), "g_save"), _ptr(u_save, dt, (T, F), "u_save"),
                              _ptr(ws, name="ws"), ws_bytes, _stream()))
    return y, g_save, u_save


def moc_swiglu_bwd(x, wg, wu, wd, g_save, u_save, dy, ws=None, out=None):
    """Dense SwiGLU backward.  Returns (dx, dwg, dwu, dwd)."""
    lib = load_library()
    T, d = x.shape
    F = wg.shape[0]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        dx = torch.empty((T, d), dtype=dt, device=x.device)
        dwg = torch.empty((F, d), dtype=dt, device=x.device)
        dwu = torch.empty((F, d), dtype=dt, device=x.device)
        dwd = torch.empty((F, d), dtype=dt, device=x.device)
    else:
        dx, dwg, dwu, dwd = out
    ws, ws_bytes = _workspace(ws, T, d, F, F, dt, OP_SWIGLU_BWD, x.device)
    shp = _shape(T, d, F, F, code)
    _check(lib.moc_swiglu_bwd(ctypes.byref(shp), _ptr(x, dt, (T, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                              _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"),
                              _ptr(g_save, dt, (T, F), "g_save"), _ptr(u_save, dt, (T, F), "u_save"),
                              _ptr(dy, dt, (T, d), "dy"), _ptr(dx, dt, (T, d), "dx"), _ptr(dwg, dt, (F, d), "dwg"),
                              _ptr(dwu, dt, (F, d), "dwu"), _ptr(dwd, dt, (F, d), "dwd"),
                              _ptr(ws, name="ws"), ws_bytes, _stream()))
    return dx, dwg, dwu, dwd


def moc_topk_rows(g, K):
    """Row-wise Top-K of an fp32 matrix g [T,F] (rows may be strided).  Returns (idx [T,K]
    ascending, gsel [T,K])."""
    lib = load_library()
    T, F = g.shape
    if not g.is_cuda or g.dtype != torch.float32 or g.stride(1) != 1:
        raise MocError("MOC_ERR_BAD_ARG", "g must be a GPU fp32 matrix with unit column stride")
    ldg = g.stride(0) if T > 1 else F
    idx = torch.empty((T, K), dtype=torch.int32, device=g.device)
    gsel = torch.empty((T, K), dtype=torch.float32, device=g.device)
    _check(lib.moc_topk_rows(T, F, K, ctypes.c_void_p(g.data_ptr()), ldg, _ptr(idx), _ptr(gsel), _stream()))
    return idx, gsel


def _offsets(offsets):
    arr = (ctypes.c_int32 * len(offsets))(*[int(o) for o in offsets])
    return arr, len(offsets) - 1


def moc_ffn_fwd_experts(x, offsets, wg, wu, wd, K, ws=None, out=None):
    """MoC as the MLP of MoE experts.  x [A,d]: routed rows sorted by expert; offsets: n_experts + 1 host
    integers; wg, wu, wd [n_experts, F, d].  Returns (y, idx, gvals, uvals) for all rows."""
    lib = load_library()
    T, d = x.shape
    E, F = wg.shape[0], wg.shape[1]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((T, d), dtype=dt, device=x.device)
        idx = torch.empty((T, K), dtype=torch.int32, device=x.device)
        gvals = torch.empty((T, K), dtype=dt, device=x.device)
        uvals = torch.empty((T, K), dtype=dt, device=x.device)
    else:
        y, idx, gvals, uvals = out
    ws, ws_bytes = _workspace(ws, T, d, F, K, dt, OP_FWD, x.device)
    shp = _shape(T, d, F, K, code)
    off, n = _offsets(offsets)
    if n != E:
        raise MocError("MOC_ERR_BAD_ARG", "offsets must have n_experts + 1 entries")
    _check(lib.moc_ffn_fwd_experts(ctypes.byref(shp), n, off, _ptr(x, dt, (T, d), "x"), _ptr(wg, dt, (E, F, d), "wg"),
                                   _ptr(wu, dt, (E, F, d), "wu"), _ptr(wd, dt, (E, F, d), "wd"), _ptr(y, dt, (T, d), "y"),
                                   _ptr(idx, torch.int32, (T, K), "idx"), _ptr(gvals, dt, (T, K), "gvals"),
                                   _ptr(uvals, dt, (T, K), "uvals"), _ptr(ws, name="ws"), ws_bytes, _stream()))
    return y, idx, gvals, uvals


def moc_ffn_bwd_experts(x, offsets, wg, wu, wd, idx, gvals, uvals, dy, ws=None, out=None):
    """Backward of moc_ffn_fwd_experts.  Returns (dx [A,d], dwg, dwu, dwd [n_experts, F, d])."""
    lib = load_library()
    T, d = x.shape
    E, F = wg.shape[0], wg.shape[1]
    K = idx.shape[1]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        dx = torch.empty((T, d), dtype=dt, device=x.device)
        dwg = torch.empty((E, F, d), dtype=dt, device=x.device)
        dwu = torch.empty((E, F, d), dtype=dt, device=x.device)
        dwd = torch.empty((E, F, d), dtype=dt, device=x.device)
    else:
        dx, dwg, dwu, dwd = out
    ws, ws_bytes = _workspace(ws, T, d, F, K, dt, OP_BWD, x.device)
    shp = _shape(T, d, F, K, code)
    off, n = _offsets(offsets)
    if n != E:
        raise MocError("MOC_ERR_BAD_ARG", "offsets must have n_experts + 1 entries")
    _check(lib.moc_ffn_bwd_experts(ctypes.byref(shp), n, off, _ptr(x, dt, (T, d), "x"), _ptr(wg, dt, (E, F, d), "wg"),
                                   _ptr(wu, dt, (E, F, d), "wu"), _ptr(wd, dt, (E, F, d), "wd"),
                                   _ptr(idx, torch.int32, (T, K), "idx"), _ptr(gvals, dt, (T, K), "gvals"),
                                   _ptr(uvals, dt, (T, K), "uvals"), _ptr(dy, dt, (T, d), "dy"),
                                   _ptr(dx, dt, (T, d), "dx"), _ptr(dwg, dt, (E, F, d), "dwg"),
                                   _ptr(dwu, dt, (E, F, d), "dwu"), _ptr(dwd, dt, (E, F, d), "dwd"),
                                   _ptr(ws, name="ws"), ws_bytes, _stream()))
    return dx, dwg, dwu, dwd


KEY_MODES = {"gate": 0, "silu": 1, "abs_silu": 2}
OP_FWD_KEYED = 5


def _key_code(key):
    if key not in KEY_MODES:
        raise MocError("MOC_ERR_BAD_ARG", "selection key must be one of %s" % sorted(KEY_MODES))
    return KEY_MODES[key]


def moc_ffn_fwd_keyed(x, wg, wu, wd, K, key, ws=None, out=None):
    """moc_ffn_fwd with the Top-K taken on key(g): "gate" (plain), "silu" or "abs_silu".
    Returns (y, idx, gvals, uvals); gvals are the gate values themselves."""
    lib = load_library()
    T, d = x.shape
    F = wg.shape[0]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((T, d), dtype=dt, device=x.device)
        idx = torch.empty((T, K), dtype=torch.int32, device=x.device)
        gvals = torch.empty((T, K), dtype=dt, device=x.device)
        uvals = torch.empty((T, K), dtype=dt, device=x.device)
    else:
        y, idx, gvals, uvals = out
    ws, ws_bytes = _workspace(ws, T, d, F, K, dt, OP_FWD_KEYED, x.device)
    shp = _shape(T, d, F, K, code)
    _check(lib.moc_ffn_fwd_keyed(ctypes.byref(shp), _key_code(key), _ptr(x, dt, (T, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                                 _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"), _ptr(y, dt, (T, d), "y"),
                                 _ptr(idx, torch.int32, (T, K), "idx"), _ptr(gvals, dt, (T, K), "gvals"),
                                 _ptr(uvals, dt, (T, K), "uvals"), _ptr(ws, name="ws"), ws_bytes, _stream()))
    return y, idx, gvals, uvals


def moc_ffn_decode_keyed(x, wg, wu, wd, K, key, ws=None, want_idx=True, out=None):
    """moc_ffn_decode with the Top-K taken on key(g).  Returns (y, idx or None)."""
    lib = load_library()
    B, d = x.shape
    F = wg.shape[0]
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((B, d), dtype=dt, device=x.device)
        idx = torch.empty((B, K), dtype=torch.int32, device=x.device) if want_idx else None
    else:
        y, idx = out
    ws, ws_bytes = _workspace(ws, B, d, F, K, dt, OP_DECODE, x.device)
    shp = _shape(B, d, F, K, code)
    _check(lib.moc_ffn_decode_keyed(ctypes.byref(shp), _key_code(key), _ptr(x, dt, (B, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                                    _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"), _ptr(y, dt, (B, d), "y"),
                                    _ptr(idx, torch.int32, (B, K), "idx") if idx is not None else None,
                                    _ptr(ws, name="ws"), ws_bytes, _stream()))
    return y, idx


def moc_topk_rows_keyed(g, K, key):
    """Row-wise Top-K of key(g) for an fp32 matrix g [T,F].  Returns (idx ascending, gsel = g there)."""
    lib = load_library()
    T, F = g.shape
    if not g.is_cuda or g.dtype != torch.float32 or g.stride(1) != 1:
        raise MocError("MOC_ERR_BAD_ARG", "g must be a GPU fp32 matrix with unit column stride")
    ldg = g.stride(0) if T > 1 else F
    idx = torch.empty((T, K), dtype=torch.int32, device=g.device)
    gsel = torch.empty((T, K), dtype=torch.float32, device=g.device)
    scratch = torch.empty((T, ldg), dtype=torch.float32, device=g.device)
    _check(lib.moc_topk_rows_keyed(T, F, K, _key_code(key), ctypes.c_void_p(g.data_ptr()), ldg, _ptr(scratch), _ptr(idx),
                                   _ptr(gsel), _stream()))
    return idx, gsel


def _grouped_K(F, a, b):
    return F // b * a if b > 0 and F % b == 0 else max(1, min(F, a))   # the library reports bad a:b itself


def moc_ffn_fwd_grouped(x, wg, wu, wd, a, b, ws=None, out=None):
    """MoC_{a:b} forward (a kept of every b consecutive channels).  Returns (y, idx, gvals, uvals)
    with K = a*F/b columns, usable by moc_ffn_bwd as they are."""
    lib = load_library()
    T, d = x.shape
    F = wg.shape[0]
    K = _grouped_K(F, a, b)
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((T, d), dtype=dt, device=x.device)
        idx = torch.empty((T, K), dtype=torch.int32, device=x.device)
        gvals = torch.empty((T, K), dtype=dt, device=x.device)
        uvals = torch.empty((T, K), dtype=dt, device=x.device)
    else:
        y, idx, gvals, uvals = out
    ws, ws_bytes = _workspace(ws, T, d, F, K, dt, OP_FWD, x.device)
    shp = _shape(T, d, F, K, code)
    _check(lib.moc_ffn_fwd_grouped(ctypes.byref(shp), a, b, _ptr(x, dt, (T, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                                   _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"), _ptr(y, dt, (T, d), "y"),
                                   _ptr(idx, torch.int32, (T, K), "idx"), _ptr(gvals, dt, (T, K), "gvals"),
                                   _ptr(uvals, dt, (T, K), "uvals"), _ptr(ws, name="ws"), ws_bytes, _stream()))
    return y, idx, gvals, uvals


def moc_ffn_decode_grouped(x, wg, wu, wd, a, b, ws=None, want_idx=True, out=None):
    """MoC_{a:b} decode for a batch x [B,d], B <= 16.  Returns (y, idx or None)."""
    lib = load_library()
    B, d = x.shape
    F = wg.shape[0]
    K = _grouped_K(F, a, b)
    dt = x.dtype
    code = _dtype_code(x)
    if out is None:
        y = torch.empty((B, d), dtype=dt, device=x.device)
        idx = torch.empty((B, K), dtype=torch.int32, device=x.device) if want_idx else None
    else:
        y, idx = out
    ws, ws_bytes = _workspace(ws, B, d, F, K, dt, OP_DECODE, x.device)
    shp = _shape(B, d, F, K, code)
    _check(lib.moc_ffn_decode_grouped(ctypes.byref(shp), a, b, _ptr(x, dt, (B, d), "x"), _ptr(wg, dt, (F, d), "wg"),
                                      _ptr(wu, dt, (F, d), "wu"), _ptr(wd, dt, (F, d), "wd"),
                                      _ptr(y, dt, (B, d), "y"),
                                      _ptr(idx, torch.int32, (B, K), "idx") if idx is not None else None,
                                      _ptr(ws, name="ws"), ws_bytes, _stream()))
    return y, idx


def moc_topk_grouped_rows(g, a, b):
    """Grouped Top-K (a of every b consecutive columns) of an fp32 matrix g [T,F] (rows may be
    strided).  Returns (idx [T, a*F/b] ascending, gsel)."""
    lib = load_library()
    T, F = g.shape
    if not g.is_cuda or g.dtype != torch.float32 or g.stride(1) != 1:
        raise MocError("MOC_ERR_BAD_ARG", "g must be a GPU fp32 matrix with unit column stride")
    ldg = g.stride(0) if T > 1 else F
    K = _grouped_K(F, a, b)
    idx = torch.empty((T, K), dtype=torch.int32, device=g.device)
    gsel = torch.empty((T, K), dtype=torch.float32, device=g.device)
    _check(lib.moc_topk_grouped_rows(T, F, a, b, ctypes.c_void_p(g.data_ptr()), ldg, _ptr(idx), _ptr(gsel), _stream()))
    return idx, gsel


def moc_rmsnorm(h, gain, eps, out=None):
    lib = load_library()
    T, d = h.shape
    if out is None:
        out = torch.empty_like(h)
    _check(lib.moc_rmsnorm(T, d, _dtype_code(h), _ptr(h, None, None, "h"), _ptr(gain, h.dtype, (d,), "gain"),
                           float(eps), _ptr(out, h.dtype, (T, d), "out"), _stream()))
    return out


def moc_residual_add(h, y):
    lib = load_library()
    T, d = h.shape
    _check(lib.moc_residual_add(T, d, _dtype_code(h), _ptr(h, None, None, "h"), _ptr(y, h.dtype, (T, d), "y"),
                                _stream()))
    return h


def timing_enable(on):
    load_library().moc_timing_enable(1 if on else 0)


def timing_reset():
    load_library().moc_timing_reset()


def timing_read():
    """{kernel name: (total_ms, launches)} accumulated since the last reset (synchronises)."""
    lib = load_library()
    n = lib.moc_timing_collect()
    out = {}
    buf = ctypes.create_string_buffer(128)
    ms = ctypes.c_double()
    cnt = ctypes.c_int64()
    for i in range(n):
        _check(lib.moc_timing_get(i, buf, 128, ctypes.byref(ms), ctypes.byref(cnt)))
        out[buf.value.decode()] = (ms.value, cnt.value)
    return out


def version():
    return load_library().moc_version().decode()
