"""moc_ffn_decode_static (the decode entry point that allocates nothing: its scratch is a static
device array inside the library) against moc_ffn_decode on the same inputs, through the C ABI.
Two calls in a row share the array, the second with a smaller input; a third repeats the first."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2511_09323_amd as moc
from paper_2511_09323_amd import binding as B
from paper_2511_09323_amd import inputs
from tests import parity as P

pytestmark = pytest.mark.gpu


def _case(seed, Bt, d, F, K, dtype):
    L = inputs.make_layer(seed, Bt, d, F, dtype)
    G = {k: P.to_dev(v, dtype) for k, v in L.items()}
    G["host"] = L
    return G


def _decode_static_raw(lib, G, K):
    """Straight through ctypes: nothing but the C entry point runs between the two markers."""
    x = G["x"]
    Bt, d = x.shape
    F = G["wg"].shape[0]
    y = torch.empty((Bt, d), dtype=x.dtype, device=x.device)
    idx = torch.empty((Bt, K), dtype=torch.int32, device=x.device)
    shp = B.MocShape(Bt, d, F, K, B.MOC_BF16 if x.dtype == torch.bfloat16 else B.MOC_F32)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = lib.moc_ffn_decode_static(ctypes.byref(shp), ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(G["wg"].data_ptr()),
                                   ctypes.c_void_p(G["wu"].data_ptr()), ctypes.c_void_p(G["wd"].data_ptr()),
                                   ctypes.c_void_p(y.data_ptr()), ctypes.c_void_p(idx.data_ptr()),
                                   ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, lib.moc_last_error()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return y, idx


def test_static_scratch_decode_matches_the_workspace_entry_point():
    lib = moc.load_library()
    assert moc.static_scratch_bytes() == 16 << 20
    big = _case(97, 16, 1024, 2752, 344, "bf16")
    small = _case(98, 3, 256, 515, 64, "bf16")
    one = _case(99, 1, 512, 1376, 172, "f32")
    for name, G, K in (("big", big, 344), ("small", small, 64), ("big again", big, 344), ("one fp32 token", one, 172)):
        print("[case] static-scratch decode:", name, flush=True)
        y_ref, idx_ref = moc.moc_ffn_decode(G["x"], G["wg"], G["wu"], G["wd"], K)
        y, idx = _decode_static_raw(lib, G, K)
        assert torch.equal(idx, idx_ref), name
        assert torch.equal(y, y_ref), name
        # and the binding's wrapper
        y2, idx2 = moc.moc_ffn_decode_static(G["x"], G["wg"], G["wu"], G["wd"], K)
        torch.cuda.synchronize()
        assert torch.equal(idx2, idx_ref) and torch.equal(y2, y_ref), name
    # oracle check of one of them (the workspace entry point has its own parity tests)
    Ln = small["host"]
    y, idx = _decode_static_raw(lib, small, 64)
    D, _, _, G64 = P.oracle_forward_for(Ln, idx.cpu().numpy())
    P.check_index_sets(idx.cpu().numpy(), G64, 64)
    P.assert_close("static decode y", P.to_np(y), D, P.TOL["bf16"])


def test_static_scratch_decode_refuses_what_does_not_fit():
    lib = moc.load_library()
    fake = ctypes.c_void_p(0x1000)
    # 16 tokens of d = 16384: the partial outputs alone fill 16 MiB
    shp = B.MocShape(16, 16384, 32768, 4096, B.MOC_BF16)
    need = lib.moc_workspace_bytes(ctypes.byref(shp), B.OP_DECODE)
    assert need > moc.static_scratch_bytes()
    rc = lib.moc_ffn_decode_static(ctypes.byref(shp), fake, fake, fake, fake, fake, None, None)
    assert rc == -3 and b"static" in lib.moc_last_error()
    shp = B.MocShape(17, 64, 128, 16, B.MOC_BF16)
    assert lib.moc_ffn_decode_static(ctypes.byref(shp), fake, fake, fake, fake, fake, None, None) == -1
