"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
include/moc.h declares, sizes workspaces consistently and rejects bad arguments before touching
the device."""
import ctypes
import os
import re

import pytest

from paper_2511_09323_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2511_09323_amd import build
        build.build(verbose=False)
    return B.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "moc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert "moc_ffn_fwd" in names and "moc_ffn_bwd" in names and "moc_ffn_decode" in names
    assert "moc_swiglu_fwd" in names and "moc_swiglu_bwd" in names
    for n in names:
        assert hasattr(lib, n), n
    assert set(B.EXPORTS) == set(names)


def test_version_and_status_strings(lib):
    assert b"gfx950" in lib.moc_version()
    assert lib.moc_status_string(0) == b"MOC_OK"
    assert lib.moc_status_string(-1) == b"MOC_ERR_BAD_ARG"
    assert lib.moc_status_string(-2) == b"MOC_ERR_WORKSPACE"
    assert lib.moc_status_string(-3) == b"MOC_ERR_UNSUPPORTED"
    assert lib.moc_status_string(-4) == b"MOC_ERR_HIP"


def _ws(lib, T, d, F, K, dt, op):
    s = B.MocShape(T, d, F, K, dt)
    return lib.moc_workspace_bytes(ctypes.byref(s), op)


def test_workspace_sizes(lib):
    # forward, bf16, cfg2: fp32 gate [T, ldF] + two bf16 [T, ldF] arrays, ldF = 5504
    T, d, F, K = 8192, 2048, 5461, 683
    ldF = 5504
    want = T * ldF * 4 + 2 * T * ldF * 2
    got = _ws(lib, T, d, F, K, B.MOC_BF16, B.OP_FWD)
    assert want <= got <= want + 4 * 256
    # fp32 needs more than bf16; invalid shapes give 0
    assert _ws(lib, T, d, F, K, B.MOC_F32, B.OP_FWD) > got
    assert _ws(lib, T, d, F, F + 1, B.MOC_BF16, B.OP_FWD) == 0
    assert _ws(lib, T, d, F, 0, B.MOC_BF16, B.OP_FWD) == 0
    assert _ws(lib, 17, 4096, 11008, 1376, B.MOC_BF16, B.OP_DECODE) == 0      # decode batch > 16
    assert _ws(lib, 16, 4096, 11008, 1376, B.MOC_BF16, B.OP_DECODE) > 0
    assert _ws(lib, T, d, F, K, B.MOC_BF16, 99) == 0
    assert _ws(lib, T, d, F, K, 7, B.OP_FWD) == 0
    for op in (B.OP_BWD, B.OP_SWIGLU_FWD, B.OP_SWIGLU_BWD):
        assert _ws(lib, T, d, F, K, B.MOC_BF16, op) > 0


def test_bad_arguments_are_rejected_before_any_launch(lib):
    fake = ctypes.c_void_p(0x1000)      # aligned, never dereferenced: validation fails first
    s = B.MocShape(4, 64, 128, 200, B.MOC_BF16)          # K > F
    rc = lib.moc_ffn_fwd(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, None)
    assert rc == -1 and b"K" in lib.moc_last_error()
    s = B.MocShape(4, 64, 128, 16, B.MOC_BF16)
    rc = lib.moc_ffn_fwd(ctypes.byref(s), None, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, None)
    assert rc == -1 and b"NULL" in lib.moc_last_error()
    rc = lib.moc_ffn_fwd(ctypes.byref(s), ctypes.c_void_p(0x1004), fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, None)
    assert rc == -1 and b"aligned" in lib.moc_last_error()
    rc = lib.moc_ffn_fwd(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, fake, fake, 16, None)
    assert rc == -2 and b"workspace" in lib.moc_last_error()
    rc = lib.moc_ffn_fwd(None, fake, fake, fake, fake, fake, fake, fake, fake, fake, 16, None)
    assert rc == -1
    s = B.MocShape(4, 60, 128, 16, B.MOC_BF16)           # bf16 needs d % 8 == 0
    rc = lib.moc_ffn_bwd(ctypes.byref(s), *([fake] * 13), 1 << 30, None)
    assert rc == -1
    s = B.MocShape(4, 64, 40000, 16, B.MOC_BF16)         # F too large
    rc = lib.moc_ffn_decode(ctypes.byref(s), *([fake] * 7), 1 << 30, None)
    assert rc == -3
    assert lib.moc_topk_rows(4, 16, 17, fake, 16, fake, fake, None) == -1
    assert lib.moc_topk_rows(4, 16, 4, fake, 8, fake, fake, None) == -1     # ldg < F
    s = B.MocShape(4, 64, 128, 16, B.MOC_BF16)
    assert lib.moc_ffn_fwd_keyed(ctypes.byref(s), 3, *([fake] * 9), 1 << 30, None) == -1          # unknown key
    assert lib.moc_ffn_fwd_keyed(ctypes.byref(s), 1, *([fake] * 9), 16, None) == -2               # short workspace
    assert lib.moc_ffn_decode_keyed(ctypes.byref(s), -1, *([fake] * 7), 1 << 30, None) == -1
    assert lib.moc_topk_rows_keyed(4, 16, 4, 1, fake, 16, None, fake, fake, None) == -1            # keyed needs key_scratch
    assert _ws(lib, 4, 64, 128, 16, B.MOC_BF16, 5) > _ws(lib, 4, 64, 128, 16, B.MOC_BF16, B.OP_FWD)
    # MoE experts: offsets are validated on the host
    s = B.MocShape(50, 64, 128, 16, B.MOC_BF16)
    off_ok = (ctypes.c_int32 * 3)(0, 20, 50)
    off_bad = (ctypes.c_int32 * 3)(0, 60, 50)
    assert lib.moc_ffn_fwd_experts(ctypes.byref(s), 2, off_bad, *([fake] * 9), 1 << 30, None) == -1
    assert lib.moc_ffn_fwd_experts(ctypes.byref(s), 2, off_ok, *([fake] * 9), 16, None) == -2
    assert lib.moc_ffn_fwd_experts(ctypes.byref(s), 9, off_ok, *([fake] * 9), 1 << 30, None) == -3
    assert lib.moc_ffn_bwd_experts(ctypes.byref(s), 2, None, *([fake] * 13), 1 << 30, None) == -1
    # grouped Top-K (MoC_{a:b}): b in {4, 8, 16} dividing F, 1 <= a <= b, K = a F / b
    s = B.MocShape(4, 64, 128, 32, B.MOC_BF16)
    for a, b in ((2, 8), ):
        assert lib.moc_ffn_fwd_grouped(ctypes.byref(s), a, b, *([fake] * 9), 16, None) == -2     # valid a:b, short workspace
    for a, b in ((2, 4), (0, 8), (9, 8), (2, 5), (2, 2)):
        rc = lib.moc_ffn_fwd_grouped(ctypes.byref(s), a, b, *([fake] * 9), 1 << 30, None)
        assert rc == -1, (a, b)
        rc = lib.moc_ffn_decode_grouped(ctypes.byref(s), a, b, *([fake] * 7), 1 << 30, None)
        assert rc == -1, (a, b)
    s = B.MocShape(4, 64, 100, 50, B.MOC_BF16)           # 8 does not divide F
    assert lib.moc_ffn_fwd_grouped(ctypes.byref(s), 4, 8, *([fake] * 9), 1 << 30, None) == -1
    assert lib.moc_topk_grouped_rows(4, 20, 2, 8, fake, 20, fake, fake, None) == -1
    assert lib.moc_topk_grouped_rows(4, 16, 2, 8, fake, 8, fake, fake, None) == -1      # ldg < F
    assert lib.moc_rmsnorm(0, 16, 0, fake, fake, 1e-5, fake, None) == -1
    assert lib.moc_residual_add(4, 16, 5, fake, fake, None) == -1


def test_python_binding_refuses_cpu_tensors(lib):
    import torch
    x = torch.zeros(4, 64)
    w = torch.zeros(128, 64)
    with pytest.raises(B.MocError):
        B.moc_ffn_fwd(x, w, w, w, 16, ws=torch.zeros(1 << 20, dtype=torch.uint8))


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_committed_traffic_summary_has_the_roofline_kernel():
    # bench.py takes roofline.traffic from this file; a renamed kernel must not silently drop it
    import json
    tj = json.load(open(os.path.join(ROOT, "profiles", "cfg2_traffic.json")))
    ent = tj["gemm_bf16_mfma<256,256,KC,KC,tail0,EpiStore<float>>"]
    assert ent["hbm_read_bytes"] > 0 and ent["hbm_written_bytes"] > 0
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert "gemm_bf16_mfma<256,256,KC,KC,tail0,EpiStore<float>>" in src


def test_bench_reports_committed_traffic_only_for_the_sources_it_was_measured_on(tmp_path, monkeypatch):
    """bench.py's roofline `traffic` comes from the committed rocprofv3 counter summary.  It must be null unless
    that summary names the hash of the kernel sources in this tree AND the loaded library was built from them."""
    import json
    import bench
    from paper_2511_09323_amd.build import source_hash
    here = source_hash()
    assert len(here) == 16 and here == source_hash()          # a pure function of the source files
    prof = tmp_path / "profiles"
    prof.mkdir()
    key = "gemm_bf16_mfma<256,256,KC,KC,tail0,EpiStore<float>>"
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))

    def write(h):
        (prof / "cfg2_traffic.json").write_text(json.dumps({key: {"hbm_read_bytes": 100, "hbm_written_bytes": 23}, "_source_hash": h}))

    write(here)
    val, why = bench.committed_traffic(key, "moc-ffn 0.2 gfx950 src:" + here)
    assert val == 123 and here in why
    val, why = bench.committed_traffic(key, "moc-ffn 0.2 gfx950 src:0000000000000000")
    assert val is None and "not built from these sources" in why
    val, why = bench.committed_traffic("some_other_kernel", "moc-ffn 0.2 gfx950 src:" + here)
    assert val is None
    write("feedfeedfeedfeed")
    val, why = bench.committed_traffic(key, "moc-ffn 0.2 gfx950 src:" + here)
    assert val is None and "other sources" in why
    (prof / "cfg2_traffic.json").unlink()
    val, why = bench.committed_traffic(key, "moc-ffn 0.2 gfx950 src:" + here)
    assert val is None


def test_library_version_names_the_sources_it_was_built_from(lib):
    import re
    v = lib.moc_version().decode()
    assert re.search(r"src:[0-9a-f]{16}$", v), v
