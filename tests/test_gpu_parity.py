"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Index sets are bit-exact outside the 1e-6 near-tie window of the fp32 gate; outputs and
gradients are within 1e-4 (fp32) or 2e-2 (bf16) max-norm relative error."""
import sys

import numpy as np
import pytest
import torch

import paper_2511_09323_amd as moc
from oracle import moc_oracle as O
from paper_2511_09323_amd import inputs
from paper_2511_09323_amd.configs import CONFIGS, RMSNORM_EPS
from tests import parity as P

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def gpu_layer(L, dtype):
    return {k: P.to_dev(v, dtype) for k, v in L.items()}


def run_fwd_bwd_case(tag, cfg_index, T, d, F, K, dtype, bwd=True, expect_window_rows=None):
    say("[case] %s T=%d d=%d F=%d K=%d dtype=%s" % (tag, T, d, F, K, dtype))
    tol = P.TOL[dtype]
    L = inputs.make_layer(cfg_index, T, d, F, dtype, with_dy=True)
    Gd = gpu_layer(L, dtype)
    y, idx, gvals, uvals = moc.moc_ffn_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K)
    torch.cuda.synchronize()
    idx_np = idx.cpu().numpy()
    D, gv_ref, uv_ref, G64 = P.oracle_forward_for(L, idx_np)
    window = P.check_index_sets(idx_np, G64, K)
    say("  idx sets: %d of %d rows inside the near-tie window" % (len(window), T))
    if expect_window_rows is not None:
        assert len(window) <= expect_window_rows
    e = [P.assert_close("y", P.to_np(y), D, tol), P.assert_close("gvals", P.to_np(gvals), gv_ref, tol),
         P.assert_close("uvals", P.to_np(uvals), uv_ref, tol)]
    say("  fwd errors y/gvals/uvals: %.2e %.2e %.2e" % tuple(e))
    if not bwd:
        return
    dx, dwg, dwu, dwd = moc.moc_ffn_bwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], idx, gvals, uvals, Gd["dy"])
    torch.cuda.synchronize()
    ref = P.oracle_backward_for(L, idx_np, P.to_np(gvals), P.to_np(uvals))
    errs = [P.assert_close(n, P.to_np(g), r, tol) for n, g, r in zip(("dx", "dwg", "dwu", "dwd"), (dx, dwg, dwu, dwd), ref)]
    say("  bwd errors dx/dwg/dwu/dwd: %.2e %.2e %.2e %.2e" % tuple(errs))
    # channels selected by no token get exactly zero weight gradients
    unused = np.setdiff1d(np.arange(F), np.unique(idx_np))
    if unused.size:
        for g in (dwg, dwu, dwd):
            assert float(g[torch.from_numpy(unused).cuda()].abs().max()) == 0.0


# ------------------------------------------------------------------------- Top-K alone
def _topk_case(g_np, K):
    g = torch.from_numpy(g_np).cuda()
    idx, gsel = moc.moc_topk_rows(g, K)
    torch.cuda.synchronize()
    ref = np.stack([np.flatnonzero(r) for r in O.topk_mask(g_np, K)])
    np.testing.assert_array_equal(idx.cpu().numpy(), ref)
    want = np.take_along_axis(g_np, ref, axis=1)
    got = gsel.cpu().numpy()
    assert np.array_equal(got == 0, want == 0)
    np.testing.assert_array_equal(np.where(want == 0, 0.0, got), np.where(want == 0, 0.0, want))


def test_topk_bit_exact_random_and_adversarial():
    rng = np.random.default_rng(7)
    for T, F, K in [(5, 1, 1), (3, 7, 7), (4, 64, 1), (9, 333, 41), (16, 1376, 172), (8, 5461, 683),
                    (4, 11008, 1376), (2, 32768, 4096), (3, 1023, 1000), (2, 2050, 3), (2, 8000, 5000), (3, 11264, 4096),
                    (2, 11008, 9000), (3, 6144, 6143), (2, 4100, 4100)]:
        say("[topk] random T=%d F=%d K=%d" % (T, F, K))
        _topk_case(rng.standard_normal((T, F)).astype(np.float32), K)
    say("[topk] ties, signed zeros, constant rows, negative rows")
    g = np.zeros((6, 300), dtype=np.float32)
    g[0] = 1.0                                              # all equal
    g[1] = np.tile(np.array([1, 2, 3], dtype=np.float32), 100)
    g[2] = -np.abs(rng.standard_normal(300)).astype(np.float32)   # all negative
    g[3, ::2] = -0.0                                        # -0.0 and +0.0 mixed
    g[4] = np.round(rng.standard_normal(300) * 2).astype(np.float32)   # many duplicates
    g[5] = np.linspace(-1, 1, 300, dtype=np.float32)[::-1]
    for K in (1, 2, 37, 150, 299, 300):
        _topk_case(g, K)
    say("[topk] tiny and huge magnitudes, denormals")
    h = rng.standard_normal((4, 515)).astype(np.float32)
    h[0] *= 1e-40
    h[1] *= 1e30
    h[2, :100] = np.float32(1.0) + np.arange(100, dtype=np.float32) * np.float32(2 ** -23)
    _topk_case(h, 64)
    say("[topk] strided input (ldg not a multiple of 4)")
    base_np = rng.standard_normal((6, 1001)).astype(np.float32)
    view = torch.from_numpy(base_np).cuda()[:, :997]
    idx, _ = moc.moc_topk_rows(view, 100)
    torch.cuda.synchronize()
    ref = np.stack([np.flatnonzero(r) for r in O.topk_mask(base_np[:, :997], 100)])
    np.testing.assert_array_equal(idx.cpu().numpy(), ref)


def test_topk_full_size_rows_match_oracle():
    # the shapes of the 1B and 7B configurations, gate-like values (sigma = 0.02 sqrt(d))
    rng = np.random.default_rng(8)
    for T, F, K, sigma in [(64, 5461, 683, 0.905), (32, 11008, 1376, 1.28)]:
        say("[topk] full rows T=%d F=%d K=%d" % (T, F, K))
        _topk_case((rng.standard_normal((T, F)) * sigma).astype(np.float32), K)


# ---------------------------------------------------------------- forward and backward
def test_cfg0_fp32_forward_backward():
    c = CONFIGS["cfg0"]
    run_fwd_bwd_case("cfg0", 0, c.T, c.d, c.F, c.K, "f32", bwd=True, expect_window_rows=2)


@pytest.mark.parametrize("T,d,F,K,dtype", [
    (200, 128, 333, 41, "bf16"),      # ragged everywhere, MFMA path (d % 64 == 0)
    (77, 72, 100, 100, "bf16"),       # d % 64 != 0 -> generic GEMM; K = F
    (1, 64, 64, 1, "bf16"),           # degenerate: one token, one channel kept
    (130, 36, 50, 7, "f32"),          # fp32, nothing aligned
    (513, 256, 1030, 129, "bf16"),    # several tiles with ragged tails in every dimension
])
def test_small_ragged_shapes(T, d, F, K, dtype):
    run_fwd_bwd_case("ragged", 90, T, d, F, K, dtype)


@pytest.mark.parametrize("T,d,F,K,dtype", [
    (24, 64, 12000, 1500, "bf16"),    # row too long for registers: LDS-resident fused Top-K
    (16, 64, 14000, 200, "f32"),      # dense rows too large for the LDS expansion: mask + GEMM-epilogue backward
    (8, 128, 32768, 4096, "bf16"),    # largest supported d_ff
    (40, 96, 200, 25, "bf16"),        # contraction tails everywhere (d % 32 != 0, T % 32 != 0, F % 32 != 0)
])
def test_fallback_paths_and_limits(T, d, F, K, dtype):
    run_fwd_bwd_case("limits", 95, T, d, F, K, dtype)


def test_cfg1_bf16_forward_backward():
    c = CONFIGS["cfg1"]
    run_fwd_bwd_case("cfg1", 1, c.T, c.d, c.F, c.K, "bf16", expect_window_rows=12)


def test_cfg2_bf16_forward_backward_full_size():
    c = CONFIGS["cfg2"]
    run_fwd_bwd_case("cfg2", 2, c.T, c.d, c.F, c.K, "bf16", expect_window_rows=40)


def test_forward_is_deterministic_and_workspace_is_reusable():
    L = inputs.make_layer(91, 300, 128, 400, "bf16")
    Gd = gpu_layer(L, "bf16")
    nbytes = moc.workspace_bytes(300, 128, 400, 50, torch.bfloat16, 0)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    a = moc.moc_ffn_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], 50, ws=ws)
    ws.fill_(0xFF)      # NaN patterns everywhere: no result may depend on stale workspace
    b = moc.moc_ffn_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], 50, ws=ws)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    with pytest.raises(moc.MocError):
        moc.moc_ffn_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], 50, ws=ws[:1024])


def test_backward_ignores_stale_workspace():
    T, d, F, K = 100, 64, 200, 30        # T not a multiple of 64: padded token columns must be cleared
    L = inputs.make_layer(92, T, d, F, "bf16", with_dy=True)
    Gd = gpu_layer(L, "bf16")
    y, idx, gv, uv = moc.moc_ffn_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K)
    ws = torch.empty(moc.workspace_bytes(T, d, F, K, torch.bfloat16, 1), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    a = moc.moc_ffn_bwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], idx, gv, uv, Gd["dy"], ws=ws)
    torch.cuda.synchronize()
    ref = P.oracle_backward_for(L, idx.cpu().numpy(), P.to_np(gv), P.to_np(uv))
    for n, g, r in zip(("dx", "dwg", "dwu", "dwd"), a, ref):
        P.assert_close(n, P.to_np(g), r, P.TOL["bf16"])


# ------------------------------------------------------------------- dense SwiGLU call
@pytest.mark.parametrize("T,d,F,dtype", [(150, 128, 333, "bf16"), (64, 40, 90, "f32")])
def test_dense_swiglu_and_K_equal_F(T, d, F, dtype):
    say("[case] dense swiglu T=%d d=%d F=%d %s" % (T, d, F, dtype))
    tol = P.TOL[dtype]
    L = inputs.make_layer(93, T, d, F, dtype, with_dy=True)
    Gd = gpu_layer(L, dtype)
    Wg, Wu, Wd = P.paper_weights(L)
    X = L["x"].astype(np.float64)
    y, g_save, u_save = moc.moc_swiglu_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"])
    torch.cuda.synchronize()
    D, G, U = O.swiglu_forward(X, Wg, Wu, Wd)
    P.assert_close("y", P.to_np(y), D, tol)
    P.assert_close("g_save", P.to_np(g_save), G, tol)
    P.assert_close("u_save", P.to_np(u_save), U, tol)
    # K = F through the MoC entry point is the same function
    y2, idx, gv, uv = moc.moc_ffn_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], F)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), np.tile(np.arange(F, dtype=np.int32), (T, 1)))
    P.assert_close("y(K=F)", P.to_np(y2), D, tol)
    grads = moc.moc_swiglu_bwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], g_save, u_save, Gd["dy"])
    torch.cuda.synchronize()
    dX, dWg, dWu, dWd = O.swiglu_backward(X, Wg, Wu, Wd, P.to_np(g_save), P.to_np(u_save), L["dy"].astype(np.float64))
    for n, g, r in zip(("dx", "dwg", "dwu", "dwd"), grads, (dX, dWg.T, dWu.T, dWd)):
        P.assert_close(n, P.to_np(g), r, tol)


# ------------------------------------------------------------------------------ decode
def run_decode_case(tag, cfg_index, B, d, F, K, dtype, x_seed_offset=0):
    say("[case] %s decode B=%d d=%d F=%d K=%d %s" % (tag, B, d, F, K, dtype))
    tol = P.TOL[dtype]
    L = inputs.make_layer(cfg_index, B, d, F, dtype, x_seed_offset=x_seed_offset)
    Gd = gpu_layer(L, dtype)
    y, idx = moc.moc_ffn_decode(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K)
    torch.cuda.synchronize()
    idx_np = idx.cpu().numpy()
    Wg, Wu, Wd = P.paper_weights(L)
    X = L["x"].astype(np.float64)
    window = P.check_index_sets(idx_np, X @ Wg, K)
    y_ref, sets = O.moc_decode(X, Wg, Wu, Wd, K)
    keep = np.setdiff1d(np.arange(B), window)
    np.testing.assert_array_equal(idx_np[keep], sets[keep])
    if keep.size:
        P.assert_close("y", P.to_np(y)[keep], y_ref[keep], tol)
    D, _, _, _ = P.oracle_forward_for(L, idx_np)
    P.assert_close("y(given idx)", P.to_np(y), D, tol)
    # the training forward on the same rows picks the same channels and the same output
    y_f, idx_f, _, _ = moc.moc_ffn_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K)
    torch.cuda.synchronize()
    same = (idx_f == idx).all(dim=1).cpu().numpy()
    assert same[keep].all()
    P.assert_close("decode vs fwd", P.to_np(y)[same], P.to_np(y_f)[same], 2 * tol)
    # idx is optional
    y2, none = moc.moc_ffn_decode(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K, want_idx=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(y2, y)


@pytest.mark.parametrize("B", [1, 4, 16])
def test_cfg3_decode_7b_shape(B):
    c = CONFIGS["cfg3"]
    run_decode_case("cfg3", 3, B, c.d, c.F, c.K, "bf16", x_seed_offset=B)


@pytest.mark.parametrize("B,d,F,K,dtype", [(3, 64, 100, 9, "bf16"), (16, 256, 515, 64, "bf16"), (2, 36, 50, 50, "f32"),
                                           (7, 512, 1376, 172, "f32"), (9, 1024, 333, 40, "bf16"), (16, 2048, 1000, 125, "bf16")])
def test_decode_small_shapes(B, d, F, K, dtype):
    run_decode_case("small", 94, B, d, F, K, dtype)


# ------------------------------------------------------ RMSNorm, residual and the stack
@pytest.mark.parametrize("T,d", [(37, 200), (5, 203), (3, 4096), (2, 8192), (1, 1)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rmsnorm_and_residual(dtype, T, d):
    h = inputs.normal((T, d), 950, 1.0, dtype)
    gain = inputs.normal((d,), 951, 1.0, dtype)
    yv = inputs.normal((T, d), 952, 1.0, dtype)
    hd, gd, yd = P.to_dev(h, dtype), P.to_dev(gain, dtype), P.to_dev(yv, dtype)
    out = moc.moc_rmsnorm(hd, gd, RMSNORM_EPS)
    torch.cuda.synchronize()
    P.assert_close("rmsnorm", P.to_np(out), O.rmsnorm(h, gain, RMSNORM_EPS), P.TOL[dtype] / 2)
    moc.moc_residual_add(hd, yd)
    torch.cuda.synchronize()
    P.assert_close("residual", P.to_np(hd), O.residual_add(h, yv), P.TOL[dtype] / 2)


def test_cfg4_stack_teacher_forced_layers():
    """h <- h + MoC(RMSNorm(h)) at the 7B shape, all 32 layers with independent weights.  Each layer
    is checked against the oracle on one token row out of every band of 256 (so every row tile of
    the gate / up launch is sampled) plus the first and the last row, feeding the oracle the GPU's
    own layer input: after layer 1 the bf16 residual stream differs from float64 by far more than
    the spacing of gate values at the threshold, so end-to-end index parity is not defined.  The
    drift of the final residual stream against a float64 stack run on the sampled rows is printed
    as information."""
    from paper_2511_09323_amd.configs import STACK_LAYERS
    c = CONFIGS["cfg4"]
    T, d, F, K = c.T, c.d, c.F, c.K
    rng = np.random.default_rng(4)
    rows = np.unique(np.concatenate([[0, T - 1], np.arange(0, T, 256) + rng.integers(0, 256, size=T // 256)]))
    sel = torch.from_numpy(rows).cuda()
    h0_np = inputs.normal((T, d), inputs.seed_for(4, 0, "x"), 1.0, "bf16")
    h = P.to_dev(h0_np, "bf16")
    h_ref = h0_np[rows].astype(np.float64)          # float64 stack on the sampled rows (tokens are independent)
    gain_np = np.ones(d, dtype=np.float32)
    gain = P.to_dev(gain_np, "bf16")
    ws = torch.empty(moc.workspace_bytes(T, d, F, K, torch.bfloat16, 0), dtype=torch.uint8, device="cuda")
    in_window = 0
    for layer in range(STACK_LAYERS):
        say("[case] cfg4 stack layer %d" % layer)
        L = inputs.make_layer(4, 1, d, F, "bf16", layer=layer)
        Wd_ = {k: P.to_dev(L[k], "bf16") for k in ("wg", "wu", "wd")}
        h_in = P.to_np(h[sel])
        xn = moc.moc_rmsnorm(h, gain, RMSNORM_EPS)
        y, idx, _, _ = moc.moc_ffn_fwd(xn, Wd_["wg"], Wd_["wu"], Wd_["wd"], K, ws=ws)
        moc.moc_residual_add(h, y)
        torch.cuda.synchronize()
        P.assert_close("rmsnorm", P.to_np(xn[sel]), O.rmsnorm(h_in, gain_np, RMSNORM_EPS), 1e-2)
        Ls = {"x": xn[sel].float().cpu().numpy(), "wg": L["wg"], "wu": L["wu"], "wd": L["wd"]}
        idx_np = idx[sel].cpu().numpy()
        D, _, _, G64 = P.oracle_forward_for(Ls, idx_np)
        window = P.check_index_sets(idx_np, G64, K)
        in_window += len(window)
        assert len(window) <= 2
        P.assert_close("y", P.to_np(y[sel]), D, P.TOL["bf16"])
        P.assert_close("h", P.to_np(h[sel]), O.residual_add(h_in, P.to_np(y[sel])), 1e-2)
        # the float64 stack on its own trajectory (own selection), for the drift figure only
        Wg, Wu, Wdn = P.paper_weights(L)
        Dr = O.moc_forward(O.rmsnorm(h_ref, gain_np, RMSNORM_EPS), Wg, Wu, Wdn, K)[0]
        h_ref = O.residual_add(h_ref, Dr)
        del Wd_, L
    drift = np.abs(P.to_np(h[sel]).astype(np.float64) - h_ref).max() / np.abs(h_ref).max()
    say("[info] cfg4: %d sampled rows x %d layers, %d rows inside the near-tie window; max-norm drift of h_%d against "
        "the float64 stack: %.3e" % (len(rows), STACK_LAYERS, in_window, STACK_LAYERS, drift))


# ------------------------------------------------------------------------- graph capture
def test_forward_backward_and_decode_replay_from_a_graph():
    """The library allocates nothing, records no memset and keeps no per-call state, so a captured
    graph of its calls can be replayed on new data; every replay must equal the eager result bit
    for bit (replays are interleaved with eager work and synchronisation)."""
    T, d, F, K, B = 300, 256, 520, 65, 4
    dt = torch.bfloat16
    L = inputs.make_layer(92, T, d, F, "bf16", with_dy=True)
    Gd = gpu_layer(L, "bf16")
    x, dy = Gd["x"].clone(), Gd["dy"].clone()
    xd = x[:B].clone()
    ws_f = torch.empty(moc.workspace_bytes(T, d, F, K, dt, 0), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(moc.workspace_bytes(T, d, F, K, dt, 1), dtype=torch.uint8, device="cuda")
    ws_d = torch.empty(moc.workspace_bytes(B, d, F, K, dt, 2), dtype=torch.uint8, device="cuda")
    out_f = (torch.empty((T, d), dtype=dt, device="cuda"), torch.empty((T, K), dtype=torch.int32, device="cuda"),
             torch.empty((T, K), dtype=dt, device="cuda"), torch.empty((T, K), dtype=dt, device="cuda"))
    out_b = tuple(torch.empty(s, dtype=dt, device="cuda") for s in ((T, d), (F, d), (F, d), (F, d)))
    out_d = (torch.empty((B, d), dtype=dt, device="cuda"), torch.empty((B, K), dtype=torch.int32, device="cuda"))

    def run():
        y, idx, gv, uv = moc.moc_ffn_fwd(x, Gd["wg"], Gd["wu"], Gd["wd"], K, ws=ws_f, out=out_f)
        moc.moc_ffn_bwd(x, Gd["wg"], Gd["wu"], Gd["wd"], idx, gv, uv, dy, ws=ws_b, out=out_b)
        moc.moc_ffn_decode(xd, Gd["wg"], Gd["wu"], Gd["wd"], K, ws=ws_d, out=out_d)

    # no warm-up call: the library's per-device set-up makes no stream operation, so even the first
    # call of a process may be captured
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        x.copy_(P.to_dev(inputs.normal((T, d), 9200 + rep, 1.0, "bf16"), "bf16"))
        dy.copy_(P.to_dev(inputs.normal((T, d), 9210 + rep, 1.0, "bf16"), "bf16"))
        xd.copy_(x[:B])
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (*out_f, *out_b, *out_d)]
        for t in (*out_f, *out_b, *out_d):
            t.zero_()
        run()                                   # eager, same buffers
        torch.cuda.synchronize()
        for g, w in zip(got, (*out_f, *out_b, *out_d)):
            assert torch.equal(g, w), "replay %d differs from the eager run" % rep


@pytest.mark.parametrize("B", [1, 4, 16])
def test_decode_workspace_reuse_and_ties(B):
    run_decode_reuse_case(B, 1024, 2752, 344)


def test_persistent_single_launch_decode():
    """MOC_DECODE_PERSISTENT=1 (read once per process, hence the child process) runs row-wide decode as one
    persistent launch: gate, exact selection, union gather of W_up and W_down with data-flow
    synchronisation between the workgroups.  Same oracle checks as the default path, at the 7B shape for
    1, 4 and 16 tokens (both kernel variants), on small and odd shapes, twice in a row on one workspace
    (the tag of a call must not match what the previous call left), and bit-identical on repetition."""
    import os
    import subprocess
    code = ("import torch\n"
            "import tests.test_gpu_parity as t\n"
            "from paper_2511_09323_amd.configs import CONFIGS\n"
            "c = CONFIGS['cfg3']\n"
            "for B in (1, 4, 16):\n"
            "    t.run_decode_case('cfg3-persistent', 3, B, c.d, c.F, c.K, 'bf16', x_seed_offset=B)\n"
            "for B, d, F, K, dt in ((3, 64, 100, 9, 'bf16'), (2, 36, 50, 50, 'f32'), (9, 1024, 333, 40, 'bf16'),\n"
            "                       (16, 2048, 1000, 125, 'bf16'), (1, 512, 1376, 172, 'f32'), (4, 768, 2048, 256, 'bf16')):\n"
            "    t.run_decode_case('small-persistent', 94, B, d, F, K, dt)\n"
            "for B in (1, 4, 16):\n"
            "    t.run_decode_reuse_case(B, 1024, 2752, 344)\n"
            "print('ok')\n")
    env = dict(os.environ, MOC_DECODE_PERSISTENT="1")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-3000:] + r.stderr[-3000:]


def test_decode_with_the_selection_inside_the_gather_launch():
    """MOC_DECODE_SELECT_GATHER=1 (read once per process, hence the child process): every gather workgroup of
    row-wide decode finds its token's Top-K threshold itself, so the selection needs no launch of its own.  Same
    oracle checks as the default path at the 7B shape for 1, 4 and 16 tokens, on small, odd and fp32 shapes (rows
    shorter than one chunk of keys, K = F, ranges that end inside a 32-channel word), and on one workspace reused
    with tied gate values."""
    import os
    import subprocess
    code = ("import tests.test_gpu_parity as t\n"
            "from paper_2511_09323_amd.configs import CONFIGS\n"
            "c = CONFIGS['cfg3']\n"
            "for B in (1, 4, 16):\n"
            "    t.run_decode_case('cfg3-select-gather', 3, B, c.d, c.F, c.K, 'bf16', x_seed_offset=B)\n"
            "for B, d, F, K, dt in ((3, 64, 100, 9, 'bf16'), (2, 36, 50, 50, 'f32'), (9, 1024, 333, 40, 'bf16'),\n"
            "                       (16, 2048, 1000, 125, 'bf16'), (1, 512, 1376, 172, 'f32'), (4, 768, 2048, 256, 'bf16'),\n"
            "                       (5, 256, 20000, 2500, 'bf16')):\n"
            "    t.run_decode_case('small-select-gather', 94, B, d, F, K, dt)\n"
            "for B in (1, 4, 16):\n"
            "    t.run_decode_reuse_case(B, 1024, 2752, 344)\n"
            "print('ok')\n")
    env = dict(os.environ, MOC_DECODE_SELECT_GATHER="1")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-3000:] + r.stderr[-3000:]


def run_decode_reuse_case(B, d, F, K):
    """Three decode calls on ONE workspace with different inputs, then the first again: every result must
    equal that of a fresh workspace bit for bit (nothing a call leaves in the workspace may leak into the
    next), and tied gate values (a repeated weight row) must be cut at the lower channel."""
    dt = torch.bfloat16
    ws = torch.empty(moc.workspace_bytes(B, d, F, K, dt, 2), dtype=torch.uint8, device="cuda")
    ws.fill_(0xAB)                                 # not zero: the kernels must not rely on a cleared workspace
    cases = []
    for s in range(3):
        L = inputs.make_layer(96 + s, B, d, F, "bf16")
        if s == 1:
            L["wg"][7] = L["wg"][3]                # channels 3 and 7 tie for every token
            L["wg"][F - 1] = L["wg"][3]
        cases.append({k: P.to_dev(v, "bf16") for k, v in L.items()})
    fresh = []
    for G in cases:
        y, idx = moc.moc_ffn_decode(G["x"], G["wg"], G["wu"], G["wd"], K)
        fresh.append((y.clone(), idx.clone()))
    for rep in (0, 1, 2, 0, 0):
        G = cases[rep]
        y, idx = moc.moc_ffn_decode(G["x"], G["wg"], G["wu"], G["wd"], K, ws=ws)
        torch.cuda.synchronize()
        assert torch.equal(idx, fresh[rep][1]) and torch.equal(y, fresh[rep][0]), "reuse %d" % rep
    # the tied channels: never 7 without 3, never the last one without 7
    idx1 = fresh[1][1].cpu().numpy()
    for row in idx1:
        s = set(row.tolist())
        assert not (7 in s and 3 not in s) and not (F - 1 in s and 7 not in s)


def test_gemms_split_along_the_contraction():
    """MOC_GEMM_STREAMK=1 (read once per process, hence the child process) lets the products whose whole tiles
    would leave part of the chip idle in their last round split their work along the contraction: workgroups
    hand partial accumulators to each other through the workspace.  Same oracle checks as the default path at
    the 1B shape (gate, up, dZ' and the three weight gradients take the split) and at a shape with 17 k-slices
    and ragged edges; twice on one workspace filled with junk (the words the workgroups signal through need no
    initialisation and are left clean), bit-identical."""
    import os
    import subprocess
    code = ("import torch\n"
            "import tests.test_gpu_parity as t\n"
            "from paper_2511_09323_amd.configs import CONFIGS\n"
            "import paper_2511_09323_amd as moc\n"
            "c = CONFIGS['cfg2']\n"
            "t.run_fwd_bwd_case('cfg2-split', 2, c.T, c.d, c.F, c.K, 'bf16', expect_window_rows=40)\n"
            "t.run_fwd_bwd_case('ragged-split', 93, 8100, 544, 2500, 300, 'bf16')\n"
            "L = t.inputs.make_layer(93, 8100, 544, 2500, 'bf16')\n"
            "G = t.gpu_layer(L, 'bf16')\n"
            "ws = torch.empty(moc.workspace_bytes(8100, 544, 2500, 300, torch.bfloat16, 0), dtype=torch.uint8, device='cuda')\n"
            "ws.fill_(0x5A)\n"
            "outs = []\n"
            "for rep in range(3):\n"
            "    y, idx, gv, uv = moc.moc_ffn_fwd(G['x'], G['wg'], G['wu'], G['wd'], 300, ws=ws)\n"
            "    torch.cuda.synchronize()\n"
            "    outs.append((y.clone(), idx.clone()))\n"
            "assert all(torch.equal(o[0], outs[0][0]) and torch.equal(o[1], outs[0][1]) for o in outs)\n"
            "print('ok')\n")
    env = dict(os.environ, MOC_GEMM_STREAMK="1")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-3000:] + r.stderr[-3000:]
    # the path a workgroup takes when its neighbour's share does not arrive: with no polls at all every workgroup
    # multiplies the rest of its last tile itself (the host forces this; nothing waits, nothing hangs)
    code2 = ("import tests.test_gpu_parity as t\n"
             "t.run_fwd_bwd_case('ragged-split-no-wait', 93, 8100, 544, 2500, 300, 'bf16')\n"
             "print('ok')\n")
    env2 = dict(env, MOC_GEMM_STREAMK_SPIN="0")
    r = subprocess.run([sys.executable, "-c", code2], cwd=root, env=env2, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-3000:] + r.stderr[-3000:]


def test_generic_kernels_serve_bf16_when_forced():
    """MOC_FORCE_GENERIC=1 (read once per process, hence the child process) routes every bf16 GEMM to the
    fp32-FMA kernel and decode to its non-MFMA kernels; results must still match the oracle."""
    import os
    import subprocess
    code = ("import tests.test_gpu_parity as t\n"
            "t.run_fwd_bwd_case('forced-generic', 91, 150, 128, 330, 41, 'bf16')\n"
            "t.run_decode_case('forced-generic', 91, 9, 1024, 336, 42, 'bf16')\n"
            "print('ok')\n")
    env = dict(os.environ, MOC_FORCE_GENERIC="1")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-2000:] + r.stderr[-2000:]
