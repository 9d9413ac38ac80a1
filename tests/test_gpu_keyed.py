"""GPU parity for the Top-K position variants (ranking SiLU(g) or |SiLU(g)| instead of g): selection
alone on given values, training forward + backward, and decode, through the C ABI against the oracle."""
import sys

import numpy as np
import pytest
import torch

import paper_2511_09323_amd as moc
from oracle import moc_oracle as O
from paper_2511_09323_amd import inputs
from tests import parity as P

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def gpu_layer(L, dtype):
    return {k: P.to_dev(v, dtype) for k, v in L.items()}


@pytest.mark.parametrize("key", ["gate", "silu", "abs_silu"])
def test_keyed_selection_on_given_values(key):
    rng = np.random.default_rng(41)
    for T, F, K in [(4, 64, 9), (9, 333, 200), (6, 5461, 683), (3, 11008, 1376), (2, 11008, 9000), (5, 1001, 500)]:
        say("[keyed %s] T=%d F=%d K=%d" % (key, T, F, K))
        g_np = (rng.standard_normal((T, F)) * 1.3).astype(np.float32)
        idx, gsel = moc.moc_topk_rows_keyed(torch.from_numpy(g_np).cuda(), K, key)
        torch.cuda.synchronize()
        idx_np = idx.cpu().numpy()
        window = P.check_keyed_index_sets(idx_np, g_np.astype(np.float64), K, key)
        assert len(window) <= 1
        # gsel holds the gate values themselves at the selected channels, whatever was ranked
        np.testing.assert_array_equal(gsel.cpu().numpy(), np.take_along_axis(g_np, idx_np, axis=1))
    # hand case around SiLU's minimum (the same as the oracle's pin)
    g = torch.tensor([[-6.0, -1.3, -0.5, 0.05, 0.3, -3.0]], dtype=torch.float32, device="cuda")
    want = {"gate": [2, 3, 4], "silu": [0, 3, 4], "abs_silu": [1, 2, 4]}[key]
    idx, _ = moc.moc_topk_rows_keyed(g, 3, key)
    assert idx.cpu().numpy().tolist() == [want]


@pytest.mark.parametrize("key", ["silu", "abs_silu"])
@pytest.mark.parametrize("T,d,F,K,dtype", [(200, 128, 520, 300, "bf16"), (64, 96, 200, 150, "f32"), (1024, 768, 2048, 256, "bf16")])
def test_keyed_forward_backward(T, d, F, K, dtype, key):
    say("[case] keyed %s T=%d d=%d F=%d K=%d %s" % (key, T, d, F, K, dtype))
    tol = P.TOL[dtype]
    L = inputs.make_layer(90, T, d, F, dtype, with_dy=True)
    if K > F // 4:
        L["wg"] = L["wg"] * np.float32(8.0)            # wider gates: many values below SiLU's minimum matter at large K
        if dtype == "bf16":
            L["wg"] = inputs.round_to_bf16(L["wg"])
    Gd = gpu_layer(L, dtype)
    y, idx, gvals, uvals = moc.moc_ffn_fwd_keyed(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K, key)
    torch.cuda.synchronize()
    idx_np = idx.cpu().numpy()
    D, gv_ref, uv_ref, G64 = P.oracle_forward_for(L, idx_np)
    window = P.check_keyed_index_sets(idx_np, G64, K, key)
    say("  %d of %d rows inside the near-tie window" % (len(window), T))
    assert len(window) <= max(2, T // 50)
    P.assert_close("y", P.to_np(y), D, tol)
    P.assert_close("gvals", P.to_np(gvals), gv_ref, tol)
    P.assert_close("uvals", P.to_np(uvals), uv_ref, tol)
    if K > F // 4:
        # the variant really selects something else than the raw gate does on these inputs
        assert (O.topk_mask_keyed(G64, K, key) != O.topk_mask(G64, K)).any()
    dx, dwg, dwu, dwd = moc.moc_ffn_bwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], idx, gvals, uvals, Gd["dy"])
    torch.cuda.synchronize()
    ref = P.oracle_backward_for(L, idx_np, P.to_np(gvals), P.to_np(uvals))
    for n, g, r in zip(("dx", "dwg", "dwu", "dwd"), (dx, dwg, dwu, dwd), ref):
        P.assert_close(n, P.to_np(g), r, tol)
    # key "gate" is the plain call
    y0, idx0, _, _ = moc.moc_ffn_fwd_keyed(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K, "gate")
    y1, idx1, _, _ = moc.moc_ffn_fwd(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K)
    torch.cuda.synchronize()
    assert torch.equal(idx0, idx1) and torch.equal(y0, y1)


@pytest.mark.parametrize("key", ["silu", "abs_silu"])
@pytest.mark.parametrize("B,d,F,K", [(1, 4096, 11008, 1376), (4, 1024, 2048, 1200), (16, 2048, 1000, 700)])
def test_keyed_decode(B, d, F, K, key):
    say("[case] keyed %s decode B=%d d=%d F=%d K=%d" % (key, B, d, F, K))
    L = inputs.make_layer(89, B, d, F, "bf16")
    if K > F // 4:
        L["wg"] = inputs.round_to_bf16(L["wg"] * np.float32(4.0))
    Gd = gpu_layer(L, "bf16")
    y, idx = moc.moc_ffn_decode_keyed(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K, key)
    torch.cuda.synchronize()
    idx_np = idx.cpu().numpy()
    Wg, Wu, Wd = P.paper_weights(L)
    X = L["x"].astype(np.float64)
    P.check_keyed_index_sets(idx_np, X @ Wg, K, key)
    D, _, _, _ = P.oracle_forward_for(L, idx_np)
    P.assert_close("y(given idx)", P.to_np(y), D, P.TOL["bf16"])
    y_f, idx_f, _, _ = moc.moc_ffn_fwd_keyed(Gd["x"], Gd["wg"], Gd["wu"], Gd["wd"], K, key)
    torch.cuda.synchronize()
    same = (idx_f == idx).all(dim=1).cpu().numpy()
    assert same.sum() >= B - 1
    P.assert_close("decode vs fwd", P.to_np(y)[same], P.to_np(y_f)[same], 2 * P.TOL["bf16"])


def test_keyed_bad_arguments():
    g = torch.zeros((2, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(moc.MocError):
        moc.moc_topk_rows_keyed(g, 4, "largest")
