"""GPU parity for MoC as the MLP of MoE experts: rows sorted by expert, one grouped launch per
projection, against the oracle's expert-by-expert evaluation (paper section "Compatibility with
MoE architectures"; shapes of its Mixtral table: 8 experts, 2 per token, hidden 512 / 768,
intermediate 1376 / 2048, K = hidden / 2)."""
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


def make_experts(seed, E, d, F, dtype):
    """Channel-major expert weights [E, F, d] with the usual N(0, 0.02^2) entries."""
    return {n: np.stack([inputs.normal((F, d), seed + 10 * e + i, 0.02, dtype) for e in range(E)])
            for i, n in enumerate(("wg", "wu", "wd"))}


def run_experts_case(tag, seed, counts, d, F, K, dtype, bwd=True):
    E = len(counts)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    A = int(offsets[-1])
    say("[case] %s experts=%s d=%d F=%d K=%d %s" % (tag, list(counts), d, F, K, dtype))
    tol = P.TOL[dtype]
    W = make_experts(seed, E, d, F, dtype)
    x = inputs.normal((A, d), seed + 100, 1.0, dtype)
    dy = inputs.normal((A, d), seed + 101, 1.0, dtype)
    Wd_ = {k: P.to_dev(v, dtype) for k, v in W.items()}
    xd, dyd = P.to_dev(x, dtype), P.to_dev(dy, dtype)
    y, idx, gvals, uvals = moc.moc_ffn_fwd_experts(xd, offsets, Wd_["wg"], Wd_["wu"], Wd_["wd"], K)
    torch.cuda.synchronize()
    idx_np = idx.cpu().numpy()
    Wg = [W["wg"][e].astype(np.float64).T for e in range(E)]
    Wu = [W["wu"][e].astype(np.float64).T for e in range(E)]
    Wdn = [W["wd"][e].astype(np.float64) for e in range(E)]
    X64 = x.astype(np.float64)
    # index sets against the oracle's own selection, expert by expert
    G64 = np.zeros((A, F))
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        G64[lo:hi] = X64[lo:hi] @ Wg[e]
    window = P.check_index_sets(idx_np, G64, K) if A else []
    assert len(window) <= max(2, A // 200)
    # values against the oracle evaluated on the GPU's index sets
    M = O.mask_from_idx(idx_np, F)
    D = np.zeros((A, d))
    U64 = np.zeros((A, F))
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:
            D[lo:hi], _, U64[lo:hi] = O.moc_forward_given_mask(X64[lo:hi], Wg[e], Wu[e], Wdn[e], M[lo:hi])
    rows = np.arange(A)[:, None]
    P.assert_close("y", P.to_np(y), D, tol)
    P.assert_close("gvals", P.to_np(gvals), G64[rows, idx_np], tol)
    P.assert_close("uvals", P.to_np(uvals), U64[rows, idx_np], tol)
    if not bwd:
        return
    dx, dwg, dwu, dwd = moc.moc_ffn_bwd_experts(xd, offsets, Wd_["wg"], Wd_["wu"], Wd_["wd"], idx, gvals, uvals, dyd)
    torch.cuda.synchronize()
    Ms, GM, UM = O.expand_saved(idx_np, P.to_np(gvals), P.to_np(uvals), F)
    rdx, rdwg, rdwu, rdwd = O.moc_backward_experts(X64, offsets, Wg, Wu, Wdn, Ms, GM, UM, dy.astype(np.float64))
    P.assert_close("dx", P.to_np(dx), rdx, tol)
    for e in range(E):
        if counts[e] == 0:
            for g in (dwg, dwu, dwd):
                assert float(g[e].abs().max()) == 0.0, "an expert without rows must get zero gradients"
            continue
        P.assert_close("dwg[%d]" % e, P.to_np(dwg[e]), rdwg[e].T, tol)
        P.assert_close("dwu[%d]" % e, P.to_np(dwu[e]), rdwu[e].T, tol)
        P.assert_close("dwd[%d]" % e, P.to_np(dwd[e]), rdwd[e], tol)


def test_one_expert_is_the_plain_layer():
    T, d, F, K = 300, 128, 520, 65
    W = make_experts(700, 1, d, F, "bf16")
    x = P.to_dev(inputs.normal((T, d), 800, 1.0, "bf16"), "bf16")
    Wd_ = {k: P.to_dev(v, "bf16") for k, v in W.items()}
    y, idx, gv, uv = moc.moc_ffn_fwd_experts(x, [0, T], Wd_["wg"], Wd_["wu"], Wd_["wd"], K)
    y0, idx0, gv0, uv0 = moc.moc_ffn_fwd(x, Wd_["wg"][0], Wd_["wu"][0], Wd_["wd"][0], K)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx0) and torch.equal(y, y0) and torch.equal(gv, gv0) and torch.equal(uv, uv0)


@pytest.mark.parametrize("counts,d,F,K,dtype", [
    ((40, 0, 33, 200, 7, 64, 90, 50), 128, 520, 65, "bf16"),       # ragged, one empty, one below 32 rows
    ((64, 96, 160), 96, 200, 25, "f32"),
    ((256, 512, 0, 300), 256, 1376, 172, "bf16"),
    ((35,), 64, 96, 12, "bf16"),
])
def test_experts_small_shapes(counts, d, F, K, dtype):
    run_experts_case("small", 600, counts, d, F, K, dtype)


def test_experts_mixtral_180m_shape():
    # 8 experts, 2 per token: 2048 tokens -> 4096 routed rows with an uneven split
    counts = (700, 420, 512, 384, 650, 330, 600, 500)
    run_experts_case("mixtral-180M", 610, counts, 512, 1376, 256, "bf16")


def test_experts_bad_arguments():
    d, F, K = 64, 96, 12
    W = make_experts(620, 2, d, F, "bf16")
    Wd_ = {k: P.to_dev(v, "bf16") for k, v in W.items()}
    x = P.to_dev(inputs.normal((50, d), 621, 1.0, "bf16"), "bf16")
    for offsets in ([0, 60, 50], [1, 20, 50], [0, 20, 49]):
        with pytest.raises(moc.MocError):
            moc.moc_ffn_fwd_experts(x, offsets, Wd_["wg"], Wd_["wu"], Wd_["wd"], K)
