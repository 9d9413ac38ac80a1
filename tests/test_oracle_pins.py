"""Pins for the CPU oracle: every check compares oracle/moc_oracle.py with something that is not
itself -- a hand-worked example, brute force, library routines (numpy partition, torch topk,
torch silu / rms_norm / autograd), finite differences, or an invariant of the method."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import brute
from oracle import moc_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")


def _rand_layer(seed, s, d, F, scale=0.3):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((s, d))
    Wg = rng.standard_normal((d, F)) * scale
    Wu = rng.standard_normal((d, F)) * scale
    Wd = rng.standard_normal((F, d)) * scale
    return X, Wg, Wu, Wd


# ----------------------------------------------------------------- hand-worked example
def test_hand_example_forward_and_backward():
    g = json.load(open(GOLDEN))
    X, Wg, Wu, Wd = (np.array(g[k]) for k in ("X", "W_gate", "W_up", "W_down"))
    D, M, G, U = O.moc_forward(X, Wg, Wu, Wd, g["K"])
    np.testing.assert_allclose(G, g["G"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(U, g["U"], rtol=0, atol=1e-15)
    assert [list(np.flatnonzero(r)) for r in M] == g["C"]
    np.testing.assert_allclose(D, g["D"], rtol=1e-14)
    idx, gv, uv = O.compact_saved(M, G, U)
    assert idx.tolist() == g["C"]
    M2, GM, UM = O.expand_saved(idx, gv, uv, 4)
    dX, dWg, dWu, dWd = O.moc_backward(X, Wg, Wu, Wd, M2, GM, UM, np.array(g["dD"]))
    np.testing.assert_allclose(dX, g["dX"], rtol=1e-13)
    np.testing.assert_allclose(dWd, g["dW_down"], rtol=1e-13, atol=1e-300)
    np.testing.assert_allclose(dWg, g["dW_gate"], rtol=1e-13, atol=1e-300)
    np.testing.assert_allclose(dWu, g["dW_up"], rtol=1e-13, atol=1e-300)
    # the decode recipe gives the same token output and set
    dvec, C = O.moc_decode(X[0], Wg, Wu, Wd, g["K"])
    np.testing.assert_allclose(dvec, g["D"][0], rtol=1e-14)
    assert C.tolist() == g["C"][0]


def test_silu_closed_forms():
    assert O.silu(0.0) == 0.0
    np.testing.assert_allclose(O.silu(np.array([3.0, 2.0])), [3 / (1 + np.exp(-3)), 2 / (1 + np.exp(-2))], rtol=1e-15)
    # SiLU(x) - SiLU(-x) = x, SiLU'(0) = 1/2, SiLU'(x) + SiLU'(-x) = 1
    x = np.linspace(-20, 20, 401)
    np.testing.assert_allclose(O.silu(x) - O.silu(-x), x, atol=1e-12)
    assert O.silu_grad(0.0) == 0.5
    np.testing.assert_allclose(O.silu_grad(x) + O.silu_grad(-x), 1.0, atol=1e-12)
    # against torch's own silu and its autograd derivative
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.silu(xt)
    yt.sum().backward()
    np.testing.assert_allclose(O.silu(x), yt.detach().numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O.silu_grad(x), xt.grad.numpy(), rtol=1e-12, atol=1e-15)
    # extreme arguments stay finite
    assert np.all(np.isfinite(O.silu(np.array([-1000.0, 1000.0]))))


# ---------------------------------------------------------------------------- selection
@pytest.mark.parametrize("seed,s,F,K", [(0, 7, 33, 1), (1, 5, 64, 8), (2, 9, 100, 37), (3, 3, 17, 17), (4, 4, 257, 256)])
def test_topk_matches_brute_force_and_libraries(seed, s, F, K):
    rng = np.random.default_rng(seed)
    G = rng.standard_normal((s, F))
    M = O.topk_mask(G, K)
    assert M.sum(axis=1).tolist() == [K] * s
    G32 = G.astype(np.float32)
    for i in range(s):
        assert list(np.flatnonzero(M[i])) == brute.select_full_sort(list(G[i]), K)
        sel, rest = G32[i][M[i]], G32[i][~M[i]]
        if rest.size:
            assert sel.min() >= rest.max()
        # value multiset against numpy's partition and torch's topk (independent routines)
        part = np.sort(np.partition(G32[i], F - K)[F - K:])
        np.testing.assert_array_equal(np.sort(sel), part)
        tk = torch.topk(torch.from_numpy(G32[i]), K).values.numpy()
        np.testing.assert_array_equal(np.sort(sel), np.sort(tk))


def test_topk_is_signed_not_absolute():
    G = np.array([[-9.0, 1.0, 0.5, -0.1]])
    assert list(np.flatnonzero(O.topk_mask(G, 2)[0])) == [1, 2]


def test_topk_ties_lower_index_wins_and_signed_zero():
    G = np.array([[1.0, 2.0, 1.0, 1.0, 0.0, 1.0]])
    assert list(np.flatnonzero(O.topk_mask(G, 3)[0])) == [0, 1, 2]
    Z = np.array([[-0.0, 0.0, -0.0, 0.0, -1.0]])
    assert list(np.flatnonzero(O.topk_mask(Z, 2)[0])) == [0, 1]
    # values that differ in float64 but collapse in float32 count as a tie
    T = np.array([[1.0, 1.0 + 1e-12, 0.0]])
    assert list(np.flatnonzero(O.topk_mask(T, 1)[0])) == [0]


def test_topk_rejects_bad_arguments():
    with pytest.raises(ValueError):
        O.topk_mask(np.zeros((1, 4)), 0)
    with pytest.raises(ValueError):
        O.topk_mask(np.zeros((1, 4)), 5)
    with pytest.raises(ValueError):
        O.topk_mask(np.array([[1.0, np.nan]]), 1)


# ------------------------------------------------------------------------------ forward
def test_forward_matches_loop_twin():
    X, Wg, Wu, Wd = _rand_layer(10, 4, 5, 12)
    D, M, _, _ = O.moc_forward(X, Wg, Wu, Wd, 3)
    Db, sets = brute.moc_forward_loops(X.tolist(), Wg.tolist(), Wu.tolist(), Wd.tolist(), 3)
    np.testing.assert_allclose(D, np.array(Db), rtol=1e-12, atol=1e-14)
    assert [list(np.flatnonzero(r)) for r in M] == sets


def test_K_equal_dffn_is_dense_swiglu_by_torch():
    X, Wg, Wu, Wd = _rand_layer(11, 6, 8, 20)
    D, M, _, _ = O.moc_forward(X, Wg, Wu, Wd, 20)
    assert M.all()
    Xt, Wgt, Wut, Wdt = (torch.from_numpy(a) for a in (X, Wg, Wu, Wd))
    ref = (torch.nn.functional.silu(Xt @ Wgt) * (Xt @ Wut)) @ Wdt
    np.testing.assert_allclose(D, ref.numpy(), rtol=1e-12, atol=1e-14)
    Dd, _, _ = O.swiglu_forward(X, Wg, Wu, Wd)
    np.testing.assert_allclose(Dd, ref.numpy(), rtol=1e-12, atol=1e-14)


def test_decode_recipe_equals_training_forward():
    X, Wg, Wu, Wd = _rand_layer(12, 5, 16, 48)
    D, M, _, _ = O.moc_forward(X, Wg, Wu, Wd, 6)
    Dd, sets = O.moc_decode(X, Wg, Wu, Wd, 6)
    np.testing.assert_allclose(Dd, D, rtol=1e-12, atol=1e-14)
    assert [list(np.flatnonzero(r)) for r in M] == sets.tolist()


def test_unselected_channels_contribute_nothing():
    X, Wg, Wu, Wd = _rand_layer(13, 6, 10, 40)
    K = 4
    D, M, G, U = O.moc_forward(X, Wg, Wu, Wd, K)
    dD = np.random.default_rng(99).standard_normal(D.shape)
    idx, gv, uv = O.compact_saved(M, G, U)
    base = O.moc_backward(X, Wg, Wu, Wd, *O.expand_saved(idx, gv, uv, 40), dD)
    unused = ~M.any(axis=0)
    assert unused.any()
    Wu2, Wd2 = Wu.copy(), Wd.copy()
    Wu2[:, unused] = 1e6
    Wd2[unused, :] = -1e6
    D2, M2, G2, U2 = O.moc_forward(X, Wg, Wu2, Wd2, K)
    np.testing.assert_array_equal(D2, D)
    np.testing.assert_array_equal(M2, M)
    dX2, dWg2, dWu2, dWd2 = O.moc_backward(X, Wg, Wu2, Wd2, *O.expand_saved(idx, gv, uv, 40), dD)
    np.testing.assert_array_equal(dX2, base[0])
    for grad in (base[1].T, base[2].T, base[3]):          # channel-major views
        assert np.all(grad[unused] == 0.0)
    # a channel's weight gradients depend only on the tokens that selected it
    j = int(np.flatnonzero(M.any(axis=0))[0])
    toks = np.flatnonzero(M[:, j])
    sub = O.moc_backward(X[toks], Wg, Wu, Wd, *O.expand_saved(idx[toks], gv[toks], uv[toks], 40), dD[toks])
    np.testing.assert_allclose(sub[3][j], base[3][j], rtol=1e-12)
    np.testing.assert_allclose(sub[1][:, j], base[1][:, j], rtol=1e-12)


def test_token_independence_permutation_and_gate_scaling():
    X, Wg, Wu, Wd = _rand_layer(14, 8, 12, 30)
    K = 5
    D, M, _, _ = O.moc_forward(X, Wg, Wu, Wd, K)
    rows = [6, 1, 3]
    Ds, Ms, _, _ = O.moc_forward(X[rows], Wg, Wu, Wd, K)
    np.testing.assert_array_equal(Ds, D[rows])
    np.testing.assert_array_equal(Ms, M[rows])
    perm = np.random.default_rng(5).permutation(30)
    Dp, Mp, _, _ = O.moc_forward(X, Wg[:, perm], Wu[:, perm], Wd[perm, :], K)
    np.testing.assert_allclose(Dp, D, rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(Mp, M[:, perm])
    _, Mc, _, _ = O.moc_forward(X, 4.0 * Wg, Wu, Wd, K)       # power-of-two scale: exact
    np.testing.assert_array_equal(Mc, M)


# ----------------------------------------------------------------------------- backward
def _torch_masked_dense(X, Wg, Wu, Wd, M, dD):
    Xt, Wgt, Wut, Wdt = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (X, Wg, Wu, Wd))
    Mt = torch.tensor(M, dtype=torch.float64)
    D = ((torch.nn.functional.silu(Xt @ Wgt) * Mt) * (Xt @ Wut)) @ Wdt
    D.backward(torch.tensor(dD, dtype=torch.float64))
    return D.detach().numpy(), [t.grad.numpy() for t in (Xt, Wgt, Wut, Wdt)]


@pytest.mark.parametrize("K", [3, 24])
def test_backward_matches_torch_autograd(K):
    X, Wg, Wu, Wd = _rand_layer(20, 7, 9, 24)
    D, M, G, U = O.moc_forward(X, Wg, Wu, Wd, K)
    dD = np.random.default_rng(21).standard_normal(D.shape)
    Dt, grads_t = _torch_masked_dense(X, Wg, Wu, Wd, M, dD)
    np.testing.assert_allclose(D, Dt, rtol=1e-12, atol=1e-14)
    grads = O.moc_backward(X, Wg, Wu, Wd, M, G * M, U * M, dD)
    for a, b in zip(grads, grads_t):
        np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)
    if K == 24:     # dense special case
        dense = O.swiglu_backward(X, Wg, Wu, Wd, G, U, dD)
        for a, b in zip(dense, grads_t):
            np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)


def test_backward_matches_finite_differences_with_frozen_mask():
    X, Wg, Wu, Wd = _rand_layer(22, 3, 4, 10)
    K = 3
    D, M, G, U = O.moc_forward(X, Wg, Wu, Wd, K)
    dD = np.random.default_rng(23).standard_normal(D.shape)
    grads = O.moc_backward(X, Wg, Wu, Wd, M, G * M, U * M, dD)

    def loss(X_, Wg_, Wu_, Wd_):
        D_, _, _ = O.moc_forward_given_mask(X_, Wg_, Wu_, Wd_, M)
        return float(np.sum(D_ * dD))

    h = 1e-6
    args = [X, Wg, Wu, Wd]
    for which in range(4):
        num = np.zeros_like(args[which])
        it = np.nditer(args[which], flags=["multi_index"])
        for _ in it:
            mi = it.multi_index
            plus = [a.copy() for a in args]
            minus = [a.copy() for a in args]
            plus[which][mi] += h
            minus[which][mi] -= h
            num[mi] = (loss(*plus) - loss(*minus)) / (2 * h)
        np.testing.assert_allclose(grads[which], num, rtol=1e-6, atol=1e-7)


def test_compact_and_expand_are_inverse():
    X, Wg, Wu, Wd = _rand_layer(24, 5, 6, 21)
    _, M, G, U = O.moc_forward(X, Wg, Wu, Wd, 4)
    idx, gv, uv = O.compact_saved(M, G, U)
    assert np.all(np.diff(idx, axis=1) > 0)
    M2, GM, UM = O.expand_saved(idx, gv, uv, 21)
    np.testing.assert_array_equal(M2, M)
    np.testing.assert_array_equal(GM, G * M)
    np.testing.assert_array_equal(UM, U * M)
    np.testing.assert_array_equal(O.mask_from_idx(idx, 21), M)


# --------------------------------------------------------------- counts the paper prints
def test_memory_and_mac_counts():
    # Table 1: MoC+GCP stores 0.6 * b*s*d_ffn elements (besides D) when 20% of channels are kept
    s, F = 640, 1000
    assert O.stored_activation_elements(s, F, F // 5) == int(0.6 * s * F)
    # section "Accelerated inference": 3 d d_ffn dense vs d d_ffn + 2 K d for MoC
    assert O.decode_macs(4096, 11008, 1376) == (3 * 4096 * 11008, 4096 * 11008 + 2 * 1376 * 4096)


# ------------------------------------------------------------------ RMSNorm and the stack
def test_rmsnorm_against_torch_and_stack():
    rng = np.random.default_rng(30)
    x = rng.standard_normal((5, 16))
    gain = rng.standard_normal(16)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (16,), torch.from_numpy(gain), 1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, gain, 1e-5), ref, rtol=1e-12)
    # x = c * ones, gain = 1, eps = 0 -> sign(c)
    np.testing.assert_allclose(O.rmsnorm(np.full((1, 8), -3.0), np.ones(8), 0.0), -np.ones((1, 8)))
    layers = []
    for l in range(3):
        _, Wg, Wu, Wd = _rand_layer(40 + l, 1, 16, 40)
        layers.append((np.ones(16), Wg, Wu, Wd))
    h = O.prefill_stack(x, layers, 5, 1e-5)
    h_ref = x.copy()
    for gain_l, Wg, Wu, Wd in layers:
        xn = torch.nn.functional.rms_norm(torch.from_numpy(h_ref), (16,), None, 1e-5).numpy()
        Dd, _ = O.moc_decode(xn, Wg, Wu, Wd, 5)
        h_ref = h_ref + Dd
    np.testing.assert_allclose(h, h_ref, rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------- grouped Top-K (MoC_{a:b})
GOLDEN_GROUPED = os.path.join(os.path.dirname(__file__), "golden", "grouped_example.json")


def test_grouped_hand_example():
    g = json.load(open(GOLDEN_GROUPED))
    X, Wg, Wu, Wd = (np.array(g[k]) for k in ("X", "W_gate", "W_up", "W_down"))
    D, M, G, U = O.moc_forward_grouped(X, Wg, Wu, Wd, g["a"], g["b"])
    np.testing.assert_allclose(G, g["G"], rtol=0, atol=1e-15)
    assert [list(np.flatnonzero(r)) for r in M] == g["C"]
    np.testing.assert_allclose(D, g["D"], rtol=1e-14)
    # the row-wide Top-2 of the same gate is a different set
    assert [list(np.flatnonzero(r)) for r in O.topk_mask(G, 2)] == g["C_rowwide_top2"]
    dvec, C = O.moc_decode_grouped(X[0], Wg, Wu, Wd, g["a"], g["b"])
    np.testing.assert_allclose(dvec, g["D"][0], rtol=1e-14)
    assert C.tolist() == g["C"][0]


def test_grouped_mask_explicit_cases():
    # ties inside a group go to the lower channel; -0.0 equals +0.0; negative groups still give a
    row = np.array([[0.2, 0.2, -5.0, 0.2, -1.0, -3.0, -2.0, -4.0, 0.0, -0.0, -0.0, 0.0]])
    M = O.grouped_topk_mask(row, 2, 4)
    assert list(np.flatnonzero(M[0])) == [0, 1, 4, 6, 8, 9]
    M = O.grouped_topk_mask(row, 1, 4)
    assert list(np.flatnonzero(M[0])) == [0, 4, 8]
    M = O.grouped_topk_mask(row, 3, 4)
    assert list(np.flatnonzero(M[0])) == [0, 1, 3, 4, 5, 6, 8, 9, 10]
    with pytest.raises(ValueError):
        O.grouped_topk_mask(row, 2, 8)      # 8 does not divide 12
    with pytest.raises(ValueError):
        O.grouped_topk_mask(row, 5, 4)


def test_grouped_mask_properties_and_library_routines():
    rng = np.random.default_rng(77)
    G = rng.standard_normal((37, 96)).astype(np.float32)
    G[:, 5] = G[:, 3]                                    # planted ties inside a group
    for a, b in ((2, 8), (1, 8), (2, 4), (3, 16), (1, 2), (4, 4)):
        M = O.grouped_topk_mask(G, a, b)
        Mg = M.reshape(37, 96 // b, b)
        assert np.all(Mg.sum(axis=2) == a)
        Gg = G.reshape(37, 96 // b, b).astype(np.float64)
        if a < b:
            lo_sel = np.where(Mg, Gg, np.inf).min(axis=2)
            hi_unsel = np.where(~Mg, Gg, -np.inf).max(axis=2)
            assert np.all(lo_sel >= hi_unsel)
        # torch.topk on the reshaped row: same multiset of kept values in every group
        tv = torch.topk(torch.from_numpy(G).reshape(37, 96 // b, b), a, dim=2).values.numpy()
        kept = np.sort(np.where(Mg, Gg, -np.inf), axis=2)[:, :, b - a:]
        np.testing.assert_array_equal(np.sort(tv, axis=2), kept.astype(np.float32))
        # loop twin
        for i in (0, 17, 36):
            assert brute.select_grouped_full_sort([float(v) for v in G[i]], a, b) == list(np.flatnonzero(M[i]))
    # one group spanning the whole row is the row-wide Top-K
    np.testing.assert_array_equal(O.grouped_topk_mask(G, 11, 96), O.topk_mask(G, 11))
    # any 2:8 mask has at most two ones in every aligned group of four (the 2:4 pattern of the
    # structured-sparse matrix instructions)
    M28 = O.grouped_topk_mask(G, 2, 8)
    assert M28.reshape(37, 24, 4).sum(axis=2).max() <= 2


def test_grouped_forward_reductions_and_twin():
    X, Wg, Wu, Wd = _rand_layer(5, 6, 5, 16)
    # a = b keeps every channel: dense SwiGLU
    D_all, M_all, _, _ = O.moc_forward_grouped(X, Wg, Wu, Wd, 4, 4)
    assert M_all.all()
    np.testing.assert_allclose(D_all, O.swiglu_forward(X, Wg, Wu, Wd)[0], rtol=1e-13)
    # b = d_ffn is the row-wide layer
    D_row, M_row, _, _ = O.moc_forward(X, Wg, Wu, Wd, 5)
    D_g, M_g, _, _ = O.moc_forward_grouped(X, Wg, Wu, Wd, 5, 16)
    np.testing.assert_array_equal(M_row, M_g)
    np.testing.assert_array_equal(D_row, D_g)
    # loop twin and decode recipe on 2:8
    D28, M28, _, _ = O.moc_forward_grouped(X, Wg, Wu, Wd, 2, 8)
    D_loops, sets = brute.moc_forward_loops(X.tolist(), Wg.tolist(), Wu.tolist(), Wd.tolist(), None, group=(2, 8))
    assert sets == [list(np.flatnonzero(r)) for r in M28]
    np.testing.assert_allclose(D28, np.array(D_loops), rtol=1e-12, atol=1e-14)
    D_dec, C_dec = O.moc_decode_grouped(X, Wg, Wu, Wd, 2, 8)
    np.testing.assert_allclose(D_dec, D28, rtol=1e-12, atol=1e-14)
    assert C_dec.tolist() == sets
    # unselected channels contribute nothing
    Wu2, Wd2 = Wu.copy(), Wd.copy()
    never = ~M28.any(axis=0)
    Wu2[:, never] = 1e6
    Wd2[never, :] = -1e6
    np.testing.assert_array_equal(O.moc_forward_given_mask(X, Wg, Wu2, Wd2, M28)[0], D28)


# ------------------------------------------------- Top-K position variants (keyed selection)
def test_selection_key_hand_cases():
    # SiLU has its minimum at x = -1.2785 (value -0.2785): below it the order reverses.
    g = np.array([[-6.0, -1.3, -0.5, 0.05, 0.3, -3.0]])
    s = g / (1 + np.exp(-g))                     # [-0.0148, -0.2784, -0.1888, 0.0256, 0.1723, -0.1423]
    assert list(np.flatnonzero(O.topk_mask_keyed(g, 3, "gate")[0])) == [2, 3, 4]
    assert list(np.flatnonzero(O.topk_mask_keyed(g, 3, "silu")[0])) == [0, 3, 4]          # -6 beats -0.5 after SiLU
    assert list(np.flatnonzero(O.topk_mask_keyed(g, 3, "abs_silu")[0])) == [1, 2, 4]      # largest |SiLU|
    np.testing.assert_allclose(O.selection_key(g, "silu")[0], s[0].astype(np.float32), rtol=1e-6)
    np.testing.assert_allclose(O.selection_key(g, "abs_silu")[0], np.abs(s[0]).astype(np.float32), rtol=1e-6)
    with pytest.raises(ValueError):
        O.selection_key(g, "nonsense")


def test_keyed_masks_against_library_routines_and_monotonicity():
    rng = np.random.default_rng(31)
    G = (rng.standard_normal((23, 300)) * 1.5).astype(np.float32)
    for key in ("silu", "abs_silu"):
        for K in (1, 17, 150, 299):
            M = O.topk_mask_keyed(G, K, key)
            assert np.all(M.sum(axis=1) == K)
            st = torch.nn.functional.silu(torch.from_numpy(G).double())
            if key == "abs_silu":
                st = st.abs()
            tv = torch.topk(st.float(), K, dim=1).values.numpy()
            kept = np.sort(np.where(M, st.float().numpy(), -np.inf), axis=1)[:, 300 - K:]
            np.testing.assert_array_equal(np.sort(tv, axis=1), kept)
    # while the K-th largest gate value is above SiLU's minimiser, "silu" selects what "gate" selects
    for K in (5, 40, 100):
        kth = np.sort(G, axis=1)[:, 300 - K]
        rows = kth > -1.0
        assert rows.any()
        np.testing.assert_array_equal(O.topk_mask_keyed(G, K, "silu")[rows], O.topk_mask(G, K)[rows])
    # forward through the keyed mask: same as the given-mask forward
    X, Wg, Wu, Wd = _rand_layer(8, 7, 6, 24)
    D, M, Gm, U = O.moc_forward_keyed(X, Wg, Wu, Wd, 9, "abs_silu")
    np.testing.assert_array_equal(D, O.moc_forward_given_mask(X, Wg, Wu, Wd, M)[0])
    np.testing.assert_array_equal(M, O.topk_mask_keyed(Gm, 9, "abs_silu"))
    np.testing.assert_array_equal(O.moc_forward_keyed(X, Wg, Wu, Wd, 9, "gate")[0], O.moc_forward(X, Wg, Wu, Wd, 9)[0])


# ------------------------------------------------------------- MoC inside MoE experts
def _rand_experts(seed, E, d, F, scale=0.3):
    rng = np.random.default_rng(seed)
    return ([rng.standard_normal((d, F)) * scale for _ in range(E)], [rng.standard_normal((d, F)) * scale for _ in range(E)],
            [rng.standard_normal((F, d)) * scale for _ in range(E)])


def test_experts_reduce_to_the_plain_layer_and_to_single_rows():
    rng = np.random.default_rng(50)
    E, d, F, K = 3, 5, 12, 4
    Wg, Wu, Wd = _rand_experts(51, E, d, F)
    X = rng.standard_normal((11, d))
    offsets = [0, 4, 4, 11]                                 # the second expert gets no rows
    D, M, G, U = O.moc_forward_experts(X, offsets, Wg, Wu, Wd, K)
    # one expert holding every row is the plain layer
    D1, M1, _, _ = O.moc_forward_experts(X, [0, 11], Wg[:1], Wu[:1], Wd[:1], K)
    D0, M0, _, _ = O.moc_forward(X, Wg[0], Wu[0], Wd[0], K)
    np.testing.assert_array_equal(D1, D0)
    np.testing.assert_array_equal(M1, M0)
    # every row is what the decode recipe gives for that row with its expert's weights
    for t in range(11):
        e = 0 if t < 4 else 2
        dvec, C = O.moc_decode(X[t], Wg[e], Wu[e], Wd[e], K)
        np.testing.assert_allclose(D[t], dvec, rtol=1e-12, atol=1e-14)
        assert list(np.flatnonzero(M[t])) == C.tolist()
    with pytest.raises(ValueError):
        O.moc_forward_experts(X, [0, 5, 3, 11], Wg, Wu, Wd, K)


def test_experts_dense_limit_is_a_mixtral_style_layer_in_torch():
    # K = d_ffn, top-2 of 4 experts, softmax weights over the two: written independently with torch ops
    rng = np.random.default_rng(52)
    E, d, F, T = 4, 6, 10, 9
    Wg, Wu, Wd = _rand_experts(53, E, d, F)
    Xtok = rng.standard_normal((T, d))
    router = rng.standard_normal((d, E))
    logits = torch.tensor(Xtok @ router)
    top = torch.topk(logits, 2, dim=1)
    wts = torch.softmax(top.values, dim=1).numpy()
    experts = top.indices.numpy()
    # torch reference: dense SwiGLU experts, weighted sum
    ref = np.zeros((T, d))
    for t in range(T):
        for s in range(2):
            e = experts[t, s]
            xt = torch.tensor(Xtok[t])
            h = torch.nn.functional.silu(xt @ torch.tensor(Wg[e])) * (xt @ torch.tensor(Wu[e]))
            ref[t] += wts[t, s] * (h @ torch.tensor(Wd[e])).numpy()
    # oracle path: sort the 2T routed copies by expert, run the expert form, combine
    pairs = sorted((int(experts[t, s]), t, s) for t in range(T) for s in range(2))
    offsets = [0] + [sum(1 for p in pairs if p[0] <= e) for e in range(E)]
    Xs = np.stack([Xtok[t] for _, t, _ in pairs])
    D, M, _, _ = O.moc_forward_experts(Xs, offsets, Wg, Wu, Wd, F)
    assert M.all()
    got = np.zeros((T, d))
    for row, (_, t, s) in enumerate(pairs):
        got[t] += wts[t, s] * D[row]
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_experts_backward_finite_differences():
    rng = np.random.default_rng(54)
    E, d, F, K = 2, 4, 8, 3
    Wg, Wu, Wd = _rand_experts(55, E, d, F, scale=0.7)
    X = rng.standard_normal((6, d))
    offsets = [0, 2, 6]
    dD = rng.standard_normal((6, d))
    D, M, G, U = O.moc_forward_experts(X, offsets, Wg, Wu, Wd, K)
    dX, dWg, dWu, dWd = O.moc_backward_experts(X, offsets, Wg, Wu, Wd, M, G * M, U * M, dD)

    def loss(Xv, Wgv, Wuv, Wdv):
        out = np.zeros_like(D)
        for e in range(E):
            lo, hi = offsets[e], offsets[e + 1]
            out[lo:hi] = O.moc_forward_given_mask(Xv[lo:hi], Wgv[e], Wuv[e], Wdv[e], M[lo:hi])[0]
        return float((out * dD).sum())

    h = 1e-6
    for (t, c) in ((0, 1), (3, 2), (5, 0)):
        Xp, Xm = X.copy(), X.copy()
        Xp[t, c] += h
        Xm[t, c] -= h
        assert abs((loss(Xp, Wg, Wu, Wd) - loss(Xm, Wg, Wu, Wd)) / (2 * h) - dX[t, c]) < 1e-6
    for e, (r, c) in ((0, (1, 5)), (1, (3, 2))):
        for which, grad in ((0, dWg), (1, dWu)):
            Wp = [w.copy() for w in (Wg if which == 0 else Wu)]
            Wm = [w.copy() for w in (Wg if which == 0 else Wu)]
            Wp[e][r, c] += h
            Wm[e][r, c] -= h
            lp = loss(X, Wp, Wu, Wd) if which == 0 else loss(X, Wg, Wp, Wd)
            lm = loss(X, Wm, Wu, Wd) if which == 0 else loss(X, Wg, Wm, Wd)
            assert abs((lp - lm) / (2 * h) - grad[e][r, c]) < 1e-6
        Wp = [w.copy() for w in Wd]
        Wm = [w.copy() for w in Wd]
        Wp[e][c, r] += h
        Wm[e][c, r] -= h
        assert abs((loss(X, Wg, Wu, Wp) - loss(X, Wg, Wu, Wm)) / (2 * h) - dWd[e][c, r]) < 1e-6
    # an expert without rows has zero weight gradients
    _, M1, G1, U1 = O.moc_forward_experts(X, [0, 6, 6], Wg, Wu, Wd, K)
    _, g0, _, d0 = O.moc_backward_experts(X, [0, 6, 6], Wg, Wu, Wd, M1, G1 * M1, U1 * M1, dD)
    assert not g0[1].any() and not d0[1].any()
