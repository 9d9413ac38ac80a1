"""Helpers shared by the GPU parity tests: moving seeded inputs to the device, calling the CPU
oracle in the paper's layout, and the comparison rules (max-norm relative error; index sets
bit-exact except inside the near-tie window of the fp32 gate)."""
import numpy as np
import torch

from oracle import moc_oracle as O

TOL = {"f32": 1e-4, "bf16": 2e-2}
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
TIE_WINDOW = 1e-6


def to_dev(a, dtype):
    """float32 numpy array (bf16-exact when dtype is bf16) -> GPU tensor of that dtype, exactly."""
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(TORCH_DTYPE[dtype]).contiguous()


def to_np(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def paper_weights(L):
    """Channel-major [F, d] arrays -> the paper's W_gate [d,F], W_up [d,F], W_down [F,d] in float64."""
    return (L["wg"].astype(np.float64).T, L["wu"].astype(np.float64).T, L["wd"].astype(np.float64))


def maxrel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.max(np.abs(b))
    return float(np.max(np.abs(a - b)) / (den if den > 0 else 1.0))


def frobrel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (den if den > 0 else 1.0))


def assert_close(name, got, want, tol):
    """The bar is the max-norm relative error per tensor; the relative Frobenius error is printed
    beside it as information."""
    err = maxrel(got, want)
    print("[parity] %-18s max-norm rel %.3e (tol %.1e)  Frobenius rel %.3e" % (name, err, tol, frobrel(got, want)), flush=True)
    assert err <= tol, "%s: max-norm relative error %.3e > %.1e" % (name, err, tol)
    return err


def check_index_sets(idx_gpu, G64, K):
    """idx_gpu [T,K] int; G64 the oracle's float64 gate [T,F].  Every row must be strictly
    ascending, in range, and equal to the oracle's set -- unless the row's K-th / (K+1)-th fp32 gate
    values are within the 1e-6 relative window, in which case any set that keeps everything
    clearly above the threshold and nothing clearly below it is accepted.  Returns the rows that
    needed the window."""
    idx_gpu = np.asarray(idx_gpu)
    T, F = G64.shape
    assert idx_gpu.shape == (T, K)
    assert np.all(idx_gpu >= 0) and np.all(idx_gpu < F)
    if K > 1:
        assert np.all(np.diff(idx_gpu, axis=1) > 0), "idx rows must ascend strictly"
    M_ref = O.topk_mask(G64, K)
    M_gpu = O.mask_from_idx(idx_gpu, F)
    differing = np.flatnonzero((M_ref != M_gpu).any(axis=1))
    g32 = G64.astype(np.float32)
    for t in differing:
        row = g32[t].astype(np.float64)
        tau = np.sort(row)[F - K]
        tol = TIE_WINDOW * max(abs(tau), 1e-30)
        must = row > tau + tol
        never = row < tau - tol
        assert np.all(M_gpu[t][must]), "row %d drops a channel clearly above the threshold" % t
        assert not np.any(M_gpu[t][never]), "row %d keeps a channel clearly below the threshold" % t
    return differing


def oracle_forward_for(L, idx_gpu):
    """Oracle outputs for the GPU's own index sets: (D, gvals, uvals, G) in float64."""
    Wg, Wu, Wd = paper_weights(L)
    X = L["x"].astype(np.float64)
    F = Wg.shape[1]
    M = O.mask_from_idx(np.asarray(idx_gpu), F)
    D, G, U = O.moc_forward_given_mask(X, Wg, Wu, Wd, M)
    rows = np.arange(X.shape[0])[:, None]
    return D, G[rows, idx_gpu], U[rows, idx_gpu], G


def oracle_backward_for(L, idx, gvals, uvals):
    """Oracle gradients from the stored set exactly as the GPU stored it; weight gradients are
    returned channel-major [F, d] like the library's."""
    Wg, Wu, Wd = paper_weights(L)
    X = L["x"].astype(np.float64)
    F = Wg.shape[1]
    M, GM, UM = O.expand_saved(idx, gvals, uvals, F)
    dX, dWg, dWu, dWd = O.moc_backward(X, Wg, Wu, Wd, M, GM, UM, L["dy"].astype(np.float64))
    return dX, dWg.T, dWu.T, dWd


def check_grouped_index_sets(idx_gpu, G64, a, b):
    """The grouped counterpart of check_index_sets for MoC_{a:b}: every row ascends, every group of
    b channels holds exactly a kept channels, and a group's kept set equals the oracle's unless the
    group's a-th / (a+1)-th fp32 gate values are within the 1e-6 window, where any set that keeps
    everything clearly above and nothing clearly below is accepted.  A group's threshold can lie
    arbitrarily close to zero (the row-wide one never does), while the rounding error of an fp32
    dot product scales with its terms, not with its possibly cancelling sum; the window is
    therefore 1e-6 relative to the larger of |threshold| and the row's RMS gate value.  Returns
    the rows in which some group needed the window."""
    idx_gpu = np.asarray(idx_gpu)
    T, F = G64.shape
    K = F // b * a
    assert idx_gpu.shape == (T, K)
    assert np.all(idx_gpu >= 0) and np.all(idx_gpu < F)
    if K > 1:
        assert np.all(np.diff(idx_gpu, axis=1) > 0), "idx rows must ascend strictly"
    M_gpu = O.mask_from_idx(idx_gpu, F)
    assert np.all(M_gpu.reshape(T, F // b, b).sum(axis=2) == a), "every group must keep exactly a channels"
    M_ref = O.grouped_topk_mask(G64, a, b)
    differing = np.flatnonzero((M_ref != M_gpu).any(axis=1))
    g32 = G64.astype(np.float32)
    for t in differing:
        rms = float(np.sqrt(np.mean(g32[t].astype(np.float64) ** 2)))
        for q in np.flatnonzero((M_ref[t] != M_gpu[t]).reshape(F // b, b).any(axis=1)):
            grp = g32[t, q * b:(q + 1) * b].astype(np.float64)
            tau = np.sort(grp)[b - a]
            tol = TIE_WINDOW * max(abs(tau), rms, 1e-30)
            kept = M_gpu[t, q * b:(q + 1) * b]
            assert np.all(kept[grp > tau + tol]), "row %d group %d drops a channel clearly above the threshold" % (t, q)
            assert not np.any(kept[grp < tau - tol]), "row %d group %d keeps a channel clearly below it" % (t, q)
    return differing


def check_keyed_index_sets(idx_gpu, G64, K, key):
    """check_index_sets for the Top-K position variants: the ranking, the threshold and the near-tie
    window (1e-6 relative to the larger of |threshold| and the row's RMS key, because SiLU outputs of
    negative gates cluster near zero) are those of the oracle's float32 selection key."""
    idx_gpu = np.asarray(idx_gpu)
    T, F = G64.shape
    assert idx_gpu.shape == (T, K)
    assert np.all(idx_gpu >= 0) and np.all(idx_gpu < F)
    if K > 1:
        assert np.all(np.diff(idx_gpu, axis=1) > 0), "idx rows must ascend strictly"
    keys = O.selection_key(G64, key).astype(np.float64)
    M_ref = O.topk_mask_keyed(G64, K, key)
    M_gpu = O.mask_from_idx(idx_gpu, F)
    differing = np.flatnonzero((M_ref != M_gpu).any(axis=1))
    for t in differing:
        row = keys[t]
        tau = np.sort(row)[F - K]
        tol = TIE_WINDOW * max(abs(tau), float(np.sqrt(np.mean(row ** 2))), 1e-30)
        assert np.all(M_gpu[t][row > tau + tol]), "row %d drops a channel clearly above the threshold" % t
        assert not np.any(M_gpu[t][row < tau - tol]), "row %d keeps a channel clearly below the threshold" % t
    return differing
