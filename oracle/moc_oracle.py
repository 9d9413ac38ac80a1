"""CPU oracle for the Mixture-of-Channels (MoC) feed-forward layer.  TEST INFRASTRUCTURE ONLY.

Plain numpy, float64, written from the paper's equations in the paper's notation:
X is [s, d], W_gate and W_up are [d, d_ffn], W_down is [d_ffn, d].  Nothing here is
blocked, fused or reordered, and nothing is shared with the HIP kernels.  Only tests,
the smoke check and the benchmark's cpu_baseline leg may import this module; the
product never does.

What each function follows:
  silu, silu_grad          Section "SiLU activation pattern", Eq. (3); the derivative is the
                           textbook one of that formula (the paper names the operator only).
  swiglu_forward/backward  Section "Activation memory profiling", Eqs. (FFN-1), (FFN-2).
  topk_mask                Section "Mixture-of-Channels architecture": M = TopK(G), row-wise,
                           largest signed values, exactly K ones per row.
  grouped_topk_mask        The grouped Top-K of MoC_{a:b} (item "MoC with structured 2:8 sparsity" and
                           the definition before Theorem 1): a entries are kept in every contiguous
                           group of b entries of a row; b divides d_ffn.
  moc_forward_grouped, moc_decode_grouped   the same layer and recipe with that mask.
  moc_forward_experts, moc_backward_experts   Section "Compatibility with MoE architectures": the
                           MoC network as the MLP of every expert, on rows already routed.
  selection_key, topk_mask_keyed, moc_forward_keyed   the Top-K position variants of the ablation
                           ("After SiLU") and of the proof of Theorem 1 (|SiLU|).
  moc_forward*             Eqs. (MoC-1), (MoC-2).
  moc_backward             Section "Activation-efficient pre-training", Eqs. (bp-1)...(bp-5),
                           with S' and Z' recomputed from the stored G.M and U.M (MoC + GCP).
  moc_decode               Section "Accelerated inference", the four-step per-token recipe.
  rmsnorm, residual_add    Section "Activation memory profiling", RMSNorm and residual items.

Readings where the paper is silent (also listed in the design notes):
  * ties at the K-th value: the lower channel index wins; -0.0 and +0.0 are equal;
  * the selection is decided on the gate rounded to float32 (the precision the HIP path
    selects in), everything else stays float64;
  * compact form of the stored set: idx ascending by channel, gvals = G at idx, uvals = U at idx.

Pins (tests/test_oracle_*.py): a hand-worked example from Eq. (3) and (MoC-2), brute-force
full-sort selection, numpy/torch library selection routines, dense SwiGLU through torch's own
silu at K = d_ffn, torch.autograd and central finite differences for the backward, torch's
rms_norm, and the invariants (unselected channels contribute nothing, token independence,
channel-permutation equivariance, decode == training forward); for the grouped mask: a hand example,
the loop twin, b = d_ffn reducing to topk_mask, a = b reducing to dense SwiGLU, torch.topk on the
reshaped row, exactly a per group, the 2:4 compatibility of 2:8 masks; for the keyed masks: monotonicity of
SiLU above its minimum (same set as the raw gate when the threshold is positive), hand cases below it, torch.topk on
torch's own silu; for the expert form: one expert equals the plain layer, a dense Mixtral-style layer written with
torch ops at K = d_ffn, row-wise single-token evaluation, finite differences.  No function here is unpinned.
"""
import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------- Eq. (3)
def silu(x):
    x = _f64(x)
    with np.errstate(over="ignore"):
        return x / (1.0 + np.exp(-x))


def sigmoid(x):
    x = _f64(x)
    with np.errstate(over="ignore"):
        return 1.0 / (1.0 + np.exp(-x))


def silu_grad(x):
    """d/dx [x * sigmoid(x)] = sigmoid(x) * (1 + x * (1 - sigmoid(x)))."""
    x = _f64(x)
    sg = sigmoid(x)
    return sg * (1.0 + x * (1.0 - sg))


# ------------------------------------------------------------------ Eqs. (FFN-1), (FFN-2)
def swiglu_forward(X, W_gate, W_up, W_down):
    X, W_gate, W_up, W_down = map(_f64, (X, W_gate, W_up, W_down))
    G = X @ W_gate
    U = X @ W_up
    S = silu(G)
    Z = S * U
    D = Z @ W_down
    return D, G, U


def swiglu_backward(X, W_gate, W_up, W_down, G, U, dD):
    """Gradients of the dense FFN given its stored G and U (Eqs. (bp-1)...(bp-5) with M = 1)."""
    ones = np.ones(np.shape(G), dtype=bool)
    return moc_backward(X, W_gate, W_up, W_down, ones, G, U, dD)


# ------------------------------------------------------------------------ M = TopK(G)
def topk_mask(G, K, select_dtype=np.float32):
    """Boolean mask with exactly K ones per row marking the K largest signed entries.

    The decision is taken on G cast to `select_dtype`.  Equal values are ordered by
    channel index, lower first (stable sort on the negated row).
    """
    G = np.asarray(G)
    s, F = G.shape
    if not (1 <= K <= F):
        raise ValueError("K must satisfy 1 <= K <= d_ffn")
    if not np.all(np.isfinite(G)):
        raise ValueError("non-finite gate values")
    key = G.astype(select_dtype)
    M = np.zeros((s, F), dtype=bool)
    for i in range(s):
        order = np.argsort(-key[i], kind="stable")
        M[i, order[:K]] = True
    return M


def selection_key(G, key="gate", select_dtype=np.float32):
    """What the Top-K ranks.  "gate": the raw signed SiLU input (the paper's choice, section
    "Mixture-of-Channels architecture"); "silu": the SiLU output, signed (ablation "Effect of top-K's
    position", row "After SiLU"); "abs_silu": its absolute value (the selection used in the proof of
    Theorem 1, see the remark after it).  The gate is first rounded to `select_dtype`, the precision
    the selection is decided in, and so is the transformed key."""
    g = np.asarray(G).astype(select_dtype)
    if key == "gate":
        return g
    s = silu(g.astype(F64))
    if key == "silu":
        return s.astype(select_dtype)
    if key == "abs_silu":
        return np.abs(s).astype(select_dtype)
    raise ValueError("unknown selection key %r" % (key,))


def topk_mask_keyed(G, K, key="gate"):
    """topk_mask on selection_key(G, key): exactly K ones per row, ties to the lower channel."""
    return topk_mask(selection_key(G, key), K)


def moc_forward_keyed(X, W_gate, W_up, W_down, K, key):
    """Eqs. (MoC-1), (MoC-2) with the mask taken on selection_key(G, key) instead of on G."""
    G = _f64(X) @ _f64(W_gate)
    M = topk_mask_keyed(G, K, key)
    D, G, U = moc_forward_given_mask(X, W_gate, W_up, W_down, M)
    return D, M, G, U


def grouped_topk_mask(G, a, b, select_dtype=np.float32):
    """Mask of MoC_{a:b}: in every contiguous group of b channels (channels q*b ... q*b + b - 1) the
    a largest signed entries are marked, so each row holds a * d_ffn / b ones.  Same precision and
    tie rule as topk_mask (float32 decision, lower channel first among equal values)."""
    G = np.asarray(G)
    s, F = G.shape
    if b < 1 or F % b != 0:
        raise ValueError("b must divide d_ffn")
    if not (1 <= a <= b):
        raise ValueError("a must satisfy 1 <= a <= b")
    if not np.all(np.isfinite(G)):
        raise ValueError("non-finite gate values")
    key = G.astype(select_dtype)
    M = np.zeros((s, F), dtype=bool)
    for i in range(s):
        for q in range(F // b):
            group = key[i, q * b:(q + 1) * b]
            order = np.argsort(-group, kind="stable")
            M[i, q * b + order[:a]] = True
    return M


# ------------------------------------------------------------- Eqs. (MoC-1), (MoC-2)
def moc_forward_given_mask(X, W_gate, W_up, W_down, M):
    X, W_gate, W_up, W_down = map(_f64, (X, W_gate, W_up, W_down))
    G = X @ W_gate
    U = X @ W_up
    S = silu(G)
    S_prime = S * M
    Z_prime = S_prime * U
    D = Z_prime @ W_down
    return D, G, U


def moc_forward(X, W_gate, W_up, W_down, K):
    G = _f64(X) @ _f64(W_gate)
    M = topk_mask(G, K)
    D, G, U = moc_forward_given_mask(X, W_gate, W_up, W_down, M)
    return D, M, G, U


def moc_forward_grouped(X, W_gate, W_up, W_down, a, b):
    """MoC_{a:b}: Eqs. (MoC-1), (MoC-2) with the grouped mask in place of the row-wide Top-K."""
    G = _f64(X) @ _f64(W_gate)
    M = grouped_topk_mask(G, a, b)
    D, G, U = moc_forward_given_mask(X, W_gate, W_up, W_down, M)
    return D, M, G, U


# ------------------------------------------------ compact stored set (Table 1, MoC+GCP)
def compact_saved(M, G, U):
    """(idx, gvals, uvals), each [s, K]: the ones of M in ascending channel order, G and U there."""
    s, F = M.shape
    K = int(M[0].sum())
    idx = np.empty((s, K), dtype=np.int32)
    for i in range(s):
        cols = np.flatnonzero(M[i])
        if cols.size != K:
            raise ValueError("mask rows must all hold K ones")
        idx[i] = cols
    rows = np.arange(s)[:, None]
    return idx, _f64(G)[rows, idx], _f64(U)[rows, idx]


def expand_saved(idx, gvals, uvals, F):
    """Inverse of compact_saved: M, G.M and U.M as dense [s, d_ffn] arrays."""
    idx = np.asarray(idx)
    s, K = idx.shape
    rows = np.arange(s)[:, None]
    M = np.zeros((s, F), dtype=bool)
    M[rows, idx] = True
    GM = np.zeros((s, F), dtype=F64)
    UM = np.zeros((s, F), dtype=F64)
    GM[rows, idx] = _f64(gvals)
    UM[rows, idx] = _f64(uvals)
    return M, GM, UM


def mask_from_idx(idx, F):
    idx = np.asarray(idx)
    M = np.zeros((idx.shape[0], F), dtype=bool)
    M[np.arange(idx.shape[0])[:, None], idx] = True
    return M


# ------------------------------------------------------------ Eqs. (bp-1) ... (bp-5)
def moc_backward(X, W_gate, W_up, W_down, M, GM, UM, dD):
    """Backward of the MoC layer from the stored set {M, G.M, U.M} and the upstream gradient.

    S' and Z' are recomputed from G.M (gradient checkpointing of the two element-wise steps).
    Returns (dX, dW_gate, dW_up, dW_down) in the paper's shapes.
    """
    X, W_gate, W_up, W_down, GM, UM, dD = map(_f64, (X, W_gate, W_up, W_down, GM, UM, dD))
    M = np.asarray(M, dtype=bool)
    S_prime = silu(GM) * M                      # S' = SiLU(G) . M
    Z_prime = S_prime * UM                      # Z' = S' . U
    dW_down = Z_prime.T @ dD                    # (bp-1)
    dZ_prime = dD @ W_down.T                    # (bp-1)
    dS_prime = (UM * M) * dZ_prime              # (bp-2)
    dU = S_prime * dZ_prime                     # (bp-2)
    dS = dS_prime                               # (bp-3)
    dG = dS * silu_grad(GM)                     # (bp-3)
    dW_gate = X.T @ dG                          # (bp-4)
    dW_up = X.T @ dU                            # (bp-4)
    dX = dG @ W_gate.T + dU @ W_up.T            # (bp-5)
    return dX, dW_gate, dW_up, dW_down


# -------------------------------------------------- inference recipe, one token at a time
def moc_decode(x, W_gate, W_up, W_down, K):
    """Per-token recipe: g = x W_gate, Top-K set C, z'_j = SiLU(g_j) (x . W_up[:, j]) for j in C,
    d = sum_{j in C} z'_j w_j with w_j the j-th row of W_down.  Only the K selected columns of
    W_up and rows of W_down are touched.  x may be [d] or [B, d]; tokens are independent."""
    x = _f64(x)
    single = x.ndim == 1
    xs = x[None, :] if single else x
    W_gate, W_up, W_down = map(_f64, (W_gate, W_up, W_down))
    B, d = xs.shape
    out = np.zeros((B, d), dtype=F64)
    sets = np.empty((B, K), dtype=np.int32)
    for b in range(B):
        g = xs[b] @ W_gate
        C = np.flatnonzero(topk_mask(g[None, :], K)[0])
        u_C = xs[b] @ W_up[:, C]
        z_C = silu(g[C]) * u_C
        acc = np.zeros(d, dtype=F64)
        for zj, j in zip(z_C, C):
            acc += zj * W_down[j]
        out[b] = acc
        sets[b] = C
    return (out[0], sets[0]) if single else (out, sets)


def moc_decode_grouped(x, W_gate, W_up, W_down, a, b):
    """The per-token recipe of moc_decode with the set C chosen group by group (MoC_{a:b})."""
    x = _f64(x)
    single = x.ndim == 1
    xs = x[None, :] if single else x
    W_gate, W_up, W_down = map(_f64, (W_gate, W_up, W_down))
    B, d = xs.shape
    K = W_gate.shape[1] // b * a
    out = np.zeros((B, d), dtype=F64)
    sets = np.empty((B, K), dtype=np.int32)
    for t in range(B):
        g = xs[t] @ W_gate
        C = np.flatnonzero(grouped_topk_mask(g[None, :], a, b)[0])
        acc = np.zeros(d, dtype=F64)
        for j in C:
            u_j = xs[t] @ W_up[:, j]
            acc += silu(g[j]) * u_j * W_down[j]
        out[t] = acc
        sets[t] = C
    return (out[0], sets[0]) if single else (out, sets)


def decode_macs(d, d_ffn, K):
    """Multiply-accumulates per token: dense FFN and MoC (section "Accelerated inference")."""
    return 3 * d * d_ffn, d * d_ffn + 2 * K * d


def stored_activation_elements(s, d_ffn, K):
    """Elements of the MoC+GCP stored set besides D: M, G.M and U.M kept compactly (Table 1)."""
    return 3 * s * K


# ------------------------------------------------ MoC inside the experts of an MoE layer
def moc_forward_experts(X, offsets, W_gate, W_up, W_down, K):
    """Section "Compatibility with MoE architectures": every expert's MLP is a MoC feed-forward
    network with its own weights.  X [A, d] holds the routed token copies sorted by expert; rows
    offsets[e] .. offsets[e+1]-1 belong to expert e; W_* are lists (or stacked arrays) with one
    matrix per expert in the paper's shapes.  Routing and the weighted combination of the experts'
    outputs are the surrounding MoE layer's and not part of this function.
    Returns (D, M, G, U) for all rows, in the order of X."""
    X = _f64(X)
    offsets = [int(o) for o in offsets]
    if offsets[0] != 0 or offsets[-1] != X.shape[0] or any(b < a for a, b in zip(offsets, offsets[1:])):
        raise ValueError("offsets must ascend from 0 to the number of rows")
    F = np.asarray(W_gate[0]).shape[1]
    D = np.zeros((X.shape[0], np.asarray(W_down[0]).shape[1]), dtype=F64)
    M = np.zeros((X.shape[0], F), dtype=bool)
    G = np.zeros((X.shape[0], F), dtype=F64)
    U = np.zeros((X.shape[0], F), dtype=F64)
    for e in range(len(offsets) - 1):
        lo, hi = offsets[e], offsets[e + 1]
        if hi > lo:
            D[lo:hi], M[lo:hi], G[lo:hi], U[lo:hi] = moc_forward(X[lo:hi], W_gate[e], W_up[e], W_down[e], K)
    return D, M, G, U


def moc_backward_experts(X, offsets, W_gate, W_up, W_down, M, GM, UM, dD):
    """Backward of moc_forward_experts: Eqs. (bp-1)...(bp-5) expert by expert.  Returns dX [A, d] and
    per-expert lists dW_gate, dW_up, dW_down (zero for an expert without rows)."""
    X, dD = _f64(X), _f64(dD)
    offsets = [int(o) for o in offsets]
    dX = np.zeros_like(X)
    dWg, dWu, dWd = [], [], []
    for e in range(len(offsets) - 1):
        lo, hi = offsets[e], offsets[e + 1]
        Wg, Wu, Wd = _f64(W_gate[e]), _f64(W_up[e]), _f64(W_down[e])
        if hi > lo:
            dx, dg, du, dd = moc_backward(X[lo:hi], Wg, Wu, Wd, M[lo:hi], GM[lo:hi], UM[lo:hi], dD[lo:hi])
            dX[lo:hi] = dx
        else:
            dg, du, dd = np.zeros_like(Wg), np.zeros_like(Wu), np.zeros_like(Wd)
        dWg.append(dg)
        dWu.append(du)
        dWd.append(dd)
    return dX, dWg, dWu, dWd


# ----------------------------------------------------------- RMSNorm, residual, the stack
def rmsnorm(x, gain, eps):
    x = _f64(x)
    rms = np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x / rms * _f64(gain)


def residual_add(x, y):
    return _f64(x) + _f64(y)


def prefill_stack(h, layers, K, eps):
    """h <- h + MoC_l(RMSNorm(h)) for every layer; layers = [(gain, W_gate, W_up, W_down), ...]."""
    h = _f64(h)
    for gain, W_gate, W_up, W_down in layers:
        xn = rmsnorm(h, gain, eps)
        D, _, _, _ = moc_forward(xn, W_gate, W_up, W_down, K)
        h = residual_add(h, D)
    return h
