"""Pure-Python loop twin of the MoC layer for tiny shapes.  TEST INFRASTRUCTURE ONLY.

Scalar loops over tokens and channels, Python floats (float64), no numpy arithmetic: a second,
independent writing of Eqs. (MoC-1), (MoC-2) and of the per-token inference recipe, used to
pin oracle/moc_oracle.py.  Selection is a full descending sort of each gate row with the lower
channel index first among equal values.
"""
import math
import struct


def _f32(v):
    return struct.unpack("f", struct.pack("f", v))[0]


def silu_scalar(v):
    return v / (1.0 + math.exp(-v))


def select_full_sort(row, K):
    """Channels of the K largest signed values (compared after rounding to float32)."""
    order = sorted(range(len(row)), key=lambda j: (-_f32(row[j]), j))
    return sorted(order[:K])


def select_grouped_full_sort(row, a, b):
    """MoC_{a:b}: the a largest of every b consecutive channels, decided like select_full_sort."""
    chosen = []
    for first in range(0, len(row), b):
        members = list(range(first, first + b))
        members.sort(key=lambda j: (-_f32(row[j]), j))
        chosen.extend(members[:a])
    return sorted(chosen)


def moc_forward_loops(X, W_gate, W_up, W_down, K, group=None):
    """X[s][d], W_gate[d][F], W_up[d][F], W_down[F][d] as nested lists -> (D, sets).
    group = (a, b) switches to the grouped selection of MoC_{a:b} (K is then ignored)."""
    s, d, F = len(X), len(X[0]), len(W_gate[0])
    D, sets = [], []
    for i in range(s):
        g = [sum(X[i][k] * W_gate[k][j] for k in range(d)) for j in range(F)]
        C = select_full_sort(g, K) if group is None else select_grouped_full_sort(g, group[0], group[1])
        out = [0.0] * d
        for j in C:
            u = sum(X[i][k] * W_up[k][j] for k in range(d))
            z = silu_scalar(g[j]) * u
            for c in range(d):
                out[c] += z * W_down[j][c]
        D.append(out)
        sets.append(C)
    return D, sets
