"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's callers.

Only data generation lives here: normal draws from numpy's PCG64 generator and a
round-to-nearest-even cast to bfloat16 precision.  Nothing of the MoC method is
computed in this module, so both the HIP path and the oracle can be fed from it.

Recipe: x ~ N(0,1), every weight ~ N(0, 0.02^2), upstream gradient dy ~ N(0,1);
seed = 10000*cfg + 100*layer + tensor_id with tensor_id x=0, W_gate=1, W_up=2,
W_down=3, dy=4.  Weights are produced channel-major, shape [F, d]: row j is column j
of the paper's W_gate / W_up and row j of its W_down.
"""
import numpy as np

TENSOR_ID = {"x": 0, "wg": 1, "wu": 2, "wd": 3, "dy": 4}
WEIGHT_STD = 0.02


def seed_for(cfg_index, layer, tensor):
    return 10_000 * int(cfg_index) + 100 * int(layer) + TENSOR_ID[tensor]


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(a):
    """uint16 bit patterns of values that are already exactly representable in bfloat16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def normal(shape, seed, std=1.0, dtype="f32"):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if dtype == "bf16":
        a = round_to_bf16(a)
    return a


def make_layer(cfg_index, T, d, F, dtype="f32", layer=0, with_dy=False, x_seed_offset=0):
    """One layer's tensors as float32 arrays (bf16-exact values when dtype == 'bf16')."""
    out = {
        "x": normal((T, d), seed_for(cfg_index, layer, "x") + 10 * x_seed_offset, 1.0, dtype),
        "wg": normal((F, d), seed_for(cfg_index, layer, "wg"), WEIGHT_STD, dtype),
        "wu": normal((F, d), seed_for(cfg_index, layer, "wu"), WEIGHT_STD, dtype),
        "wd": normal((F, d), seed_for(cfg_index, layer, "wd"), WEIGHT_STD, dtype),
    }
    if with_dy:
        out["dy"] = normal((T, d), seed_for(cfg_index, layer, "dy"), 1.0, dtype)
    return out
