"""Workload shapes of the MoC FFN hot path.

The (d_model, d_ff) pairs are the LLaMA shapes the paper trains (appendix table of
model configurations: 512/1376, 768/2048, 2048/5461) and the LLaMA-7B shape it
names for its larger runs (4096/11008).  K is d_ff/8 here.  This module holds
shapes only: no arithmetic of the method.
"""
from collections import namedtuple

MocConfig = namedtuple("MocConfig", "name T d F K dtype what")

CONFIGS = {
    "cfg0": MocConfig("cfg0", 256, 512, 1376, 172, "f32", "fwd"),
    "cfg1": MocConfig("cfg1", 4096, 768, 2048, 256, "bf16", "fwd+bwd"),
    "cfg2": MocConfig("cfg2", 8192, 2048, 5461, 683, "bf16", "fwd+bwd"),      # "1B shape"
    "cfg3": MocConfig("cfg3", 16, 4096, 11008, 1376, "bf16", "decode"),       # "7B shape", B = 1, 4, 16
    "cfg4": MocConfig("cfg4", 8192, 4096, 11008, 1376, "bf16", "stack32"),
}

DECODE_BATCHES = (1, 4, 16)
STACK_LAYERS = 32
RMSNORM_EPS = 1e-5
