"""Task instances: one operator sequence at ten shape configurations (paper Sec. 3.1 and the
benchmark-construction section: every subgraph is instantiated at 10 shapes and 3 dtypes; shapes
are bucketed per dimension by floor(log2(d) / 4)).

Each family below is one of the named subgraphs; `instance(family, dtype)` returns its ten
workloads.  The last dims cover buckets 1, 2 and 3 (16 ... 65535), power-of-two and awkward
lengths, and the leading dims range from a handful of rows to tens of thousands, so that no single
tiling fits all members.  Sizes stay near two million elements so that the fp64 oracle takes
seconds per member.
"""
import math

from . import configs

FAMILIES = ("add_layernorm", "masked_softmax", "bias_gelu_gate", "rmsnorm_rope", "masked_mean_pooling")


def bucket(d):
    """The paper's logarithmic shape quantisation of one dimension."""
    return int(math.floor(math.log2(d) / 4))


_LN = [(60000, 24), (16384, 96), (11279, 133), (8192, 192), (4000, 384), (2048, 768), (1500, 1000), (733, 2048), (384, 4096),
       (130, 11008)]
_SM = [(4096, 16), (900, 48), (512, 64), (200, 100), (128, 128), (113, 133), (32, 256), (8, 512), (2, 1000), (1, 4096)]
_GG = [(100000, 16), (65536, 24), (20000, 96), (15000, 133), (5000, 384), (2000, 1000), (2048, 1024), (500, 4096), (190, 11008),
       (67, 30000)]
_RR = [(2, 512, 32, 64), (1, 2048, 8, 128), (4, 17, 32, 128), (1, 128, 128, 96), (8, 64, 4, 256), (1, 1000, 3, 512), (16, 8, 16, 32),
       (2, 300, 32, 128), (1, 16, 2, 4096), (3, 333, 5, 160)]
_MP = [(32, 64, 256), (8, 512, 64), (4, 100, 264), (2, 1000, 133), (16, 33, 1024), (1, 2048, 512), (64, 16, 96), (3, 77, 4096),
       (5, 300, 24), (2, 4096, 48)]

SHAPES = {"add_layernorm": _LN, "masked_softmax": _SM, "bias_gelu_gate": _GG, "rmsnorm_rope": _RR, "masked_mean_pooling": _MP}
DEFAULT_DTYPE = {"add_layernorm": "f32", "masked_softmax": "bf16", "bias_gelu_gate": "bf16", "rmsnorm_rope": "bf16",
                 "masked_mean_pooling": "bf16"}


def member(family, k, dtype=None):
    """Member k (0..9) of a family's task instance."""
    dt = dtype or DEFAULT_DTYPE[family]
    s = SHAPES[family][k]
    if family == "add_layernorm":
        if dt != "f32":
            raise ValueError("add_layernorm is the fp32 subgraph")
        return configs.cfg1_add_layernorm(rows=s[0], cols=s[1], seed=100 + k)
    if family == "masked_softmax":
        return configs.cfg2_masked_softmax(heads=s[0], seq=s[1], seed=110 + k, dtype=dt)
    if family == "bias_gelu_gate":
        return configs.cfg3_bias_gelu_gate(rows=s[0], cols=s[1], seed=120 + k, dtype=dt)
    if family == "rmsnorm_rope":
        return configs.cfg4_rmsnorm_rope(*s, seed=130 + k, dtype=dt)
    if family == "masked_mean_pooling":
        return configs.masked_mean_pooling(*s, seed=140 + k, dtype=dt)
    raise ValueError(family)


def instance(family, dtype=None):
    return [member(family, k, dtype) for k in range(len(SHAPES[family]))]
