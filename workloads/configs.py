"""The four named synthetic workloads (fused subgraphs of known structure).

Each function returns a Workload: the DAG in text form, the input tensors as
stored bits, the comparison tolerances and the bytes that must cross HBM
(every external input once + every output once).  `rows` arguments shrink a
workload along its leading dims for quick tests; the defaults are the full
sizes.  "N(m, s)" means mean m and standard deviation s throughout.
"""
from dataclasses import dataclass, field
import numpy as np

from . import rng
from .irtext import Builder

ITEMSIZE = {"f32": 4, "bf16": 2, "f16": 2}
# comparison tolerances against the fp64 oracle, by dtype of the graph output
RTOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 1e-3}
ATOL = {"f32": 1e-5, "bf16": 1e-5, "f16": 1e-5}


@dataclass
class Workload:
    name: str
    text: str
    inputs: list                      # numpy arrays: float32, or uint16 for bf16
    input_dtypes: list                # 'f32' | 'bf16'
    input_shapes: list
    output_dtypes: list
    output_shapes: list
    algorithmic_bytes: int = 0
    meta: dict = field(default_factory=dict)

    def finish(self):
        b = 0
        for d, s in zip(self.input_dtypes, self.input_shapes):
            b += ITEMSIZE[d] * int(np.prod(s, dtype=np.int64))
        for d, s in zip(self.output_dtypes, self.output_shapes):
            b += ITEMSIZE[d] * int(np.prod(s, dtype=np.int64))
        self.algorithmic_bytes = b
        return self


def _tensor(seed, idx, shape, dtype, mean=0.0, std=1.0):
    n = int(np.prod(shape, dtype=np.int64))
    return rng.normal_stored(seed, idx, n, dtype, mean, std).reshape(shape)


def cfg1_add_layernorm(rows=64, cols=768, seed=0, use_var_op=False):
    """Residual add + LayerNorm over the last dim, fp32, eps = 1e-5."""
    g = Builder()
    x = g.input("f32", (rows, cols))
    r = g.input("f32", (rows, cols))
    gamma = g.input("f32", (cols,))
    beta = g.input("f32", (cols,))
    h = g.op("add", [x, r], "f32")
    mu = g.op("mean", [h], "f32")
    d = g.op("sub", [h, mu], "f32")
    if use_var_op:
        v = g.op("var", [h], "f32", correction=0)
    else:
        v = g.op("mean", [g.op("mul", [d, d], "f32")], "f32")
    eps = g.const(1e-5, "f32")
    inv = g.op("rsqrt", [g.op("add", [v, eps], "f32")], "f32")
    y = g.op("add", [g.op("mul", [g.op("mul", [d, inv], "f32"), gamma], "f32"), beta], "f32")
    g.output(y)
    ins = [_tensor(seed, 0, (rows, cols), "f32"), _tensor(seed, 1, (rows, cols), "f32"),
           _tensor(seed, 2, (cols,), "f32", 1.0, 0.1), _tensor(seed, 3, (cols,), "f32", 0.0, 0.1)]
    return Workload("cfg1_add_layernorm_f32_%dx%d" % (rows, cols), g.text(), ins,
                    ["f32"] * 4, [(rows, cols), (rows, cols), (cols,), (cols,)],
                    ["f32"], [(rows, cols)], meta={"eps": 1e-5}).finish()


def causal_mask_bits(n, dtype="bf16"):
    """Additive causal mask [n, n] in the stored form of `dtype`: 0 on and below the diagonal, -inf above."""
    if dtype == "f32":
        m = np.zeros((n, n), dtype=np.float32)
        m[np.triu_indices(n, k=1)] = -np.inf
        return m
    m = np.zeros((n, n), dtype=np.uint16)
    m[np.triu_indices(n, k=1)] = np.uint16({"bf16": 0xFF80, "f16": 0xFC00}[dtype])
    return m


def cfg2_masked_softmax(heads=32, seq=512, seed=1, dtype="bf16"):
    """Scaled, causally masked softmax over the last dim, bf16 (or fp16); scale = 1/sqrt(64)."""
    g = Builder()
    z = g.input(dtype, (heads, seq, seq))
    m = g.input(dtype, (seq, seq))
    s = g.const(0.125, dtype)
    t = g.op("add", [g.op("mul", [z, s], dtype), m], dtype)
    mx = g.op("max", [t], dtype)
    e = g.op("exp", [g.op("sub", [t, mx], dtype)], dtype)
    y = g.op("div", [e, g.op("sum", [e], dtype)], dtype)
    g.output(y)
    ins = [_tensor(seed, 0, (heads, seq, seq), dtype, 0.0, 2.0), causal_mask_bits(seq, dtype)]
    return Workload("cfg2_masked_softmax_%s_%dx%dx%d" % (dtype, heads, seq, seq), g.text(), ins,
                    [dtype, dtype], [(heads, seq, seq), (seq, seq)],
                    [dtype], [(heads, seq, seq)], meta={"scale": 0.125}).finish()


def cfg3_bias_gelu_gate(rows=8192, cols=11008, seed=2, dtype="bf16"):
    """out = gelu_tanh(a + bias) * b, bf16 (or fp16), bias broadcast over rows."""
    g = Builder()
    a = g.input(dtype, (rows, cols))
    bias = g.input(dtype, (cols,))
    b = g.input(dtype, (rows, cols))
    y = g.op("mul", [g.op("gelu", [g.op("add", [a, bias], dtype)], dtype, approx="tanh"), b], dtype)
    g.output(y)
    ins = [_tensor(seed, 0, (rows, cols), dtype), _tensor(seed, 1, (cols,), dtype, 0.0, 0.02),
           _tensor(seed, 2, (rows, cols), dtype)]
    return Workload("cfg3_bias_gelu_gate_%s_%dx%d" % (dtype, rows, cols), g.text(), ins,
                    [dtype] * 3, [(rows, cols), (cols,), (rows, cols)],
                    [dtype], [(rows, cols)]).finish()


def rotary_tables(positions, dim, base=10000.0):
    """cos/sin tables [positions, 1, dim] in fp32 for interleaved pairs.

    Pair i of the last dim (elements 2i, 2i+1) at position p turns by
    theta = p * base**(-2i/dim); both elements of a pair hold the same entry.
    """
    i = np.arange(dim // 2, dtype=np.float64)
    inv_freq = base ** (-2.0 * i / dim)
    theta = np.arange(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    cos = np.repeat(np.cos(theta), 2, axis=1).reshape(positions, 1, dim)
    sin = np.repeat(np.sin(theta), 2, axis=1).reshape(positions, 1, dim)
    return cos.astype(np.float32), sin.astype(np.float32)


def cfg4_rmsnorm_rope(batch=4, positions=2048, heads=32, dim=128, seed=3, dtype="bf16"):
    """Weighted RMSNorm over the last dim (eps = 1e-6) then rotary embedding, bf16 (or fp16)."""
    g = Builder()
    shape = (batch, positions, heads, dim)
    x = g.input(dtype, shape)
    w = g.input(dtype, (dim,))
    cos = g.input("f32", (positions, 1, dim))
    sin = g.input("f32", (positions, 1, dim))
    ms = g.op("mean", [g.op("mul", [x, x], dtype)], dtype)
    eps = g.const(1e-6, "f32")
    inv = g.op("rsqrt", [g.op("add", [ms, eps], dtype)], dtype)
    n = g.op("mul", [g.op("mul", [x, inv], dtype), w], dtype)
    y = g.op("add", [g.op("mul", [n, cos], dtype),
                     g.op("mul", [g.op("rot_pairs", [n], dtype), sin], dtype)], dtype)
    g.output(y)
    c, s = rotary_tables(positions, dim)
    ins = [_tensor(seed, 0, shape, dtype), _tensor(seed, 1, (dim,), dtype, 1.0, 0.1), c, s]
    return Workload("cfg4_rmsnorm_rope_%s_%dx%dx%dx%d" % ((dtype,) + shape), g.text(), ins,
                    [dtype, dtype, "f32", "f32"], [shape, (dim,), (positions, 1, dim), (positions, 1, dim)],
                    [dtype], [shape], meta={"eps": 1e-6, "base": 10000.0}).finish()


def roll_slice_add_layernorm(S=133, SC=128, C=96, shift=3, dtype="bf16", seed=5):
    """The paper's Case 1 subgraph: x [S,S,C] rolled by `shift` along dims 0 and 1, cut to
    [SC,SC,C], added to a residual, LayerNorm over C (eps 1e-5); both the sum and the
    normalised tensor are outputs.  Routes in the paper: (133,128,96), (70,64,192), (35,32,384)."""
    g = Builder()
    x = g.input(dtype, (S, S, C))
    r = g.input(dtype, (SC, SC, C))
    gamma = g.input(dtype, (C,))
    beta = g.input(dtype, (C,))
    t = g.op("roll", [x], dtype, shift=shift, dim=0)
    t = g.op("roll", [t], dtype, shift=shift, dim=1)
    t = g.op("slice", [t], dtype, dim=0, start=0, stop=SC)
    t = g.op("slice", [t], dtype, dim=1, start=0, stop=SC)
    h = g.op("add", [r, t], dtype)
    mu = g.op("mean", [h], dtype)
    d = g.op("sub", [h, mu], dtype)
    v = g.op("mean", [g.op("mul", [d, d], dtype)], dtype)
    inv = g.op("rsqrt", [g.op("add", [v, g.const(1e-5, "f32")], dtype)], dtype)
    y = g.op("add", [g.op("mul", [g.op("mul", [d, inv], dtype), gamma], dtype), beta], dtype)
    g.output(h)
    g.output(y)
    ins = [_tensor(seed, 0, (S, S, C), dtype), _tensor(seed, 1, (SC, SC, C), dtype),
           _tensor(seed, 2, (C,), dtype, 1.0, 0.1), _tensor(seed, 3, (C,), dtype, 0.0, 0.1)]
    w = Workload("roll_slice_add_layernorm_%s_S%d_SC%d_C%d" % (dtype, S, SC, C), g.text(), ins,
                 [dtype] * 4, [(S, S, C), (SC, SC, C), (C,), (C,)], [dtype, dtype], [(SC, SC, C), (SC, SC, C)],
                 meta={"eps": 1e-5, "shift": shift}).finish()
    # the rolled-and-cut window touches SC*SC of the S*S rows of x: bytes that must move
    isz = ITEMSIZE[dtype]
    w.algorithmic_bytes = isz * (SC * SC * C * 4 + 2 * C)
    return w


def masked_mean_pooling(B=32, S=512, D=1024, seed=6, dtype="bf16"):
    """The paper's Case 2 subgraph: out[b,d] = sum_s h[b,s,d] m[b,s,d] / max(sum_s m[b,s,d], 1e-9),
    hidden states bf16, mask fp32 (0/1 per token, expanded over d), output fp32 [B,D]."""
    g = Builder()
    m = g.input("f32", (B, S, D))
    h = g.input(dtype, (B, S, D))
    num = g.op("sum", [g.op("mul", [h, m], "f32")], "f32", dim=-2, keepdim=0)
    den = g.op("sum", [m], "f32", dim=-2, keepdim=0)
    out = g.op("div", [num, g.op("maximum", [den, g.const(1e-9, "f32")], "f32")], "f32")
    g.output(out)
    # token lengths vary per sequence; one sequence is fully masked (denominator clamps)
    lens = [0] + [1 + rng.randint(seed, 99, b, 0, S) for b in range(1, B)]
    mask = np.zeros((B, S, D), np.float32)
    for b, n in enumerate(lens):
        mask[b, :n, :] = 1.0
    ins = [mask, _tensor(seed, 1, (B, S, D), dtype)]
    return Workload("masked_mean_pooling_%s_B%d_S%d_D%d" % (dtype, B, S, D), g.text(), ins, ["f32", dtype], [(B, S, D)] * 2,
                    ["f32"], [(B, D)], meta={"lens": lens}).finish()
