"""CPU oracle: plain op-by-op evaluation of an op-DAG in fp64.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
package; it exists so that tests and the benchmark's CPU baseline have an
independent statement of what a fusible subgraph computes.

A computational graph (paper Def. 3.1) is a DAG whose nodes carry an operator
type and an output shape; f_G maps its inputs to its outputs.  Fusion must
leave f_G unchanged (Def. 3.2, Eq. 1), so the oracle is the definition
written out: one NumPy call per node, every intermediate a full fp64 array,
no fusion, no tiling, no rounding of intermediates.  It has its own reader
for the text IR and shares no code with the HIP library.

Operator definitions (x, y operands; last-dim reductions keep the dim unless
keepdim=0):
  add sub mul div      NumPy right-aligned broadcasting
  exp tanh             libm
  sigmoid              1 / (1 + exp(-x))
  rsqrt                1 / sqrt(x)
  gelu approx=tanh     0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))
       approx=erf      0.5 x (1 + erf(x / sqrt 2))
  maximum minimum      element-wise, NaN-propagating (torch.maximum; clamp(x, min=c) = maximum(x, c))
  sum max mean         over the last dim (dim=-1, default) or the one before it (dim=-2, the
                       sequence dim of the paper's Case 2: masked mean pooling sums over s in
                       out[b,d] = sum_s h[b,s,d] m[b,s,d] / max(sum_s m[b,s,d], 1e-9)); max propagates NaN
  var                  mean((x - mean x)^2) * n / (n - correction); the
                       LayerNorm of the paper's Case 1 divides by n
                       (correction 0) and adds eps inside the square root
  transpose            swaps the last two dims
  rot_pairs            out[2i] = -x[2i+1], out[2i+1] = x[2i] on the last dim
  const                a scalar (rank 0)
  roll                 out[..., i, ...] = x[..., (i - shift) mod S, ...] along dim (torch.roll / np.roll);
                       the paper's Case 1 reads a roll by 3 followed by a prefix slice as
                       input index (S + i - shift) mod S
  slice                x[..., start:stop, ...] along dim
"""
import math
import re

import numpy as np

_IN = re.compile(r"^in\s+%(\d+)\s*:\s*(\w+)\[([^\]]*)\]$")
_OP = re.compile(r"^%(\d+)\s*=\s*(\w+)\(([^)]*)\)\s*(\{[^}]*\})?\s*:\s*(\w+)$")
_OUT = re.compile(r"^out\s+%(\d+)$")


class Node:
    __slots__ = ("id", "op", "args", "attrs", "dtype", "shape")

    def __init__(self, id, op, args, attrs, dtype, shape=None):
        self.id, self.op, self.args, self.attrs, self.dtype, self.shape = id, op, args, attrs, dtype, shape


class Graph:
    def __init__(self):
        self.nodes = []
        self.inputs = []
        self.outputs = []


def parse(text):
    g = Graph()
    for raw in text.splitlines():
        line = raw.split("#", 1)[0].strip()
        if not line:
            continue
        m = _IN.match(line)
        if m:
            nid = int(m.group(1))
            if nid != len(g.nodes):
                raise ValueError("ids must be consecutive: " + line)
            shape = tuple(int(t) for t in m.group(3).split(",") if t.strip())
            g.nodes.append(Node(nid, "input", [], {}, m.group(2), shape))
            g.inputs.append(nid)
            continue
        m = _OP.match(line)
        if m:
            nid = int(m.group(1))
            if nid != len(g.nodes):
                raise ValueError("ids must be consecutive: " + line)
            args = [int(t.strip().lstrip("%")) for t in m.group(3).split(",") if t.strip()]
            if any(a >= nid for a in args):
                raise ValueError("operand defined later: " + line)
            attrs = {}
            if m.group(4):
                for kv in m.group(4)[1:-1].split(","):
                    if kv.strip():
                        k, v = kv.split("=")
                        attrs[k.strip()] = v.strip()
            g.nodes.append(Node(nid, m.group(2), args, attrs, m.group(5)))
            continue
        m = _OUT.match(line)
        if m:
            g.outputs.append(int(m.group(1)))
            continue
        raise ValueError("cannot parse: " + raw)
    return g


def upconvert(arr, dtype, to=np.float64):
    """Exact widening of stored bits ('f32' float32 array; 'bf16' and 'f16' uint16 bits)."""
    if dtype == "f32":
        return np.asarray(arr, dtype=np.float32).astype(to)
    if dtype == "bf16":
        u = np.asarray(arr, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
        return u.view(np.float32).astype(to)
    if dtype == "f16":
        # IEEE binary16: sign, 5 exponent bits (bias 15), 10 fraction bits
        u = np.asarray(arr, dtype=np.uint16).astype(np.int64)
        ex, frac = (u >> 10) & 31, u & 1023
        mag = np.where(ex == 0, np.ldexp(frac.astype(np.float64), -24),                     # zero and subnormals
                       np.ldexp((1024 + frac).astype(np.float64), (ex - 25).astype(np.int32)))
        mag = np.where(ex == 31, np.where(frac == 0, np.inf, np.nan), mag)
        return np.where((u >> 15) == 1, -mag, mag).astype(to)
    raise ValueError(dtype)


def _erf(x):
    return np.vectorize(math.erf, otypes=[x.dtype])(x)


def run(graph, inputs, dtype=np.float64, observer=None):
    """Evaluate the DAG node by node.

    inputs: stored arrays in the order of the graph's `in` lines.  Returns the
    list of output arrays (dtype `dtype`, never rounded to the node dtype).
    `dtype=np.float32` evaluates the same definition in single precision; it
    is used only to judge whether a synthetic DAG is well conditioned.
    `observer(node, value, operand_values)` sees every node as it is computed.
    """
    if isinstance(graph, str):
        graph = parse(graph)
    if len(inputs) != len(graph.inputs):
        raise ValueError("expected %d inputs" % len(graph.inputs))
    ft = dtype
    val = {}
    last_use = {}
    for n in graph.nodes:
        for a in n.args:
            last_use[a] = n.id
    for o in graph.outputs:
        last_use[o] = len(graph.nodes)
    k = 0
    for n in graph.nodes:
        if n.op == "input":
            v = upconvert(inputs[k], n.dtype, ft)
            if tuple(v.shape) != n.shape:
                raise ValueError("input %d has shape %s, declared %s" % (k, v.shape, n.shape))
            k += 1
            val[n.id] = v
            continue
        a = [val[i] for i in n.args]
        op = n.op
        with np.errstate(all="ignore"):
            if op == "const":
                v = np.array(float(n.attrs["value"]), dtype=ft)
            elif op == "add":
                v = a[0] + a[1]
            elif op == "sub":
                v = a[0] - a[1]
            elif op == "mul":
                v = a[0] * a[1]
            elif op == "div":
                v = a[0] / a[1]
            elif op == "maximum":
                v = np.maximum(a[0], a[1])
            elif op == "minimum":
                v = np.minimum(a[0], a[1])
            elif op == "exp":
                v = np.exp(a[0])
            elif op == "tanh":
                v = np.tanh(a[0])
            elif op == "sigmoid":
                v = ft(1.0) / (ft(1.0) + np.exp(-a[0]))
            elif op == "rsqrt":
                v = ft(1.0) / np.sqrt(a[0])
            elif op == "gelu":
                x = a[0]
                if n.attrs.get("approx", "tanh") == "tanh":
                    c = ft(math.sqrt(2.0 / math.pi))
                    v = ft(0.5) * x * (ft(1.0) + np.tanh(c * (x + ft(0.044715) * x * x * x)))
                else:
                    v = ft(0.5) * x * (ft(1.0) + _erf(x / ft(math.sqrt(2.0))))
            elif op in ("sum", "max", "mean", "var"):
                x = a[0]
                ax = int(n.attrs.get("dim", -1))
                if ax not in (-1, -2) or x.ndim < -ax:
                    raise ValueError("reduction dim must be -1 or -2 and exist")
                if op == "sum":
                    v = np.sum(x, axis=ax, keepdims=True)
                elif op == "max":
                    v = np.max(x, axis=ax, keepdims=True)            # np.max propagates NaN
                elif op == "mean":
                    v = np.sum(x, axis=ax, keepdims=True) / ft(x.shape[ax])
                else:
                    cnt = x.shape[ax]
                    mu = np.sum(x, axis=ax, keepdims=True) / ft(cnt)
                    d = x - mu
                    corr = int(n.attrs.get("correction", 0))
                    v = np.sum(d * d, axis=ax, keepdims=True) / ft(cnt - corr)
                if int(n.attrs.get("keepdim", 1)) == 0:
                    v = np.squeeze(v, axis=ax)
            elif op == "transpose":
                if a[0].ndim < 2:
                    raise ValueError("transpose needs rank >= 2")
                v = np.ascontiguousarray(np.swapaxes(a[0], -1, -2))
            elif op == "roll":
                x = a[0]
                d = int(n.attrs["dim"])
                if not -x.ndim <= d < x.ndim:
                    raise ValueError("roll dim out of range")
                v = np.roll(x, int(n.attrs["shift"]), axis=d)
            elif op == "slice":
                x = a[0]
                d = int(n.attrs["dim"])
                if not -x.ndim <= d < x.ndim:
                    raise ValueError("slice dim out of range")
                lo, hi = int(n.attrs["start"]), int(n.attrs["stop"])
                if not 0 <= lo < hi <= x.shape[d]:
                    raise ValueError("slice bounds")
                idx = [slice(None)] * x.ndim
                idx[d] = slice(lo, hi)
                v = np.ascontiguousarray(x[tuple(idx)])
            elif op == "rot_pairs":
                x = a[0]
                if x.ndim < 1 or x.shape[-1] % 2:
                    raise ValueError("rot_pairs needs an even last dim")
                v = np.empty_like(x)
                v[..., 0::2] = -x[..., 1::2]
                v[..., 1::2] = x[..., 0::2]
            else:
                raise ValueError("unknown op " + op)
        v = np.asarray(v, dtype=ft)
        n.shape = tuple(v.shape)
        if observer is not None:
            observer(n, v, a)
        val[n.id] = v
        for i in set(n.args):            # free what is no longer needed
            if last_use.get(i) == n.id:
                del val[i]
    return [val[o] for o in graph.outputs]
