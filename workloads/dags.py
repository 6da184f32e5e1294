"""Seeded random fusible op-DAGs (the long-tail mix of small subgraphs).

draw_dag(k, attempt) is a pure function of (seed, k, attempt): it draws a
DAG of 4-16 operator nodes over {add, sub, mul, div with broadcast, exp, tanh,
sigmoid, gelu, rsqrt, sum/max/mean over the last dim, transpose of the last
two dims}, in fp32 or bf16, with 1e4-1e7 elements per full-size tensor, and
the recipe for its input tensors.  Shapes mix powers of two with awkward last
dims so that every floor(log2(d)/4) shape bucket from 1 to 3 occurs, as do
rows that are not a multiple of 16 bytes.

The generator keeps loose interval bounds on every node so that denominators
and rsqrt arguments are positive by construction and magnitudes stay
moderate; this is bookkeeping about the workload, not part of the method.
Which attempt of each k is used is recorded in cfg5_attempts.txt by a script
that checks every candidate with the CPU oracle (finite values, moderate
magnitudes, denominators away from zero, well conditioned in fp32).
"""
import math
import os

import numpy as np

from . import rng
from .configs import Workload
from .irtext import Builder

SEED = 4
N_DAGS = 256
LAST_DIMS = [64, 96, 128, 133, 256, 384, 512, 768, 1000, 1024, 2048, 4096, 11008]
BATCHES = [2, 3, 4, 8, 16]
MAG_LIMIT = 1e4
LOW_LIMIT = 1e-2


class _Draw:
    """Sequential uniforms from one counter-based stream."""

    def __init__(self, seed, stream):
        self.seed, self.stream, self.i = seed, stream, 0

    def u(self):
        v = rng.uniform01(self.seed, self.stream, self.i, 1)[0]
        self.i += 1
        return float(v)

    def below(self, n):
        return min(int(self.u() * n), n - 1)

    def pick(self, seq):
        return seq[self.below(len(seq))]

    def weighted(self, pairs):
        tot = sum(w for _, w in pairs)
        x = self.u() * tot
        for v, w in pairs:
            x -= w
            if x < 0:
                return v
        return pairs[-1][0]


class _Val:
    __slots__ = ("id", "shape", "mag", "low", "is_const", "pre_reduce")

    def __init__(self, id, shape, mag, low=None, is_const=False):
        self.id, self.shape, self.mag, self.low, self.is_const = id, tuple(shape), mag, low, is_const
        self.pre_reduce = None


def _stream(k, attempt, j):
    return (k * 64 + attempt) * 64 + j


def draw_dag(k, attempt=0, seed=SEED, with_inputs=True, max_rows=None):
    """Return a Workload for DAG k (attempt-th redraw).

    max_rows, if set, caps the product of the leading dims; the structure of
    the DAG does not depend on it, so a capped copy is a cheap stand-in for
    screening."""
    d = _Draw(seed, _stream(k, attempt, 63))
    dtype = d.pick(["f32", "bf16"])
    rank = d.pick([2, 3])
    total = 10.0 ** (4.0 + 3.0 * d.u())
    C = d.pick(LAST_DIMS)
    if rank == 2:
        shape = (max(1, int(round(total / C))), C)
    else:
        B = d.pick(BATCHES)
        shape = (B, max(1, int(round(total / (C * B)))), C)
    if max_rows is not None:
        lead = list(shape[:-1])
        while int(np.prod(lead)) > max_rows and lead[-1] > 1:
            lead[-1] = max(1, lead[-1] // 2)
        shape = tuple(lead) + (C,)
    n_ops = 4 + d.below(13)

    g = Builder()
    input_recipes = []          # (stream j, shape, positive)
    vals = []

    def fresh(shape, positive):
        # id None: declared only once an operator really uses it (see realise)
        v = _Val(None, shape, 6.5 if positive else 6.0, 0.5 if positive else None)
        v.pre_reduce = ("fresh", positive)
        return v

    def realise(v):
        if v.id is not None:
            return v
        if v.is_const:
            v.id = g.const(v.mag, dtype)
        else:
            positive = v.pre_reduce[1]
            v.pre_reduce = None
            v.id = g.input(dtype, v.shape)
            input_recipes.append((len(input_recipes), v.shape, positive))
        vals.append(v)
        return v

    def emit(op, operands, shape, mag, low, **attrs):
        operands = [realise(o) for o in operands]
        nid = g.op(op, [o.id for o in operands], dtype, **attrs)
        v = _Val(nid, shape, mag, low)
        vals.append(v)
        used.update(o.id for o in operands)
        return v

    used = set()
    cur = realise(fresh(shape, False))
    made = 0
    guard = 0
    while made < n_ops and guard < 200:
        guard += 1
        real = [v for v in vals if not v.is_const]
        a = cur if d.u() < 0.75 else d.pick(real)
        # after a reduction, mostly combine its result with the tensor it came from
        if isinstance(cur.pre_reduce, _Val) and d.u() < 0.8:
            kind = "bin_back"
        else:
            kind = d.weighted([("bin", 40), ("un", 30), ("red", 18), ("tr", 8)])
        if kind == "un":
            op = d.pick(["exp", "tanh", "sigmoid", "gelu", "rsqrt"])
            if op == "exp":
                if a.mag > 8.0:
                    continue
                cur = emit(op, [a], a.shape, math.exp(a.mag), math.exp(-a.mag))
            elif op == "tanh":
                cur = emit(op, [a], a.shape, 1.0, None)
            elif op == "sigmoid":
                if a.mag > 8.0:
                    continue
                cur = emit(op, [a], a.shape, 1.0, 1.0 / (1.0 + math.exp(a.mag)))
            elif op == "gelu":
                cur = emit(op, [a], a.shape, a.mag, None, approx="tanh")
            else:
                if a.low is None or a.low < LOW_LIMIT:
                    cands = [v for v in real if v.low is not None and v.low >= LOW_LIMIT]
                    if not cands:
                        continue
                    a = d.pick(cands)
                cur = emit(op, [a], a.shape, 1.0 / math.sqrt(a.low), 1.0 / math.sqrt(a.mag))
            made += 1
        elif kind == "red":
            if a.shape[-1] <= 1:
                continue
            op = d.pick(["sum", "max", "mean"])
            n = a.shape[-1]
            mag = a.mag * n if op == "sum" else a.mag
            low = None if a.low is None else (a.low * n if op == "sum" else a.low)
            if mag > MAG_LIMIT:
                continue
            src = a
            cur = emit(op, [a], a.shape[:-1] + (1,), mag, low)
            cur.pre_reduce = src
            made += 1
        elif kind == "tr":
            if len(a.shape) < 2 or a.shape[-1] <= 1 or a.shape[-2] <= 1:
                continue
            cur = emit("transpose", [a], a.shape[:-2] + (a.shape[-1], a.shape[-2]), a.mag, a.low)
            made += 1
        else:
            if kind == "bin_back":
                b, a = cur, cur.pre_reduce
            else:
                how = d.weighted([("node", 35), ("full", 20), ("col", 15), ("row", 15), ("scalar", 15)])
                if how == "node":
                    cands = [v for v in real if v is not a and _joins(a.shape, v.shape)]
                    if not cands:
                        continue
                    b = d.pick(cands)
                elif how == "full":
                    b = fresh(a.shape, d.u() < 0.3)
                elif how == "col":
                    b = fresh(a.shape[-1:], d.u() < 0.3)
                elif how == "row":
                    b = fresh(a.shape[:-1] + (1,), d.u() < 0.3)
                else:
                    c = round(0.25 + 1.75 * d.u(), 3)
                    b = _Val(None, (), c, c, is_const=True)
            op = d.pick(["add", "sub", "mul", "div"])
            x, y = (a, b) if d.u() < 0.5 else (b, a)
            if op == "div":
                ok_y = y.low is not None and y.low >= LOW_LIMIT
                ok_x = x.low is not None and x.low >= LOW_LIMIT
                if not ok_y and ok_x:
                    x, y = y, x
                elif not ok_y:
                    y = fresh(_bshape(x.shape, y.shape), True)
                mag = x.mag / y.low
                low = None if x.low is None else x.low / y.mag
            elif op == "mul":
                mag = x.mag * y.mag
                low = None if (x.low is None or y.low is None) else x.low * y.low
            elif op == "add":
                mag = x.mag + y.mag
                low = None if (x.low is None or y.low is None) else x.low + y.low
            else:
                mag, low = x.mag + y.mag, None
            if mag > MAG_LIMIT:
                continue
            cur = emit(op, [x, y], _bshape(x.shape, y.shape), mag, low)
            made += 1

    # outputs: every operator node nobody consumes
    for v in vals:
        if v.is_const:
            continue
        is_input = any(v.id == i for i, _, _ in g.inputs)
        if not is_input and v.id not in used:
            g.output(v.id)
    ins, in_dtypes, in_shapes = [], [], []
    for j, shp, positive in input_recipes:
        in_dtypes.append(dtype)
        in_shapes.append(shp)
        if with_inputs:
            ins.append(make_input(seed, _stream(k, attempt, j), shp, dtype, positive))
    out_shapes = []
    shape_of = {v.id: v.shape for v in vals}
    for o in g.outputs:
        out_shapes.append(shape_of[o])
    w = Workload("cfg5_dag%03d_a%d_%s_%s" % (k, attempt, dtype, "x".join(map(str, shape))), g.text(), ins,
                 in_dtypes, in_shapes, [dtype] * len(g.outputs), out_shapes,
                 meta={"k": k, "attempt": attempt, "dtype": dtype, "n_ops": made, "shape": shape,
                       "positive": [p for _, _, p in input_recipes]})
    return w.finish()


def make_input(seed, stream, shape, dtype, positive):
    n = int(np.prod(shape, dtype=np.int64))
    if not positive:
        return rng.normal_stored(seed, stream, n, dtype).reshape(shape)
    x = np.abs(rng.normal(seed, stream, n)) + 0.5           # |N(0,1)| + 0.5
    return rng.store(x, dtype).reshape(shape)


def _bshape(s1, s2):
    r = max(len(s1), len(s2))
    a = (1,) * (r - len(s1)) + tuple(s1)
    b = (1,) * (r - len(s2)) + tuple(s2)
    return tuple(max(x, y) for x, y in zip(a, b))


def _joins(sa, sb):
    """sb broadcasts against sa without growing beyond the larger of the two."""
    r = max(len(sa), len(sb))
    a = (1,) * (r - len(sa)) + tuple(sa)
    b = (1,) * (r - len(sb)) + tuple(sb)
    if any(x != y and x != 1 and y != 1 for x, y in zip(a, b)):
        return False
    out = tuple(max(x, y) for x, y in zip(a, b))
    return out == a or out == b


def accepted_attempts(path=None):
    """attempt index per DAG, as certified against the CPU oracle."""
    path = path or os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg5_attempts.txt")
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                k, a = line.split()[:2]
                out[int(k)] = int(a)
    return out


def cfg5(k, **kw):
    return draw_dag(k, accepted_attempts()[k], **kw)
