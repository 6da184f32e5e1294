"""Emitter for the text form of the op-DAG IR.

The text is the interchange between the workload generators, the CPU oracle
and the HIP library; each of the two has its own reader.  Grammar, one
statement per line ('#' starts a comment):

    in %<id> : <dtype>[d0,d1,...]
    %<id> = <op>(%a, %b, ...) {key=value, ...} : <dtype>
    out %<id>

Ids are consecutive from 0 in order of definition, so every operand refers
to an earlier line (the text is already a topological order).  <dtype> is
'f32' or 'bf16'.  Shapes of op nodes are inferred, never written.
"""


class Builder:
    def __init__(self):
        self.lines = []
        self.n = 0
        self.inputs = []          # (id, dtype, shape)
        self.outputs = []

    def _new(self):
        i = self.n
        self.n += 1
        return i

    def input(self, dtype, shape):
        i = self._new()
        self.lines.append("in %%%d : %s[%s]" % (i, dtype, ",".join(str(int(d)) for d in shape)))
        self.inputs.append((i, dtype, tuple(int(d) for d in shape)))
        return i

    def op(self, name, operands, dtype, **attrs):
        i = self._new()
        a = ""
        if attrs:
            a = " {" + ", ".join("%s=%s" % (k, _fmt(v)) for k, v in attrs.items()) + "}"
        self.lines.append("%%%d = %s(%s)%s : %s" % (
            i, name, ", ".join("%%%d" % o for o in operands), a, dtype))
        return i

    def const(self, value, dtype):
        return self.op("const", [], dtype, value=float(value))

    def output(self, node):
        self.lines.append("out %%%d" % node)
        self.outputs.append(node)

    def text(self):
        return "\n".join(self.lines) + "\n"


def _fmt(v):
    if isinstance(v, float):
        return repr(v)
    return str(v)
