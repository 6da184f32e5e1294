"""Python binding of libpf.so, the fused-subgraph engine for MI355X (gfx950).

Argument marshalling only: every step of the hot path (planning, kernel
specialisation, fused execution, error scoring) runs inside the library.  The
names mirror include/pf.h.  There is no fallback: if the library has not been
built (python -m paper_2605_29357_amd.build, or __graft_entry__.build())
every call raises.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpf.so")

PF_OK, PF_E_INVALID, PF_E_COMPILE, PF_E_RUNTIME, PF_E_NOMEM = 0, -1, -2, -3, -4
F32, BF16, F64, F16 = 0, 1, 2, 3
DTYPES = {"f32": F32, "bf16": BF16, "f64": F64, "f16": F16}
DTYPE_NAMES = {v: k for k, v in DTYPES.items()}
OPS = ["input", "const", "add", "sub", "mul", "div", "exp", "tanh", "sigmoid", "gelu", "rsqrt",
       "sum", "max", "mean", "var", "transpose", "rot_pairs", "roll", "slice", "maximum", "minimum"]
TEMPLATES = ["ew_flat", "row_resident", "tile", "row_loop", "col_reduce"]


class PfError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("pf status %d: %s" % (status, message))
        self.status = status


class _Attr(C.Structure):
    _fields_ = [("key", C.c_char_p), ("value", C.c_char_p)]


class _Options(C.Structure):
    _fields_ = [("fuse", C.c_int), ("intermediates_f32", C.c_int), ("tune_row_lanes", C.c_int),
                ("tune_row_unroll", C.c_int), ("tune_flat_unroll", C.c_int), ("tune_col_block", C.c_int),
                ("tune_tile_edge", C.c_int), ("reserved", C.c_int * 1)]


class _NodeInfo(C.Structure):
    _fields_ = [("op", C.c_int), ("dtype", C.c_int), ("rank", C.c_int), ("shape", C.c_int64 * 4),
                ("n_in", C.c_int), ("in_nodes", C.c_int * 2), ("is_output", C.c_int)]


class _PlanInfo(C.Structure):
    _fields_ = [("n_kernels", C.c_int), ("n_inputs", C.c_int), ("n_outputs", C.c_int),
                ("algorithmic_bytes", C.c_uint64), ("workspace_bytes", C.c_uint64), ("planned_bytes", C.c_uint64),
                ("n_groups", C.c_int), ("reserved_", C.c_int)]


class _JitStats(C.Structure):
    _fields_ = [("compiled", C.c_uint64), ("memory_hits", C.c_uint64), ("disk_hits", C.c_uint64), ("code_objects", C.c_uint64)]


class _GroupInfo(C.Structure):
    _fields_ = [("tmpl", C.c_int), ("n_nodes", C.c_int), ("nodes", C.c_int * 64), ("rows", C.c_int64),
                ("cols", C.c_int64), ("block_threads", C.c_int), ("grid_blocks", C.c_int64),
                ("lanes_per_row", C.c_int), ("bytes_read", C.c_uint64), ("bytes_written", C.c_uint64)]


class Pair(C.Structure):
    _fields_ = [("d_cand", C.c_void_p), ("d_ref", C.c_void_p), ("n", C.c_uint64), ("cand_dtype", C.c_int32),
                ("ref_dtype", C.c_int32), ("rtol", C.c_double), ("atol", C.c_double), ("equal_nan", C.c_int32),
                ("reserved", C.c_int32)]


class ScoreResult(C.Structure):
    _fields_ = [("max_abs", C.c_double), ("max_rel", C.c_double), ("n", C.c_uint64), ("n_viol", C.c_uint64),
                ("nan_cand", C.c_uint64), ("nan_ref", C.c_uint64), ("inf_cand", C.c_uint64), ("inf_ref", C.c_uint64),
                ("allclose", C.c_uint32), ("bit_identical", C.c_uint32), ("reserved_", C.c_uint64)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved_"}


LADDER_LEVELS, ES_LEVELS = 11, 15


class LadderResult(C.Structure):
    _fields_ = [("n", C.c_uint64), ("n_viol", C.c_uint64 * LADDER_LEVELS)]


class Case(C.Structure):
    _fields_ = [("speedup", C.c_double), ("error_class", C.c_int32), ("reserved", C.c_int32),
                ("n_viol", C.c_uint64 * LADDER_LEVELS)]


class Metrics(C.Structure):
    _fields_ = [("es", C.c_double * ES_LEVELS), ("as_", C.c_double)]


_lib_handle = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib_handle
    if _lib_handle is not None:
        return _lib_handle
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libpf.so is not built (%s); run `python -m paper_2605_29357_amd.build`" % LIB_PATH)
    # code objects of kernels that were specialised before are kept beside the library
    cache = os.environ.setdefault("PF_CACHE_DIR", os.path.join(_HERE, "_kcache"))
    try:
        os.makedirs(cache, exist_ok=True)
    except OSError:
        os.environ["PF_CACHE_DIR"] = ""
    L = C.CDLL(LIB_PATH)
    vp, ip, sz = C.c_void_p, C.POINTER(C.c_int), C.c_size_t
    sigs = {
        "pf_graph_create": [C.POINTER(vp)],
        "pf_graph_input": [vp, C.c_int, C.c_int, C.POINTER(C.c_int64), ip],
        "pf_graph_node": [vp, C.c_int, ip, C.c_int, C.POINTER(_Attr), C.c_int, C.c_int, ip],
        "pf_graph_output": [vp, C.c_int],
        "pf_graph_parse": [C.c_char_p, sz, C.POINTER(vp)],
        "pf_graph_print": [vp, C.c_char_p, sz, C.POINTER(sz)],
        "pf_graph_variant": [vp, ip, C.POINTER(C.c_int64), C.c_int, C.c_int, C.POINTER(vp)],
        "pf_graph_size": [vp, ip, ip, ip],
        "pf_graph_node_info": [vp, C.c_int, C.POINTER(_NodeInfo)],
        "pf_compile": [vp, C.POINTER(_Options), C.POINTER(vp)],
        "pf_exec_info": [vp, C.POINTER(_PlanInfo)],
        "pf_exec_group_info": [vp, C.c_int, C.POINTER(_GroupInfo)],
        "pf_exec_source": [vp, C.c_int, C.c_char_p, sz, C.POINTER(sz)],
        "pf_exec_kernel_name": [vp, C.c_int, C.c_char_p, sz, C.POINTER(sz)],
        "pf_execute_outer": [vp, C.c_int64, C.POINTER(C.c_void_p), C.c_int, C.POINTER(C.c_void_p), C.c_int, vp],
        "pf_jit_stats_get": [C.POINTER(_JitStats)],
        "pf_execute": [vp, C.POINTER(vp), C.c_int, C.POINTER(vp), C.c_int, vp, sz, vp],
        "pf_execute_timed": [vp, C.POINTER(vp), C.c_int, C.POINTER(vp), C.c_int, vp, sz, vp, vp, vp],
        "pf_score": [C.POINTER(Pair), C.c_int, vp, vp, sz, vp],
        "pf_score_static": [C.POINTER(Pair), C.c_int, vp, vp],
        "pf_score_all": [C.POINTER(Pair), C.c_int, vp, vp, vp, sz, vp],
        "pf_copy_bytes": [vp, vp, sz, vp],
        "pf_score_ladder": [C.POINTER(Pair), C.c_int, vp, vp, sz, vp],
        "pf_tolerance": [C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)],
        "pf_aggregate": [C.POINTER(Case), C.c_int, C.c_double, C.c_double, C.POINTER(Metrics)],
        "pf_fast_p": [C.POINTER(Case), C.c_int, C.c_double, C.c_int, C.POINTER(C.c_double)],
    }
    for name, args in sigs.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = C.c_int
    L.pf_graph_destroy.argtypes = [vp]
    L.pf_graph_destroy.restype = None
    L.pf_exec_destroy.argtypes = [vp]
    L.pf_exec_destroy.restype = None
    L.pf_options_default.argtypes = [C.POINTER(_Options)]
    L.pf_options_default.restype = None
    L.pf_score_workspace_bytes.argtypes = [C.c_int]
    L.pf_score_workspace_bytes.restype = sz
    L.pf_score_ladder_workspace_bytes.argtypes = [C.c_int]
    L.pf_score_ladder_workspace_bytes.restype = sz
    L.pf_score_all_workspace_bytes.argtypes = [C.c_int]
    L.pf_score_all_workspace_bytes.restype = sz
    L.pf_last_error.restype = C.c_char_p
    L.pf_version.restype = C.c_char_p
    _lib_handle = L
    return L


def _check(status):
    if status != PF_OK:
        raise PfError(status, lib().pf_last_error().decode("utf-8", "replace"))


def version():
    return lib().pf_version().decode()


class Graph:
    """pf_graph handle."""

    def __init__(self, text=None):
        self._h = C.c_void_p()
        if text is None:
            _check(lib().pf_graph_create(C.byref(self._h)))
        else:
            b = text.encode()
            _check(lib().pf_graph_parse(b, len(b), C.byref(self._h)))

    def __del__(self):
        if getattr(self, "_h", None) and _lib_handle is not None:
            _lib_handle.pf_graph_destroy(self._h)
            self._h = None

    def input(self, dtype, shape):
        out = C.c_int()
        arr = (C.c_int64 * max(len(shape), 1))(*shape)
        _check(lib().pf_graph_input(self._h, DTYPES[dtype], len(shape), arr, C.byref(out)))
        return out.value

    def node(self, op, operands, dtype, **attrs):
        out = C.c_int()
        ins = (C.c_int * max(len(operands), 1))(*operands)
        at = (_Attr * max(len(attrs), 1))()
        for i, (k, v) in enumerate(attrs.items()):
            at[i].key = k.encode()
            at[i].value = (repr(v) if isinstance(v, float) else str(v)).encode()
        _check(lib().pf_graph_node(self._h, OPS.index(op), ins, len(operands), at, len(attrs), DTYPES[dtype], C.byref(out)))
        return out.value

    def output(self, node):
        _check(lib().pf_graph_output(self._h, node))

    def text(self):
        need = C.c_size_t()
        _check(lib().pf_graph_print(self._h, None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value)
        _check(lib().pf_graph_print(self._h, buf, need.value, C.byref(need)))
        return buf.value.decode()

    def variant(self, shapes, from_dtype=None, to_dtype=None):
        """The same operators at other input shapes (one per graph input) and, optionally, another dtype."""
        n = len(shapes)
        ranks = (C.c_int * max(n, 1))(*[len(s) for s in shapes])
        flat = (C.c_int64 * (max(n, 1) * 4))()
        for k, s in enumerate(shapes):
            for d, v in enumerate(s):
                flat[k * 4 + d] = int(v)
        if self.size()[1] != n:
            raise PfError(PF_E_INVALID, "graph has %d inputs, %d shapes given" % (self.size()[1], n))
        g = Graph.__new__(Graph)
        g._h = C.c_void_p()
        _check(lib().pf_graph_variant(self._h, ranks, flat, DTYPES[from_dtype] if from_dtype else -1,
                                      DTYPES[to_dtype] if to_dtype else -1, C.byref(g._h)))
        return g

    def size(self):
        a, b, c = C.c_int(), C.c_int(), C.c_int()
        _check(lib().pf_graph_size(self._h, C.byref(a), C.byref(b), C.byref(c)))
        return a.value, b.value, c.value

    def node_info(self, node):
        ni = _NodeInfo()
        _check(lib().pf_graph_node_info(self._h, node, C.byref(ni)))
        return {"op": OPS[ni.op], "dtype": DTYPE_NAMES[ni.dtype], "shape": tuple(ni.shape[:ni.rank]),
                "inputs": list(ni.in_nodes[:ni.n_in]), "is_output": bool(ni.is_output)}


class Exec:
    """pf_exec handle: a planned and compiled subgraph."""

    def __init__(self, graph, fuse=True, intermediates_f32=None, **tune):
        self._h = C.c_void_p()
        opt = _Options()
        lib().pf_options_default(C.byref(opt))
        opt.fuse = 1 if fuse else 0
        for k, v in tune.items():            # tune_row_lanes, tune_row_unroll, tune_flat_unroll
            setattr(opt, k, int(v))
        if intermediates_f32 is not None:
            opt.intermediates_f32 = 1 if intermediates_f32 else 0
        if isinstance(graph, str):
            graph = Graph(graph)
        self.graph = graph
        _check(lib().pf_compile(graph._h, C.byref(opt), C.byref(self._h)))

    def __del__(self):
        if getattr(self, "_h", None) and _lib_handle is not None:
            _lib_handle.pf_exec_destroy(self._h)
            self._h = None

    def info(self):
        pi = _PlanInfo()
        _check(lib().pf_exec_info(self._h, C.byref(pi)))
        return {k: getattr(pi, k) for k, _ in pi._fields_}

    def group_info(self, i):
        gi = _GroupInfo()
        _check(lib().pf_exec_group_info(self._h, i, C.byref(gi)))
        d = {k: getattr(gi, k) for k, _ in gi._fields_ if k not in ("nodes", "tmpl")}
        d["template"] = TEMPLATES[gi.tmpl]
        d["nodes"] = list(gi.nodes[:gi.n_nodes])
        return d

    def groups(self):
        return [self.group_info(i) for i in range(self.info()["n_groups"])]

    def source(self, i):
        need = C.c_size_t()
        _check(lib().pf_exec_source(self._h, i, None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value)
        _check(lib().pf_exec_source(self._h, i, buf, need.value, C.byref(need)))
        return buf.value.decode()

    def execute_outer(self, outer_extent, input_ptrs, output_ptrs, stream=0):
        """As execute, at another (smaller) outermost extent than the compiled one; one-kernel subgraphs only."""
        ins = (C.c_void_p * len(input_ptrs))(*input_ptrs)
        outs = (C.c_void_p * len(output_ptrs))(*output_ptrs)
        _check(lib().pf_execute_outer(self._h, int(outer_extent), ins, len(input_ptrs), outs, len(output_ptrs), C.c_void_p(stream)))

    def kernel_name(self, i):
        need = C.c_size_t()
        _check(lib().pf_exec_kernel_name(self._h, i, None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value)
        _check(lib().pf_exec_kernel_name(self._h, i, buf, need.value, C.byref(need)))
        return buf.value.decode()

    def execute(self, input_ptrs, output_ptrs, workspace_ptr=0, workspace_bytes=0, stream=0, start_event=0, stop_event=0):
        """Device pointers as ints; enqueues the kernels on `stream` (a hipStream_t as int).
        start_event / stop_event: optional hipEvent_t handles bracketing the kernels themselves."""
        ins = (C.c_void_p * max(len(input_ptrs), 1))(*input_ptrs)
        outs = (C.c_void_p * max(len(output_ptrs), 1))(*output_ptrs)
        if start_event or stop_event:
            _check(lib().pf_execute_timed(self._h, ins, len(input_ptrs), outs, len(output_ptrs), C.c_void_p(workspace_ptr),
                                          workspace_bytes, C.c_void_p(stream), C.c_void_p(start_event), C.c_void_p(stop_event)))
        else:
            _check(lib().pf_execute(self._h, ins, len(input_ptrs), outs, len(output_ptrs),
                                    C.c_void_p(workspace_ptr), workspace_bytes, C.c_void_p(stream)))


def score_workspace_bytes(n_pairs):
    return lib().pf_score_workspace_bytes(n_pairs)


def score(pairs, results_ptr, workspace_ptr, workspace_bytes, stream=0):
    """pairs: list of Pair; results_ptr: device pointer to len(pairs) ScoreResult structs."""
    arr = (Pair * max(len(pairs), 1))(*pairs)
    _check(lib().pf_score(arr, len(pairs), C.c_void_p(results_ptr), C.c_void_p(workspace_ptr), workspace_bytes,
                          C.c_void_p(stream)))


SCORE_STATIC_MAX_PAIRS = 256


def score_static(pairs, results_ptr, stream=0):
    """As score, with the library's own scratch array as the workspace (no device allocation anywhere)."""
    arr = (Pair * max(len(pairs), 1))(*pairs)
    _check(lib().pf_score_static(arr, len(pairs), C.c_void_p(results_ptr), C.c_void_p(stream)))


def copy_bytes(dst_ptr, src_ptr, nbytes, stream=0):
    _check(lib().pf_copy_bytes(C.c_void_p(dst_ptr), C.c_void_p(src_ptr), nbytes, C.c_void_p(stream)))


def jit_stats():
    """Code-object cache counters of this process: compiled, memory_hits, disk_hits, code_objects."""
    st = _JitStats()
    _check(lib().pf_jit_stats_get(C.byref(st)))
    return {k: getattr(st, k) for k, _ in st._fields_}


def tolerance(dtype, t):
    """(rtol, atol) of tolerance index t for a dtype name."""
    r, a = C.c_double(), C.c_double()
    _check(lib().pf_tolerance(DTYPES[dtype], t, C.byref(r), C.byref(a)))
    return r.value, a.value


def score_ladder_workspace_bytes(n_pairs):
    return lib().pf_score_ladder_workspace_bytes(n_pairs)


def score_ladder(pairs, results_ptr, workspace_ptr, workspace_bytes, stream=0):
    """results_ptr: device pointer to len(pairs) LadderResult structs."""
    arr = (Pair * max(len(pairs), 1))(*pairs)
    _check(lib().pf_score_ladder(arr, len(pairs), C.c_void_p(results_ptr), C.c_void_p(workspace_ptr), workspace_bytes,
                                 C.c_void_p(stream)))


def score_all_workspace_bytes(n_pairs):
    return lib().pf_score_all_workspace_bytes(n_pairs)


def score_all(pairs, score_results_ptr, ladder_results_ptr, workspace_ptr, workspace_bytes, stream=0):
    """Both results from one read of every pair: len(pairs) ScoreResult and len(pairs) LadderResult structs."""
    arr = (Pair * max(len(pairs), 1))(*pairs)
    _check(lib().pf_score_all(arr, len(pairs), C.c_void_p(score_results_ptr), C.c_void_p(ladder_results_ptr),
                              C.c_void_p(workspace_ptr), workspace_bytes, C.c_void_p(stream)))


def _cases(cases):
    arr = (Case * max(len(cases), 1))()
    for i, c in enumerate(cases):
        arr[i].speedup = c["speedup"]
        arr[i].error_class = c["error_class"]
        for k, v in enumerate(c["viol"]):
            arr[i].n_viol[k] = v
    return arr


def aggregate(cases, b=0.1, p=0.0):
    """cases: dicts(speedup, error_class, viol[11]).  Returns (ES_t for t=-10..4, AS)."""
    m = Metrics()
    _check(lib().pf_aggregate(_cases(cases), len(cases), b, p, C.byref(m)))
    return list(m.es), m.as_


def fast_p(cases, threshold, t=0):
    out = C.c_double()
    _check(lib().pf_fast_p(_cases(cases), len(cases), threshold, t, C.byref(out)))
    return out.value
