// Op-DAG IR: construction, shape inference, text reader and writer.
//
// A graph is the paper's Definition 3.1: operator nodes, data-dependency
// edges, an operator type per node and an output shape per node.  Shapes of
// operator nodes are inferred here; all of this is integer work.
#include <cctype>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "pf_internal.h"

namespace pf {

void fail(pf_status s, const char* fmt, ...) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    throw Error(s, buf);
}

std::string strf(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    va_list ap2;
    va_copy(ap2, ap);
    int n = vsnprintf(nullptr, 0, fmt, ap);
    va_end(ap);
    std::string out(n > 0 ? n : 0, '\0');
    if (n > 0) vsnprintf(out.data(), n + 1, fmt, ap2);
    va_end(ap2);
    return out;
}

static const char* kOpNames[PF_OP_COUNT_] = {
    "input", "const", "add", "sub", "mul", "div", "exp", "tanh", "sigmoid", "gelu",
    "rsqrt", "sum", "max", "mean", "var", "transpose", "rot_pairs", "roll", "slice", "maximum", "minimum"};

const char* op_name(pf_op op) { return (op >= 0 && op < PF_OP_COUNT_) ? kOpNames[op] : "?"; }

bool op_from_name(const std::string& name, pf_op* op) {
    for (int i = 1; i < PF_OP_COUNT_; ++i)
        if (name == kOpNames[i]) {
            *op = (pf_op)i;
            return true;
        }
    return false;
}

const char* dtype_name(pf_dtype d) { return d == PF_F32 ? "f32" : d == PF_BF16 ? "bf16" : d == PF_F16 ? "f16" : "f64"; }

bool is_reduction(pf_op op) { return op == PF_OP_SUM || op == PF_OP_MAX || op == PF_OP_MEAN || op == PF_OP_VAR; }
bool is_unary(pf_op op) {
    return op == PF_OP_EXP || op == PF_OP_TANH || op == PF_OP_SIGMOID || op == PF_OP_GELU || op == PF_OP_RSQRT ||
           op == PF_OP_ROT_PAIRS;
}
bool is_binary(pf_op op) {
    return op == PF_OP_ADD || op == PF_OP_SUB || op == PF_OP_MUL || op == PF_OP_DIV || op == PF_OP_MAXIMUM || op == PF_OP_MINIMUM;
}

Shape broadcast_shapes(const Shape& a, const Shape& b) {
    size_t r = a.size() > b.size() ? a.size() : b.size();
    Shape out(r, 1);
    for (size_t i = 0; i < r; ++i) {
        int64_t da = i < r - a.size() ? 1 : a[i - (r - a.size())];
        int64_t db = i < r - b.size() ? 1 : b[i - (r - b.size())];
        if (da != db && da != 1 && db != 1) fail(PF_E_COMPILE, "shapes do not broadcast (dim %zu: %lld vs %lld)", i,
                                                 (long long)da, (long long)db);
        out[i] = da > db ? da : db;
    }
    return out;
}

static void check_dtype(pf_dtype dt) {
    if (dt != PF_F32 && dt != PF_BF16 && dt != PF_F16) fail(PF_E_COMPILE, "unsupported tensor dtype %d (f32, bf16 and f16 only)", (int)dt);
}

int graph_add_input(pf_graph& g, pf_dtype dt, const Shape& shape) {
    check_dtype(dt);
    if (shape.size() > PF_MAX_RANK) fail(PF_E_COMPILE, "rank %zu exceeds %d", shape.size(), PF_MAX_RANK);
    for (int64_t d : shape)
        if (d <= 0) fail(PF_E_COMPILE, "dims must be positive (got %lld)", (long long)d);
    if (numel(shape) >= (int64_t(1) << 40)) fail(PF_E_COMPILE, "tensor too large");
    Node n;
    n.op = PF_OP_INPUT;
    n.dtype = dt;
    n.shape = shape;
    g.nodes.push_back(n);
    g.inputs.push_back((int)g.nodes.size() - 1);
    return (int)g.nodes.size() - 1;
}

static long long parse_ll_attr(const std::string& k, const std::string& v) {
    char* end = nullptr;
    long long x = strtoll(v.c_str(), &end, 10);
    if (end == v.c_str() || *end) fail(PF_E_COMPILE, "attribute %s needs an integer, got '%s'", k.c_str(), v.c_str());
    return x;
}

static int parse_int_attr(const std::string& k, const std::string& v) {
    char* end = nullptr;
    long x = strtol(v.c_str(), &end, 10);
    if (end == v.c_str() || *end) fail(PF_E_COMPILE, "attribute %s needs an integer, got '%s'", k.c_str(), v.c_str());
    return (int)x;
}

int graph_add_node(pf_graph& g, pf_op op, const std::vector<int>& in,
                   const std::vector<std::pair<std::string, std::string>>& attrs, pf_dtype dt) {
    check_dtype(dt);
    if (op <= PF_OP_INPUT || op >= PF_OP_COUNT_) fail(PF_E_COMPILE, "unknown operator %d", (int)op);
    const int id = (int)g.nodes.size();
    for (int i : in)
        if (i < 0 || i >= id) fail(PF_E_COMPILE, "%%%d: operand %%%d is not an earlier node", id, i);
    Node n;
    n.op = op;
    n.dtype = dt;
    n.in = in;
    const size_t want = op == PF_OP_CONST ? 0 : is_binary(op) ? 2 : 1;
    if (in.size() != want) fail(PF_E_COMPILE, "%%%d: %s takes %zu operand(s), got %zu", id, op_name(op), want, in.size());
    bool have_value = false, have_dim = false, have_shift = false, have_start = false, have_stop = false;
    for (auto& kv : attrs) {
        const std::string &k = kv.first, &v = kv.second;
        if (k == "value" && op == PF_OP_CONST) {
            char* end = nullptr;
            n.value = strtod(v.c_str(), &end);
            if (end == v.c_str() || *end) fail(PF_E_COMPILE, "%%%d: bad const value '%s'", id, v.c_str());
            have_value = true;
        } else if (k == "keepdim" && is_reduction(op)) {
            n.keepdim = parse_int_attr(k, v);
            if (n.keepdim != 0 && n.keepdim != 1) fail(PF_E_COMPILE, "%%%d: keepdim must be 0 or 1", id);
        } else if (k == "correction" && op == PF_OP_VAR) {
            n.correction = parse_int_attr(k, v);
        } else if (k == "dim" && is_reduction(op)) {
            n.red_dim = parse_int_attr(k, v);
            if (n.red_dim != -1 && n.red_dim != -2) fail(PF_E_COMPILE, "%%%d: reductions take dim=-1 or dim=-2", id);
        } else if (k == "dim" && is_view(op)) {
            n.dim = parse_int_attr(k, v);
            have_dim = true;
        } else if (k == "shift" && op == PF_OP_ROLL) {
            n.shift = parse_ll_attr(k, v);
            have_shift = true;
        } else if (k == "start" && op == PF_OP_SLICE) {
            n.start = parse_ll_attr(k, v);
            have_start = true;
        } else if (k == "stop" && op == PF_OP_SLICE) {
            n.stop = parse_ll_attr(k, v);
            have_stop = true;
        } else if (k == "approx" && op == PF_OP_GELU) {
            if (v == "tanh") n.gelu_erf = 0;
            else if (v == "erf") n.gelu_erf = 1;
            else fail(PF_E_COMPILE, "%%%d: gelu approx must be tanh or erf", id);
        } else {
            fail(PF_E_COMPILE, "%%%d: attribute '%s' is not valid for %s", id, k.c_str(), op_name(op));
        }
    }
    if (op == PF_OP_CONST) {
        if (!have_value) fail(PF_E_COMPILE, "%%%d: const needs value=", id);
        n.shape = {};
    } else if (is_binary(op)) {
        n.shape = broadcast_shapes(g.nodes[in[0]].shape, g.nodes[in[1]].shape);
    } else if (is_reduction(op)) {
        const Shape& s = g.nodes[in[0]].shape;
        if (s.empty()) fail(PF_E_COMPILE, "%%%d: cannot reduce a scalar", id);
        if ((int)s.size() < -n.red_dim) fail(PF_E_COMPILE, "%%%d: dim %d needs rank >= %d", id, n.red_dim, -n.red_dim);
        const size_t ax = s.size() + n.red_dim;
        if (op == PF_OP_VAR && s[ax] - n.correction <= 0)
            fail(PF_E_COMPILE, "%%%d: var over %lld elements with correction %d", id, (long long)s[ax], n.correction);
        n.shape = s;
        if (n.keepdim) n.shape[ax] = 1;
        else n.shape.erase(n.shape.begin() + ax);
    } else if (op == PF_OP_TRANSPOSE) {
        const Shape& s = g.nodes[in[0]].shape;
        if (s.size() < 2) fail(PF_E_COMPILE, "%%%d: transpose needs rank >= 2", id);
        n.shape = s;
        std::swap(n.shape[s.size() - 1], n.shape[s.size() - 2]);
    } else if (is_view(op)) {
        const Shape& s = g.nodes[in[0]].shape;
        const int r = (int)s.size();
        if (!have_dim) fail(PF_E_COMPILE, "%%%d: %s needs dim=", id, op_name(op));
        if (n.dim < -r || n.dim >= r) fail(PF_E_COMPILE, "%%%d: dim %d out of range for rank %d", id, n.dim, r);
        if (n.dim < 0) n.dim += r;
        n.shape = s;
        if (op == PF_OP_ROLL) {
            if (!have_shift) fail(PF_E_COMPILE, "%%%d: roll needs shift=", id);
        } else {
            if (!have_start || !have_stop) fail(PF_E_COMPILE, "%%%d: slice needs start= and stop=", id);
            if (n.start < 0 || n.start >= n.stop || n.stop > s[n.dim])
                fail(PF_E_COMPILE, "%%%d: slice [%lld:%lld] out of bounds for a dim of %lld", id, (long long)n.start, (long long)n.stop,
                     (long long)s[n.dim]);
            n.shape[n.dim] = n.stop - n.start;
        }
    } else if (op == PF_OP_ROT_PAIRS) {
        const Shape& s = g.nodes[in[0]].shape;
        if (s.empty() || (s.back() & 1)) fail(PF_E_COMPILE, "%%%d: rot_pairs needs an even last dim", id);
        n.shape = s;
    } else {
        n.shape = g.nodes[in[0]].shape;
    }
    // the same size limit as for inputs (a broadcast can grow far beyond its operands); the product is
    // formed step by step so that it cannot wrap around first
    int64_t count = 1;
    for (int64_t d : n.shape) {
        if (count >= (int64_t(1) << 40) / d + 1) fail(PF_E_COMPILE, "%%%d: result tensor too large", id);
        count *= d;
    }
    if (count >= (int64_t(1) << 40)) fail(PF_E_COMPILE, "%%%d: result tensor too large", id);
    g.nodes.push_back(n);
    return id;
}

void graph_add_output(pf_graph& g, int node) {
    if (node < 0 || node >= (int)g.nodes.size()) fail(PF_E_COMPILE, "output %%%d is not a node", node);
    if (g.nodes[node].op == PF_OP_CONST) fail(PF_E_COMPILE, "a const cannot be a graph output");
    g.nodes[node].is_output = true;
    g.outputs.push_back(node);
}

// ---------------------------------------------------------------- text form

namespace {

struct Cursor {
    const std::string& s;
    size_t p = 0;
    int line_no;
    Cursor(const std::string& str, int ln) : s(str), line_no(ln) {}
    void ws() {
        while (p < s.size() && (s[p] == ' ' || s[p] == '\t')) ++p;
    }
    bool eat(char c) {
        ws();
        if (p < s.size() && s[p] == c) {
            ++p;
            return true;
        }
        return false;
    }
    void need(char c) {
        if (!eat(c)) fail(PF_E_COMPILE, "line %d: expected '%c' at column %zu", line_no, c, p + 1);
    }
    std::string word() {
        ws();
        size_t b = p;
        while (p < s.size() && (isalnum((unsigned char)s[p]) || s[p] == '_' || s[p] == '.' || s[p] == '-' ||
                                s[p] == '+'))
            ++p;
        if (b == p) fail(PF_E_COMPILE, "line %d: expected a token at column %zu", line_no, p + 1);
        return s.substr(b, p - b);
    }
    int id() {
        need('%');
        size_t b = p;
        while (p < s.size() && isdigit((unsigned char)s[p])) ++p;
        if (b == p || p - b > 9) fail(PF_E_COMPILE, "line %d: expected a node id", line_no);
        return atoi(s.substr(b, p - b).c_str());
    }
    bool end() {
        ws();
        return p >= s.size();
    }
};

pf_dtype parse_dtype(const std::string& w, int line_no) {
    if (w == "f32") return PF_F32;
    if (w == "bf16") return PF_BF16;
    if (w == "f16") return PF_F16;
    fail(PF_E_COMPILE, "line %d: unknown dtype '%s'", line_no, w.c_str());
}

}  // namespace

void graph_parse(const std::string& text, pf_graph& g) {
    size_t pos = 0;
    int line_no = 0;
    while (pos <= text.size()) {
        size_t nl = text.find('\n', pos);
        if (nl == std::string::npos) nl = text.size();
        std::string line = text.substr(pos, nl - pos);
        pos = nl + 1;
        ++line_no;
        size_t hash = line.find('#');
        if (hash != std::string::npos) line.resize(hash);
        Cursor c(line, line_no);
        if (c.end()) continue;
        if (line.compare(c.p, 3, "in ") == 0 || line.compare(c.p, 3, "in\t") == 0) {
            c.p += 2;
            int id = c.id();
            if (id != (int)g.nodes.size()) fail(PF_E_COMPILE, "line %d: ids must be consecutive (expected %%%zu)", line_no, g.nodes.size());
            c.need(':');
            pf_dtype dt = parse_dtype(c.word(), line_no);
            c.need('[');
            Shape shape;
            if (!c.eat(']')) {
                do {
                    std::string w = c.word();
                    char* end = nullptr;
                    long long d = strtoll(w.c_str(), &end, 10);
                    if (*end) fail(PF_E_COMPILE, "line %d: bad dim '%s'", line_no, w.c_str());
                    shape.push_back(d);
                } while (c.eat(','));
                c.need(']');
            }
            if (!c.end()) fail(PF_E_COMPILE, "line %d: trailing text", line_no);
            graph_add_input(g, dt, shape);
        } else if (line.compare(c.p, 4, "out ") == 0 || line.compare(c.p, 4, "out\t") == 0) {
            c.p += 3;
            int id = c.id();
            if (!c.end()) fail(PF_E_COMPILE, "line %d: trailing text", line_no);
            graph_add_output(g, id);
        } else {
            int id = c.id();
            if (id != (int)g.nodes.size()) fail(PF_E_COMPILE, "line %d: ids must be consecutive (expected %%%zu)", line_no, g.nodes.size());
            c.need('=');
            std::string name = c.word();
            pf_op op;
            if (!op_from_name(name, &op)) fail(PF_E_COMPILE, "line %d: unknown operator '%s'", line_no, name.c_str());
            c.need('(');
            std::vector<int> in;
            if (!c.eat(')')) {
                do in.push_back(c.id());
                while (c.eat(','));
                c.need(')');
            }
            std::vector<std::pair<std::string, std::string>> attrs;
            if (c.eat('{')) {
                if (!c.eat('}')) {
                    do {
                        std::string k = c.word();
                        c.need('=');
                        attrs.emplace_back(k, c.word());
                    } while (c.eat(','));
                    c.need('}');
                }
            }
            c.need(':');
            pf_dtype dt = parse_dtype(c.word(), line_no);
            if (!c.end()) fail(PF_E_COMPILE, "line %d: trailing text", line_no);
            graph_add_node(g, op, in, attrs, dt);
        }
    }
}

// The same operator sequence at other input shapes / another dtype (the members G_i of a task
// instance, paper Sec. 3.1): the graph is printed, its input lines are rewritten, tensors of dtype
// `from` become `to`, and the text is parsed again, which re-infers every shape and re-validates
// the attributes (slice bounds, reduction sizes) against the new shapes.
void graph_variant(const pf_graph& g, const int* ranks, const int64_t* shapes, int from, int to, pf_graph& out) {
    const std::string text = graph_print(g);
    const std::string f = from >= 0 ? dtype_name((pf_dtype)from) : "", t = to >= 0 ? dtype_name((pf_dtype)to) : "";
    std::string res;
    size_t pos = 0, k = 0;
    while (pos < text.size()) {
        size_t nl = text.find('\n', pos);
        if (nl == std::string::npos) nl = text.size();
        std::string line = text.substr(pos, nl - pos);
        pos = nl + 1;
        if (line.compare(0, 3, "in ") == 0) {
            const size_t colon = line.find(':'), br = line.find('[');
            std::string dt = line.substr(colon + 2, br - colon - 2);
            if (from >= 0 && dt == f) dt = t;
            if (k >= g.inputs.size()) fail(PF_E_INVALID, "internal: input count");
            const int r = ranks[k];
            if (r < 0 || r > PF_MAX_RANK) fail(PF_E_INVALID, "input %zu: rank %d out of range", k, r);
            line = line.substr(0, colon + 2) + dt + "[";
            for (int d = 0; d < r; ++d) line += strf(d ? ",%lld" : "%lld", (long long)shapes[k * PF_MAX_RANK + d]);
            line += "]";
            ++k;
        } else if (line.compare(0, 1, "%") == 0 && from >= 0) {
            const size_t colon = line.rfind(": ");
            if (colon != std::string::npos && line.substr(colon + 2) == f) line = line.substr(0, colon + 2) + t;
        }
        res += line;
        res += '\n';
    }
    graph_parse(res, out);
}

std::string graph_print(const pf_graph& g) {
    std::string out;
    for (size_t i = 0; i < g.nodes.size(); ++i) {
        const Node& n = g.nodes[i];
        if (n.op == PF_OP_INPUT) {
            out += strf("in %%%zu : %s[", i, dtype_name(n.dtype));
            for (size_t d = 0; d < n.shape.size(); ++d) out += strf(d ? ",%lld" : "%lld", (long long)n.shape[d]);
            out += "]\n";
            continue;
        }
        out += strf("%%%zu = %s(", i, op_name(n.op));
        for (size_t k = 0; k < n.in.size(); ++k) out += strf(k ? ", %%%d" : "%%%d", n.in[k]);
        out += ")";
        if (n.op == PF_OP_CONST) out += strf(" {value=%.17g}", n.value);
        else if (n.op == PF_OP_GELU) out += strf(" {approx=%s}", n.gelu_erf ? "erf" : "tanh");
        else if (n.op == PF_OP_VAR) out += strf(" {correction=%d, keepdim=%d, dim=%d}", n.correction, n.keepdim, n.red_dim);
        else if (is_reduction(n.op)) out += strf(" {keepdim=%d, dim=%d}", n.keepdim, n.red_dim);
        else if (n.op == PF_OP_ROLL) out += strf(" {shift=%lld, dim=%d}", (long long)n.shift, n.dim);
        else if (n.op == PF_OP_SLICE) out += strf(" {dim=%d, start=%lld, stop=%lld}", n.dim, (long long)n.start, (long long)n.stop);
        out += strf(" : %s\n", dtype_name(n.dtype));
    }
    for (int o : g.outputs) out += strf("out %%%d\n", o);
    return out;
}

}  // namespace pf
