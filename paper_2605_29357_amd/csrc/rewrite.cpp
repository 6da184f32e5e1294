// Graph rewrite ahead of planning: transposes of computed values are pushed down
// to what those values are computed from.
//
// A transpose of a value that a kernel computes forces the value through memory
// (written in one orientation, read back in the other), and in the paper's terms
// ends a fusible run (Sec. 3.2).  For an elementwise producer the round trip is
// avoidable: transpose(f(a, b)) = f(transpose(a), transpose(b)), so the consumer's
// kernel can recompute f on operands it reads in its own orientation.  Operands
// with a last or second-to-last extent of 1 (weights, per-row statistics) change
// orientation without moving data; full-size ones go through the tile kernel's
// LDS transpose like any transposed input.  A value needed in both orientations is
// computed in both: recomputation costs arithmetic, the round trip costs HBM traffic.
//
// The rewrite clones the elementwise cone above such a transpose, bounded by what
// the recomputation reads compared with what the round trip would move, and drops
// nodes nothing observes any more.  Every node of the rewritten graph remembers the
// user's node it computes (Node::orig), so reports keep the user's numbering.
#include <algorithm>
#include <map>
#include <set>

#include "pf_internal.h"

namespace pf {

namespace {

bool sinkable_op(pf_op op) { return (is_unary(op) && op != PF_OP_ROT_PAIRS) || is_binary(op); }

Shape swapped(const Shape& s) {
    Shape t = s;
    if (t.size() < 2) t.insert(t.begin(), 2 - t.size(), 1);
    std::swap(t[t.size() - 1], t[t.size() - 2]);
    return t;
}

// does reading the tensor through a swap of its last two dims leave its linear order unchanged?
bool moves_no_data(const Shape& s) { return s.size() < 2 || s[s.size() - 1] == 1 || s[s.size() - 2] == 1; }

struct Sinker {
    const pf_graph& src;
    const pf_options& opt;
    pf_graph out;
    std::vector<int> map;              // old id -> new id of the same value
    std::map<int, int> tnode;          // old id -> new id of a node holding its transposed value

    Sinker(const pf_graph& g, const pf_options& o) : src(g), opt(o), map(g.nodes.size(), -1) {}

    int push(const Node& n) {
        out.nodes.push_back(n);
        return (int)out.nodes.size() - 1;
    }

    // a read of old node x through a swap of its last two dims: (new node id, read as an alias)
    struct Ref {
        int id;
        bool alias;
    };

    int mem_bytes(const Node& n) const { return opt.intermediates_f32 ? 4 : itemsize(n.dtype); }

    // What recomputing transpose(x) would read: full-size tensors that have to move, and their bytes per element.
    void cone(int x, std::set<int>& seen, int& n_nodes, int& n_full, int& bytes) const {
        if (!seen.insert(x).second) return;
        const Node& n = src.nodes[x];
        if (n.op == PF_OP_CONST || n.shape.empty()) return;
        if (n.op == PF_OP_TRANSPOSE) {
            // transpose(transpose(y)) is y itself: a plain read, or in-kernel if y is computed by the consumer's kernel
            const Node& y = src.nodes[n.in[0]];
            if (y.op == PF_OP_INPUT) bytes += moves_no_data(y.shape) ? 0 : itemsize(y.dtype);
            else bytes += moves_no_data(y.shape) ? 0 : mem_bytes(y);
            return;
        }
        if (moves_no_data(n.shape)) return;
        if (sinkable_op(n.op) && n.shape.size() >= 2) {
            ++n_nodes;
            for (int p : n.in) cone(p, seen, n_nodes, n_full, bytes);
            return;
        }
        ++n_full;
        bytes += n.op == PF_OP_INPUT ? itemsize(n.dtype) : mem_bytes(n);
    }

    bool worth_sinking(int v) const {
        const Node& n = src.nodes[v];
        if (!sinkable_op(n.op) || n.shape.size() < 2 || moves_no_data(n.shape)) return false;
        std::set<int> seen;
        int n_nodes = 0, n_full = 0, bytes = 0;
        cone(v, seen, n_nodes, n_full, bytes);
        // the round trip: a store (free if the value is an output that later kernels can read as it is) and a load
        const bool stored_anyway = n.is_output && (n.dtype == PF_F32 || !opt.intermediates_f32);
        const int saved = stored_anyway ? itemsize(n.dtype) : 2 * mem_bytes(n);
        return n_nodes <= 24 && n_full <= 3 && bytes <= saved;
    }

    Ref transposed(int x, bool top) {
        const Node& n = src.nodes[x];
        if (n.op == PF_OP_CONST || n.shape.empty()) return {map[x], false};
        if (n.op == PF_OP_TRANSPOSE && src.nodes[n.in[0]].shape.size() >= 2) return {map[n.in[0]], false};
        if (moves_no_data(n.shape)) return {map[x], true};
        auto it = tnode.find(x);
        if (it != tnode.end()) return {it->second, false};
        int id;
        if (sinkable_op(n.op) && n.shape.size() >= 2 && (!top || worth_sinking(x))) {
            Node c = n;
            c.is_output = false;
            c.orig = x;
            c.shape = swapped(n.shape);
            c.alias_t.assign(n.in.size(), 0);
            for (size_t k = 0; k < n.in.size(); ++k) {
                const Ref r = transposed(n.in[k], false);
                c.in[k] = r.id;
                c.alias_t[k] = r.alias ? 1 : 0;
            }
            id = push(c);
        } else {
            Node t;
            t.op = PF_OP_TRANSPOSE;
            t.dtype = n.dtype;
            t.in = {map[x]};
            t.shape = swapped(n.shape);
            t.orig = -1;
            id = push(t);
        }
        tnode[x] = id;
        return {id, false};
    }

    void run() {
        for (size_t i = 0; i < src.nodes.size(); ++i) {
            const Node& n = src.nodes[i];
            if (n.op == PF_OP_TRANSPOSE && n.shape.size() >= 2) {
                const int v = n.in[0];
                const Node& x = src.nodes[v];
                if (x.op == PF_OP_TRANSPOSE && x.dtype == src.nodes[x.in[0]].dtype && n.dtype == x.dtype && src.nodes[x.in[0]].shape.size() >= 2 &&
                    src.nodes[x.in[0]].op != PF_OP_INPUT) {
                    // transposed twice: the value itself (an output slot of its own if the user asked for one)
                    map[i] = map[x.in[0]];
                    if (n.is_output) out.nodes[map[i]].is_output = true;
                    continue;
                }
                const bool computed = x.op != PF_OP_INPUT && x.op != PF_OP_CONST;
                if (computed && x.op != PF_OP_TRANSPOSE && worth_sinking(v)) {
                    const Ref r = transposed(v, true);
                    // the clone at the top of the cone stands for the transpose node itself
                    out.nodes[r.id].orig = (int)i;
                    out.nodes[r.id].dtype = n.dtype;
                    if (n.is_output) out.nodes[r.id].is_output = true;
                    map[i] = r.id;
                    tnode.erase(v);            // another transpose of v would be another user node
                    continue;
                }
            }
            Node c = n;
            c.orig = (int)i;
            for (size_t k = 0; k < c.in.size(); ++k) c.in[k] = map[c.in[k]];
            map[i] = push(c);
        }
        for (int i : src.inputs) out.inputs.push_back(map[i]);
        for (int o : src.outputs) out.outputs.push_back(map[o]);
    }

    // drops what no output depends on any more (graph inputs stay: they are the call's arguments)
    void prune() {
        std::vector<char> live(out.nodes.size(), 0);
        for (int o : out.outputs) live[o] = 1;
        for (int i = (int)out.nodes.size() - 1; i >= 0; --i)
            if (live[i])
                for (int p : out.nodes[i].in) live[p] = 1;
        for (int i : out.inputs) live[i] = 1;
        std::vector<int> renum(out.nodes.size(), -1);
        pf_graph g;
        for (size_t i = 0; i < out.nodes.size(); ++i) {
            if (!live[i]) continue;
            Node c = out.nodes[i];
            for (int& p : c.in) p = renum[p];
            renum[i] = (int)g.nodes.size();
            g.nodes.push_back(c);
        }
        for (int i : out.inputs) g.inputs.push_back(renum[i]);
        for (int o : out.outputs) g.outputs.push_back(renum[o]);
        out = g;
    }
};

}  // namespace

void sink_transposes(const pf_graph& g, const pf_options& opt, pf_graph& out) {
    Sinker s(g, opt);
    s.run();
    s.prune();
    out = s.out;
}

}  // namespace pf
