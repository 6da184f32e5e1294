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
// The same identity serves reductions: a reduction over the last dim of a value that only exists
// transposed (an elementwise cone over transposed tensors) is a reduction over the second-to-last
// dim of the cone evaluated in the tensors' own orientation, which a column-reduction kernel reads
// straight from memory.  The result has the same linear order either way ([.., R, 1] against
// [.., 1, R]), so its readers take it as it lies.  Whether that pays depends on what else needs the
// transposed value, so the caller chooses the reductions to treat this way ("sites") by planning
// both ways.
//
// A third use: when a transpose of a computed value is not worth pushing down by itself (the value's kernel
// computes other results from the same tensors, so they would be read twice), the transpose's kernel can
// take over those results as well: it computes them in its own orientation from the tensors it stages
// anyway and writes them through a transposed store.  The value's kernel then disappears.  These
// transposes are sites of the caller's search, too.
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
    std::map<int, int> pnode;          // old id -> new id of a copy computed inside a column reduction's kernel
    std::set<int> sites;               // reductions (old ids) to run as column reductions in their sources' orientation
    std::set<int> standin;             // old ids whose new node has the last two dims swapped (same linear order)
    bool in_site = false;              // cloning the cone of a column-reduction site
    std::set<int> taken_over;          // outputs (old ids) a chosen transpose's kernel computes in its orientation and stores transposed

    std::vector<std::vector<int>> readers;   // per old node: the nodes that read it

    Sinker(const pf_graph& g, const pf_options& o, const std::vector<int>& chosen = {})
        : src(g), opt(o), map(g.nodes.size(), -1), sites(chosen.begin(), chosen.end()), readers(g.nodes.size()) {
        for (size_t i = 0; i < g.nodes.size(); ++i)
            for (int p : g.nodes[i].in) readers[p].push_back((int)i);
        for (int t : sites)
            if (t >= 0 && g.nodes[t].op == PF_OP_TRANSPOSE)
                for (int y : outputs_to_take_over(t)) taken_over.insert(y);
    }

    // full-size tensors the elementwise cone of x reads from memory; false if the cone holds something that
    // cannot be recomputed in the other orientation
    bool cone_leaves(int x, std::set<int>& seen, std::set<int>& leaves, int& n_nodes) const {
        if (!seen.insert(x).second) return true;
        const Node& n = src.nodes[x];
        if (n.op == PF_OP_CONST || n.shape.empty() || moves_no_data(n.shape)) return true;
        if (sinkable_op(n.op) && n.shape.size() >= 2) {
            ++n_nodes;
            for (int p : n.in)
                if (!cone_leaves(p, seen, leaves, n_nodes)) return false;
            return true;
        }
        if (n.op == PF_OP_TRANSPOSE || is_view(n.op)) return false;
        leaves.insert(x);
        return true;
    }

    // A transpose that nothing reads but the caller, of a computed elementwise value: instead of recomputing the value in
    // the other orientation (a kernel of its own unless other work of that orientation exists), the kernel that
    // computes the value can write it out both ways.  Sites of this kind are listed as store_site(node).
    static int store_site(int t) { return -(t + 1); }
    bool store_through_possible(int t) const {
        const Node& tn = src.nodes[t];
        if (tn.op != PF_OP_TRANSPOSE || tn.shape.size() < 2 || !tn.is_output || !readers[t].empty()) return false;
        const Node& x = src.nodes[tn.in[0]];
        return sinkable_op(x.op) && x.shape.size() >= 2 && !moves_no_data(x.shape) && x.dtype == tn.dtype;
    }

    // A transpose t = transpose(v) of a computed elementwise value: the outputs of v's own orientation and shape that
    // read some of what v's cone reads.  Empty if t is no such site.
    std::vector<int> outputs_to_take_over(int t) const {
        std::vector<int> ys;
        const Node& tn = src.nodes[t];
        if (tn.op != PF_OP_TRANSPOSE || tn.shape.size() < 2) return ys;
        const int v = tn.in[0];
        const Node& x = src.nodes[v];
        if (!sinkable_op(x.op) || x.shape.size() < 2 || moves_no_data(x.shape)) return ys;
        std::set<int> seen, leaves;
        int n_nodes = 0;
        if (!cone_leaves(v, seen, leaves, n_nodes) || n_nodes > 24 || leaves.empty() || leaves.size() > 8) return ys;
        for (size_t y = 0; y < src.nodes.size(); ++y) {
            const Node& yn = src.nodes[y];
            if (!yn.is_output || !sinkable_op(yn.op) || yn.shape != x.shape) continue;      // (y may be v itself: needed both ways)
            std::set<int> ys_seen, ys_leaves;
            int yn_nodes = 0;
            if (!cone_leaves((int)y, ys_seen, ys_leaves, yn_nodes) || yn_nodes > 24) continue;
            // at least one tensor in common (its bytes are saved), and few enough staged tensors in all; whether
            // the extra ones pay is the traffic model's call
            size_t shared = 0;
            for (int l : ys_leaves) shared += leaves.count(l);
            if (shared >= 1 && leaves.size() + ys_leaves.size() - shared <= 8) ys.push_back((int)y);
        }
        return ys;
    }

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

    // Is transpose(x) computable without moving data: every full-size leaf of x's elementwise cone is itself a
    // transpose (read plainly in the other orientation) and everything else is a constant or changes orientation
    // in place?  n_t counts the transposes that disappear.
    void free_cone(int x, std::set<int>& seen, int& n_nodes, int& n_t, bool& ok) const {
        if (!seen.insert(x).second) return;
        const Node& n = src.nodes[x];
        if (n.op == PF_OP_CONST || n.shape.empty()) return;
        if (n.op == PF_OP_TRANSPOSE && src.nodes[n.in[0]].shape.size() >= 2) {
            if (!moves_no_data(n.shape)) ++n_t;
            return;
        }
        if (moves_no_data(n.shape)) return;
        if (sinkable_op(n.op) && n.shape.size() >= 2) {
            ++n_nodes;
            for (int p : n.in) free_cone(p, seen, n_nodes, n_t, ok);
            return;
        }
        ok = false;
    }

    // May reduction i (over the last dim) run as a reduction over dim -2 of its operand's transposed cone?
    bool site_possible(int i, const std::vector<std::vector<int>>& consumers) const {
        const Node& n = src.nodes[i];
        if (!is_reduction(n.op) || n.red_dim != -1) return false;
        const Node& x = src.nodes[n.in[0]];
        if (x.shape.size() < 2 || moves_no_data(x.shape)) return false;
        std::set<int> seen;
        int n_nodes = 0, n_t = 0;
        bool ok = true;
        free_cone(n.in[0], seen, n_nodes, n_t, ok);
        if (!ok || n_t < 1 || n_nodes > 24) return false;
        return readers_take_it_as_it_lies(i, consumers);
    }

    // Readers take such a result as it lies, and only elementwise ones are taught to; per-row arithmetic on it
    // comes to lie the same way, so its readers are asked in turn.
    bool readers_take_it_as_it_lies(int i, const std::vector<std::vector<int>>& consumers) const {
        for (int c : consumers[i]) {
            const Node& cn = src.nodes[c];
            if (!sinkable_op(cn.op)) return false;
            if (cn.shape.size() >= 2 && moves_no_data(cn.shape) && !readers_take_it_as_it_lies(c, consumers)) return false;
        }
        return true;
    }

    // Inside a column-reduction site a transposed leaf is read as it lies; if it is elementwise arithmetic on
    // tensors in memory, the reduction's kernel computes it again from those instead of having another kernel
    // write it out (a few levels deep at most: beyond that the value is taken from memory).
    int recomputed(int y, int depth) {
        const Node& n = src.nodes[y];
        if (!sinkable_op(n.op) || n.shape.size() < 2 || moves_no_data(n.shape) || depth >= 6) return map[y];
        // a value some kernel computes in this orientation anyway (an output, or read by more than transposes) is
        // taken from there: that kernel may well be this one
        bool elsewhere = n.is_output;
        for (int c : readers[y]) elsewhere |= src.nodes[c].op != PF_OP_TRANSPOSE && depth == 0;
        if (elsewhere) return map[y];
        auto it = pnode.find(y);
        if (it != pnode.end()) return it->second;
        Node c = n;
        c.is_output = false;
        c.orig = y;
        c.col_prologue = true;
        for (size_t k = 0; k < n.in.size(); ++k) {
            c.in[k] = recomputed(n.in[k], depth + 1);
            if (standin.count(n.in[k])) {
                c.alias_t.resize(n.in.size(), 0);
                c.alias_t[k] = 1;
            }
        }
        const int id = push(c);
        pnode[y] = id;
        return id;
    }

    Ref transposed(int x, bool top) {
        const Node& n = src.nodes[x];
        if (n.op == PF_OP_CONST || n.shape.empty()) return {map[x], false};
        if (n.op == PF_OP_TRANSPOSE && src.nodes[n.in[0]].shape.size() >= 2) return {in_site ? recomputed(n.in[0], 0) : map[n.in[0]], false};
        if (moves_no_data(n.shape)) return {map[x], standin.count(x) == 0};      // a stand-in already lies the other way
        auto it = tnode.find(x);
        if (it != tnode.end()) return {it->second, false};
        int id;
        if (sinkable_op(n.op) && n.shape.size() >= 2 && (!top || worth_sinking(x))) {
            Node c = n;
            c.is_output = false;
            c.orig = x;
            c.col_prologue = in_site;
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
                if (sites.count(store_site((int)i)) && store_through_possible((int)i)) {
                    // written by the kernel that computes the value, through that kernel's transposed store
                    Node c = n;
                    c.orig = (int)i;
                    c.in = {map[v]};
                    c.store_t = true;
                    map[i] = push(c);
                    continue;
                }
                const bool chosen = sites.count((int)i) && sinkable_op(x.op) && x.shape.size() >= 2 && !moves_no_data(x.shape);
                if (computed && x.op != PF_OP_TRANSPOSE && (worth_sinking(v) || chosen)) {
                    const Ref r = transposed(v, !chosen);
                    // the clone at the top of the cone stands for the transpose node itself
                    out.nodes[r.id].orig = (int)i;
                    out.nodes[r.id].dtype = n.dtype;
                    if (n.is_output) out.nodes[r.id].is_output = true;
                    map[i] = r.id;
                    tnode.erase(v);            // another transpose of v would be another user node
                    continue;
                }
            }
            if (taken_over.count((int)i)) {
                // computed by the kernel of a chosen transpose, in that kernel's orientation, and written through a
                // transposed store: y = transpose(transpose(y)) with the inner transpose pushed down to y's sources
                const Ref r = transposed((int)i, false);
                Node t;
                t.op = PF_OP_TRANSPOSE;
                t.dtype = n.dtype;
                t.in = {r.id};
                t.shape = n.shape;
                t.orig = (int)i;
                t.is_output = true;
                t.store_t = true;
                map[i] = push(t);
                continue;
            }
            if (sites.count((int)i) && is_reduction(n.op)) {
                // reduce(x, last dim) = reduce(transpose(x), dim -2), with transpose(x) computed from x's sources as they lie
                in_site = true;
                const Ref r = transposed(n.in[0], false);
                in_site = false;
                Node c = n;
                c.orig = (int)i;
                c.in = {r.id};
                c.alias_t.assign(1, r.alias ? 1 : 0);
                c.red_dim = -2;
                if (n.keepdim) {
                    c.shape = swapped(n.shape);
                    standin.insert((int)i);
                }
                map[i] = push(c);
                continue;
            }
            Node c = n;
            c.orig = (int)i;
            bool reads_standin = false;
            for (int p : n.in) reads_standin |= standin.count(p) != 0;
            if (reads_standin && sinkable_op(n.op) && n.shape.size() >= 2 && moves_no_data(n.shape)) {
                // arithmetic on such a result alone (one value per row, like the result): computed the way the result
                // lies, so that it can finish in the reduction's kernel; it becomes a stand-in itself
                c.shape = swapped(n.shape);
                c.alias_t.assign(n.in.size(), 0);
                for (size_t k = 0; k < n.in.size(); ++k) {
                    const Node& pn = src.nodes[n.in[k]];
                    c.alias_t[k] = (standin.count(n.in[k]) || pn.op == PF_OP_CONST || pn.shape.empty()) ? 0 : 1;
                    c.in[k] = map[n.in[k]];
                }
                standin.insert((int)i);
                map[i] = push(c);
                continue;
            }
            for (size_t k = 0; k < c.in.size(); ++k) {
                if (standin.count(c.in[k])) {          // same linear order, the last two dims named the other way round
                    c.alias_t.resize(c.in.size(), 0);
                    c.alias_t[k] = 1;
                }
                c.in[k] = map[c.in[k]];
            }
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

void sink_transposes(const pf_graph& g, const pf_options& opt, const std::vector<int>& sites, pf_graph& out) {
    Sinker s(g, opt, sites);
    s.run();
    s.prune();
    out = s.out;
}

std::vector<int> rewrite_sites(const pf_graph& g, const pf_options& opt) {
    Sinker s(g, opt);
    std::vector<std::vector<int>> consumers(g.nodes.size());
    for (size_t i = 0; i < g.nodes.size(); ++i)
        for (int p : g.nodes[i].in) consumers[p].push_back((int)i);
    std::vector<int> sites;
    for (size_t i = 0; i < g.nodes.size(); ++i)
        if (s.site_possible((int)i, consumers) || !s.outputs_to_take_over((int)i).empty()) sites.push_back((int)i);
    for (size_t i = 0; i < g.nodes.size(); ++i)
        if (s.store_through_possible((int)i)) sites.push_back(Sinker::store_site((int)i));
    return sites;
}

}  // namespace pf
