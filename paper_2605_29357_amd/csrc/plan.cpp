// Fusion planner: partitions the op-DAG into kernel groups.
//
// A fusible subgraph is a run of operators that one execution unit can absorb
// (paper Sec. 3.2, prefix analysis: an operator is fusible with its prefix when
// adding it does not add a kernel).  Here a group is a set of nodes that share
// one iteration domain D = [leading..., C]:
//   - elementwise nodes whose shape is D ("full") or D with the last dim 1
//     ("row-uniform", only inside row groups),
//   - reductions over the last dim of a full value (their result is
//     row-uniform and may be consumed inside the same kernel),
//   - transposes of tensors that already sit in memory (read through a swap of
//     the last two dims; the group then iterates in tiles), and transposes the
//     rewrite marks as results that only leave the kernel (a tiled group writes
//     them through the same LDS transpose, on the store side),
//   - reductions over the second-to-last dim of a full value (the pooling over
//     the sequence dim of the paper's Case 2) followed by an epilogue of
//     elementwise nodes on the reduced ("column-uniform") shape.
// Boundaries fall where the domain changes (a transpose of a value computed in
// the same kernel that is read again, a broadcast that grows the shape) and where a reduction
// would have to join a tiled group.  A node may join any group that does not
// come to depend on itself that way (the groups its operands live in must not
// need anything the group computes); the groups are put in execution order at
// the end.
#include <algorithm>
#include <cstring>

#include "pf_internal.h"

namespace pf {

namespace {

Shape canon(const Shape& s) {
    size_t i = 0;
    while (i < s.size() && s[i] == 1) ++i;
    return Shape(s.begin() + i, s.end());
}

Shape row_scalar_of(const Shape& d) {
    if (d.empty()) return d;
    Shape r = d;
    r.back() = 1;
    return canon(r);
}

// like canon, but keeps the two innermost dims: the domain of a reduction over dim -2
Shape canon_min2(const Shape& s) {
    size_t i = 0;
    while (i + 2 < s.size() && s[i] == 1) ++i;
    return Shape(s.begin() + i, s.end());
}

bool is_col_reduction(const Node& n) { return is_reduction(n.op) && n.red_dim == -2; }

struct Builder {
    const pf_graph& g;
    const pf_options& opt;
    std::vector<int> group_of;                  // per node, -1 = none (inputs, consts)
    std::vector<std::vector<int>> consumers;
    struct G {
        pf_template tmpl;
        Shape domain;
        std::vector<int> nodes;
        std::vector<int> kinds;                 // per member: 2 full, 1 row-uniform, 3 column-uniform, 4 stored through a transpose
        bool has_rowuni = false;
        bool has_view = false;                  // a member is, or reads through, a roll / slice
        std::vector<int> t_sources;             // tensors read through a swap of their last two dims (one LDS tile each)
        Shape epilogue;                         // COL_REDUCE: canonical shape of the column-uniform members
    };
    std::vector<int> kind_of;                   // per node, kind inside its group
    std::vector<G> groups;
    std::vector<std::vector<int>> needs;        // per group: the groups it reads values from
    bool join_earlier = true;                   // a node may join the group of any operand, not only the latest of them
    bool prologue_apart = true;                 // the prologue of a column reduction avoids flat groups a row reduction may want

    // does group a need, directly or through others, something group b computes?
    bool depends(int a, int b) const {
        std::vector<int> todo = {a};
        std::vector<char> seen(groups.size(), 0);
        while (!todo.empty()) {
            const int x = todo.back();
            todo.pop_back();
            if (x == b) return true;
            if (seen[x]) continue;
            seen[x] = 1;
            for (int y : needs[x]) todo.push_back(y);
        }
        return false;
    }
    // groups node id reads from (through a view: the group of the tensor it finally reads)
    std::vector<int> producer_groups(int id) const {
        std::vector<int> r;
        auto add = [&](int p) {
            if (group_of[p] >= 0 && std::find(r.begin(), r.end(), group_of[p]) == r.end()) r.push_back(group_of[p]);
        };
        for (int p : g.nodes[id].in) {
            add(p);
            if (is_view(g.nodes[p].op)) add(root_of(p));
        }
        if (is_view(g.nodes[id].op)) add(root_of(id));
        return r;
    }
    // would the groups still have an execution order with node id in group gi?
    bool keeps_order(int id, int gi) const {
        for (int gp : producer_groups(id))
            if (gp != gi && depends(gp, gi)) return false;
        return true;
    }

    Builder(const pf_graph& gr, const pf_options& o) : g(gr), opt(o) {
        group_of.assign(g.nodes.size(), -1);
        kind_of.assign(g.nodes.size(), 0);
        consumers.resize(g.nodes.size());
        for (size_t i = 0; i < g.nodes.size(); ++i)
            for (int p : g.nodes[i].in) consumers[p].push_back((int)i);
    }

    bool grouped(int n) const { return group_of[n] >= 0; }

    // the tensor a chain of roll / slice nodes finally reads
    int root_of(int id) const {
        while (is_view(g.nodes[id].op)) id = g.nodes[id].in[0];
        return id;
    }

    // kind of node n if it were a member of a group with domain d: 2 full, 1 row-uniform, 0 neither
    int kind_in(const Node& n, const Shape& d) const {
        Shape c = canon(n.shape);
        if (c == d) return 2;
        if (!d.empty() && d.back() > 1 && c == row_scalar_of(d) && (n.keepdim || !is_reduction(n.op))) return 1;
        return 0;
    }

    // May a member of the group be read in-kernel by a consumer?  A reduction
    // with keepdim=0 has a shape that aligns differently under broadcasting,
    // so its consumers always read it back from memory.
    // A reduction over dim -2 is only ever consumed in its kernel by nodes of its
    // own reduced shape, for which alignment is not an issue.
    bool usable_in_kernel(int p) const {
        const Node& n = g.nodes[p];
        return !(is_reduction(n.op) && !n.keepdim && n.red_dim == -1);
    }

    bool reads_view(const Node& n) const {
        if (is_view(n.op)) return true;
        for (int p : n.in)
            if (is_view(g.nodes[p].op)) return true;
        return false;
    }

    // tensors node n reads in the other orientation
    std::vector<int> transposed_reads(const Node& n) const {
        std::vector<int> t;
        if (n.op == PF_OP_TRANSPOSE) t.push_back(n.in[0]);
        for (size_t k = 0; k < n.in.size(); ++k)
            if (n.reads_alias(k)) t.push_back(n.in[k]);
        return t;
    }

    // A tiled kernel stages every transposed operand through an LDS tile of its own (4,224 bytes at the
    // narrow tile edge): twelve of them fit the 64 KB a workgroup may declare.
    static constexpr size_t kMaxTransposedOperands = 12;

    bool can_join(int id, int gi) const {
        const Node& n = g.nodes[id];
        const G& grp = groups[gi];
        if (grp.nodes.size() >= 60) return false;
        if (!keeps_order(id, gi)) return false;
        {
            size_t extra = 0;
            for (int p : transposed_reads(n))
                if (group_of[p] != gi && std::find(grp.t_sources.begin(), grp.t_sources.end(), p) == grp.t_sources.end()) ++extra;
            if (extra && grp.t_sources.size() + extra > kMaxTransposedOperands) return false;
        }
        for (int p : n.in)
            if (group_of[p] == gi && (!usable_in_kernel(p) || kind_of[p] == 4)) return false;
        // the prologue of a column reduction stays where that reduction can follow it
        if (n.col_prologue) {
            if ((grp.tmpl != PF_T_EW_FLAT && grp.tmpl != PF_T_COL_REDUCE) || grp.has_rowuni || grp.has_view) return false;
            // ... and does not take a flat group of other nodes away from a row reduction over the same domain
            // that is still to come (it could not follow them into a column-reduction kernel)
            bool others = false;
            for (int m : grp.nodes) others |= !g.nodes[m].col_prologue && !is_col_reduction(g.nodes[m]);
            if (others && prologue_apart && grp.tmpl != PF_T_COL_REDUCE)
                for (size_t r = (size_t)id + 1; r < g.nodes.size(); ++r) {
                    const Node& rn = g.nodes[r];
                    if (is_reduction(rn.op) && rn.red_dim == -1 && canon(g.nodes[rn.in[0]].shape) == grp.domain) return false;
                }
        }
        for (size_t k = 0; k < n.in.size(); ++k)               // read in the other orientation: from memory only
            if (n.reads_alias(k) && group_of[n.in[k]] == gi) return false;
        if (is_col_reduction(n)) {
            // joins a flat elementwise prologue, or further reductions of the same domain
            if (grp.tmpl != PF_T_EW_FLAT && grp.tmpl != PF_T_COL_REDUCE) return false;
            if (grp.has_view || grp.has_rowuni || grp.domain.size() < 2) return false;
            const int x = n.in[0];
            if (group_of[x] == gi && kind_of[x] != 2) return false;
            return canon(g.nodes[x].shape) == grp.domain;
        }
        if (grp.tmpl == PF_T_COL_REDUCE) {
            if (reads_view(n) || n.op == PF_OP_TRANSPOSE || is_reduction(n.op) || n.op == PF_OP_ROT_PAIRS) return false;
            bool on_reduced = false;
            for (int p : n.in)
                if (group_of[p] == gi && kind_of[p] == 3) on_reduced = true;
            if (!on_reduced) return canon(n.shape) == grp.domain;      // prologue
            // epilogue: everything it reads inside the kernel has the reduced shape, and so has the node
            if (canon(n.shape) != grp.epilogue) return false;
            for (int p : n.in)
                if (group_of[p] == gi && (kind_of[p] != 3 || canon(g.nodes[p].shape) != grp.epilogue)) return false;
            return true;
        }
        if (is_view(n.op)) {
            // read through index arithmetic from the chain's root, which must already be in memory
            if (group_of[root_of(id)] == gi) return false;
            return kind_in(n, grp.domain) == 2;
        }
        for (int p : n.in)                                    // a view operand is read from its root
            if (is_view(g.nodes[p].op) && group_of[p] != gi && group_of[root_of(p)] == gi) return false;
        if (n.op == PF_OP_TRANSPOSE && group_of[n.in[0]] == gi) {
            // The operand is computed in this kernel.  Only a result that is written out and read by nobody (the
            // rewrite marks those) can leave through a transposed store; everything else needs the value in memory.
            if (!n.store_t || !n.is_output || !consumers[id].empty()) return false;
            if (grp.tmpl != PF_T_EW_FLAT && grp.tmpl != PF_T_TILE) return false;
            if (grp.has_rowuni || grp.has_view || grp.domain.size() < 2) return false;
            const Node& x = g.nodes[n.in[0]];
            return kind_of[n.in[0]] == 2 && x.op != PF_OP_TRANSPOSE && !is_view(x.op) && canon(x.shape) == grp.domain;
        }
        if (n.op == PF_OP_TRANSPOSE) {
            if (grp.tmpl != PF_T_EW_FLAT && grp.tmpl != PF_T_TILE) return false;
            if (grp.has_rowuni) return false;
            return canon(n.shape) == grp.domain && grp.domain.size() >= 2;
        }
        if (is_reduction(n.op)) {
            if (grp.tmpl == PF_T_TILE) return false;
            for (int m : grp.nodes)
                if (g.nodes[m].col_prologue) return false;
            const Node& x = g.nodes[n.in[0]];
            return canon(x.shape) == grp.domain && !grp.domain.empty();
        }
        int k = kind_in(n, grp.domain);
        if (k == 2) {
            // every operand must broadcast *into* the domain, which holds since
            // the node's own shape is the domain
            return true;
        }
        if (k == 1) return grp.tmpl == PF_T_ROW_RESIDENT || grp.tmpl == PF_T_ROW_LOOP;   // (never holds prologue nodes: see above)
        return false;
    }

    // does a member of group gi read, from memory, a tensor that node id reads too?
    bool shares_operand(int id, int gi) const {
        for (int p : g.nodes[id].in) {
            if (g.nodes[p].op == PF_OP_CONST || group_of[p] == gi) continue;
            for (int m : groups[gi].nodes)
                for (int q : g.nodes[m].in)
                    if (q == p) return true;
        }
        return false;
    }

    void join(int id, int gi) {
        const Node& n = g.nodes[id];
        G& grp = groups[gi];
        for (int gp : producer_groups(id))
            if (gp != gi && std::find(needs[gi].begin(), needs[gi].end(), gp) == needs[gi].end()) needs[gi].push_back(gp);
        grp.nodes.push_back(id);
        group_of[id] = gi;
        const bool store_side = n.op == PF_OP_TRANSPOSE && group_of[n.in[0]] == gi;
        for (int p : transposed_reads(n))
            if (!(store_side && p == n.in[0]) && std::find(grp.t_sources.begin(), grp.t_sources.end(), p) == grp.t_sources.end())
                grp.t_sources.push_back(p);
        int k = 2;
        if (is_col_reduction(n)) {
            if (grp.tmpl != PF_T_COL_REDUCE) grp.epilogue = canon(n.shape);
            grp.tmpl = PF_T_COL_REDUCE;
            k = 3;
        } else if (grp.tmpl == PF_T_COL_REDUCE) {
            for (int p : n.in)
                if (group_of[p] == gi && kind_of[p] == 3) k = 3;
        } else if (store_side) {
            grp.tmpl = PF_T_TILE;
            k = 4;
        } else {
            if (n.op == PF_OP_TRANSPOSE) grp.tmpl = PF_T_TILE;
            if (is_reduction(n.op)) grp.tmpl = PF_T_ROW_RESIDENT;
            if (kind_in(n, grp.domain) == 1 || is_reduction(n.op)) {
                grp.has_rowuni = true;
                k = 1;
            }
            if (reads_view(n)) grp.has_view = true;
        }
        kind_of[id] = k;
        grp.kinds.push_back(k);
    }

    void seed(int id) {
        const Node& n = g.nodes[id];
        G grp;
        grp.tmpl = PF_T_EW_FLAT;
        if (is_col_reduction(n)) grp.domain = canon_min2(g.nodes[n.in[0]].shape);
        else if (is_reduction(n.op)) grp.domain = canon(g.nodes[n.in[0]].shape);
        else grp.domain = canon(n.shape);
        groups.push_back(grp);
        needs.emplace_back();
        join(id, (int)groups.size() - 1);
    }

    void run() {
        for (size_t i = 0; i < g.nodes.size(); ++i) {
            const Node& n = g.nodes[i];
            if (n.op == PF_OP_INPUT || n.op == PF_OP_CONST) continue;
            if (!opt.fuse) {
                seed((int)i);
                continue;
            }
            // first choice: the latest group an operand lives in; then the other operands' groups (a group may come
            // to run after one numbered higher, as long as no cycle arises); then any later group, preferring one
            // that already reads an operand of this node, which saves its bytes (not for a transpose: it is pure
            // data movement and belongs with its readers, which come next)
            std::vector<int> from = producer_groups((int)i);
            std::sort(from.begin(), from.end(), [](int a, int b) { return a > b; });
            const int cand = from.empty() ? -1 : from[0];
            const int last = (int)groups.size() - 1;
            int pick = -1;
            for (size_t k = 0; k < (join_earlier ? from.size() : std::min<size_t>(from.size(), 1)) && pick < 0; ++k)
                if (can_join((int)i, from[k])) pick = from[k];
            for (int gi = last; gi > cand && pick < 0 && n.op != PF_OP_TRANSPOSE; --gi)
                if (shares_operand((int)i, gi) && can_join((int)i, gi)) pick = gi;
            if (pick < 0 && last > cand && can_join((int)i, last)) pick = last;
            // still none: any group of the node's own domain that takes it saves a launch (two unrelated row
            // statistics of one tensor shape are one kernel); a transpose stays with its readers
            if (pick < 0 && join_earlier && n.op != PF_OP_TRANSPOSE && !n.col_prologue) {
                const Shape own = is_col_reduction(n) ? canon_min2(g.nodes[n.in[0]].shape)
                                  : is_reduction(n.op) ? canon(g.nodes[n.in[0]].shape) : canon(n.shape);
                for (int gi = last; gi >= 0 && pick < 0; --gi)
                    if (groups[gi].domain == own && can_join((int)i, gi)) pick = gi;
            }
            if (pick >= 0) join((int)i, pick);
            else seed((int)i);
        }
        put_in_execution_order();
    }

    // renumbers the groups so that each comes after the groups it reads from (lowest old number first among the ready ones)
    void put_in_execution_order() {
        const int n = (int)groups.size();
        std::vector<int> order, pos(n, -1);
        std::vector<char> done(n, 0);
        while ((int)order.size() < n) {
            int pick = -1;
            for (int gi = 0; gi < n && pick < 0; ++gi) {
                if (done[gi]) continue;
                bool ready = true;
                for (int y : needs[gi]) ready &= done[y] != 0;
                if (ready) pick = gi;
            }
            if (pick < 0) fail(PF_E_COMPILE, "internal: kernel groups depend on each other in a cycle");
            done[pick] = 1;
            pos[pick] = (int)order.size();
            order.push_back(pick);
        }
        std::vector<G> sorted;
        std::vector<std::vector<int>> sorted_needs;
        for (int gi : order) {
            sorted.push_back(groups[gi]);
            std::vector<int> nd;
            for (int y : needs[gi]) nd.push_back(pos[y]);
            sorted_needs.push_back(nd);
        }
        groups.swap(sorted);
        needs.swap(sorted_needs);
        for (int& go : group_of)
            if (go >= 0) go = pos[go];
    }
};

uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

}  // namespace

namespace {

void plan_with(const pf_graph& g, const pf_options& opt, bool join_earlier, bool prologue_apart, Plan& plan) {
    Builder b(g, opt);
    b.join_earlier = join_earlier;
    b.prologue_apart = prologue_apart;
    b.run();

    const size_t nn = g.nodes.size();
    // where each node's bytes live once its group has run
    std::vector<int64_t> ws_off(nn, -1);
    std::vector<pf_dtype> mem_dtype(nn, PF_F32);
    std::vector<int> input_slot(nn, -1), output_slot(nn, -1);
    for (size_t k = 0; k < g.inputs.size(); ++k) {
        input_slot[g.inputs[k]] = (int)k;
        mem_dtype[g.inputs[k]] = g.nodes[g.inputs[k]].dtype;
    }
    for (size_t k = 0; k < g.outputs.size(); ++k)
        if (output_slot[g.outputs[k]] < 0) output_slot[g.outputs[k]] = (int)k;

    uint64_t ws = 0;
    plan.groups.clear();
    plan.algorithmic_bytes = 0;
    for (int i : g.inputs) plan.algorithmic_bytes += (uint64_t)numel(g.nodes[i].shape) * itemsize(g.nodes[i].dtype);
    for (int o : g.outputs) plan.algorithmic_bytes += (uint64_t)numel(g.nodes[o].shape) * itemsize(g.nodes[o].dtype);

    for (size_t gi = 0; gi < b.groups.size(); ++gi) {
        const auto& bg = b.groups[gi];
        Group grp;
        grp.tmpl = bg.tmpl;
        grp.nodes = bg.nodes;
        grp.node_kind = bg.kinds;
        grp.domain = bg.domain;
        grp.cols = bg.domain.empty() ? 1 : bg.domain.back();
        grp.rows = 1;
        for (size_t d = 0; d + 1 < bg.domain.size(); ++d) grp.rows *= bg.domain[d];
        const int rd = (int)bg.domain.size();

        // external reads
        // Column-uniform members line up with the domain minus its dim -2; an operand
        // of theirs gets stride 0 there.  `epi_keep`: they carry that dim with size 1.
        const bool is_col = bg.tmpl == PF_T_COL_REDUCE;
        Shape dom_keep = bg.domain, dom_drop = bg.domain;
        bool epi_keep = true;
        if (is_col) {
            dom_keep[rd - 2] = 1;
            dom_drop.erase(dom_drop.begin() + (rd - 2));
            epi_keep = bg.epilogue == canon(dom_keep);
            if (!epi_keep && bg.epilogue != canon(dom_drop)) fail(PF_E_COMPILE, "internal: epilogue shape of a column reduction");
        }
        auto add_operand = [&](int p, bool transposed, bool coluni = false) {
            for (auto& o : grp.operands)
                if (o.node == p && o.via_transpose == transposed && o.coluni == coluni) return;
            Operand o;
            o.node = p;
            o.coluni = coluni;
            o.transposed = transposed;
            o.via_transpose = transposed;
            o.shape = g.nodes[p].shape;
            if (input_slot[p] >= 0) {
                o.graph_input = input_slot[p];
                o.dtype = g.nodes[p].dtype;
            } else if (ws_off[p] >= 0) {
                o.ws_offset = ws_off[p];
                o.dtype = mem_dtype[p];
            } else if (output_slot[p] >= 0) {
                o.graph_output = output_slot[p];
                o.dtype = g.nodes[p].dtype;
            } else {
                fail(PF_E_COMPILE, "internal: node %%%d read before it is materialised", p);
            }
            Shape s = canon(o.shape);
            if (transposed) {
                // the operand as seen after swapping its last two dims
                Shape t = g.nodes[p].shape;
                if (t.size() < 2) t.insert(t.begin(), 2 - t.size(), 1);
                std::swap(t[t.size() - 1], t[t.size() - 2]);
                Shape tc = canon(t);
                const int64_t r_o = t[t.size() - 2], c_o = t[t.size() - 1];
                if (r_o == 1 || c_o == 1 || (int)tc.size() < 2) {
                    // no data movement: same linear order
                    s = tc;
                    o.transposed = false;
                } else {
                    if ((int)tc.size() != rd) fail(PF_E_COMPILE, "internal: transposed operand rank");
                    int64_t st = r_o * c_o;
                    for (int k = rd - 3; k >= 0; --k) {
                        o.stride[k] = tc[k] == 1 ? 0 : st;
                        st *= tc[k];
                    }
                    o.stride[rd - 2] = 1;
                    o.stride[rd - 1] = r_o;
                    grp.operands.push_back(o);
                    return;
                }
            }
            if (coluni && !epi_keep) {
                // right-align against the domain without dim -2, then skip over that dim
                const int re = rd - 1;
                if ((int)s.size() > re) fail(PF_E_COMPILE, "internal: operand %%%d rank exceeds the reduced domain", p);
                int64_t st = 1;
                for (int j = (int)s.size() - 1; j >= 0; --j) {
                    const int ke = re - ((int)s.size() - j);
                    if (s[j] != 1 && s[j] != dom_drop[ke])
                        fail(PF_E_COMPILE, "internal: operand %%%d does not broadcast into the reduced domain", p);
                    o.stride[ke < rd - 2 ? ke : rd - 1] = s[j] == 1 ? 0 : st;
                    st *= s[j];
                }
                grp.operands.push_back(o);
                return;
            }
            const Shape& dom = coluni ? dom_keep : bg.domain;
            if ((int)s.size() > rd) fail(PF_E_COMPILE, "internal: operand %%%d rank exceeds domain", p);
            int64_t st = 1;
            for (int j = (int)s.size() - 1; j >= 0; --j) {
                int k = rd - ((int)s.size() - j);
                if (s[j] != 1 && s[j] != dom[k])
                    fail(PF_E_COMPILE, "internal: operand %%%d does not broadcast into the domain", p);
                o.stride[k] = s[j] == 1 ? 0 : st;
                st *= s[j];
            }
            grp.operands.push_back(o);
        };
        // a tensor read through a chain of roll / slice nodes ending in node v
        auto add_view_operand = [&](int v) {
            for (auto& o : grp.operands)
                if (o.view == v) return;
            const int root = b.root_of(v);
            Operand o;
            o.node = root;
            o.view = v;
            o.shape = g.nodes[v].shape;              // the window that is read
            if (input_slot[root] >= 0) {
                o.graph_input = input_slot[root];
                o.dtype = g.nodes[root].dtype;
            } else if (ws_off[root] >= 0) {
                o.ws_offset = ws_off[root];
                o.dtype = mem_dtype[root];
            } else if (output_slot[root] >= 0) {
                o.graph_output = output_slot[root];
                o.dtype = g.nodes[root].dtype;
            } else {
                fail(PF_E_COMPILE, "internal: node %%%d read through a view before it is materialised", root);
            }
            const Shape& rs = g.nodes[root].shape;
            const Shape& vs = g.nodes[v].shape;
            const int r = (int)rs.size();
            // steps per source dim, in the order they apply to the consumer's index (v back to the root)
            std::vector<std::vector<ViewStep>> steps(r);
            for (int cur = v; is_view(g.nodes[cur].op); cur = g.nodes[cur].in[0]) {
                const Node& vn = g.nodes[cur];
                ViewStep st;
                if (vn.op == PF_OP_SLICE) {
                    st.add = vn.start;
                } else {
                    const int64_t size = g.nodes[vn.in[0]].shape[vn.dim];
                    int64_t sh = vn.shift % size;
                    if (sh < 0) sh += size;
                    st.add = (size - sh) % size;
                    st.mod = size;
                }
                if (st.add || st.mod) steps[vn.dim].push_back(st);
            }
            int64_t stride = 1;
            for (int d = r - 1; d >= 0; --d) {
                const int k = rd - (r - d);           // domain dim this source dim lines up with
                const bool iterated = k >= 0 && vs[d] != 1;
                if (iterated) {
                    if (vs[d] != bg.domain[k]) fail(PF_E_COMPILE, "internal: view operand %%%d does not fit the domain", v);
                    o.stride[k] = stride;
                    o.steps[k] = steps[d];
                } else {
                    if (vs[d] != 1) fail(PF_E_COMPILE, "internal: view operand %%%d rank exceeds domain", v);
                    int64_t idx = 0;                  // the window has one element here: a constant source index
                    for (auto& st : steps[d]) idx = st.mod ? (idx + st.add) % st.mod : idx + st.add;
                    o.const_offset += idx * stride;
                }
                stride *= rs[d];
            }
            grp.operands.push_back(o);
        };
        for (size_t m = 0; m < bg.nodes.size(); ++m) {
            const int id = bg.nodes[m];
            const Node& n = g.nodes[id];
            if (is_view(n.op)) {
                add_view_operand(id);
                continue;
            }
            if (bg.kinds[m] == 4) continue;            // reads nothing: its operand sits in registers
            const bool epilogue_node = is_col && bg.kinds[m] == 3 && !is_reduction(n.op);
            for (size_t k = 0; k < n.in.size(); ++k) {
                const int p = n.in[k];
                if (g.nodes[p].op == PF_OP_CONST) continue;
                bool inside = b.group_of[p] == (int)gi && b.usable_in_kernel(p);
                if (n.op == PF_OP_TRANSPOSE || n.reads_alias(k)) add_operand(p, true, epilogue_node && n.op != PF_OP_TRANSPOSE);
                else if (inside) continue;
                else if (is_view(g.nodes[p].op)) add_view_operand(p);
                else add_operand(p, false, epilogue_node);
            }
        }

        // writes: members that are graph outputs or read by another kernel
        for (size_t m = 0; m < bg.nodes.size(); ++m) {
            const int id = bg.nodes[m];
            const Node& n = g.nodes[id];
            if (bg.kinds[m] == 4) {
                Store s;
                s.node = id;
                s.value_node = n.in[0];
                s.tstore = true;
                s.dtype = n.dtype;
                s.shape = n.shape;
                s.graph_output = output_slot[id];
                for (size_t k = 0; k < g.outputs.size(); ++k)
                    if (g.outputs[k] == id && (int)k != output_slot[id]) s.also_outputs.push_back((int)k);
                grp.stores.push_back(s);
                mem_dtype[id] = n.dtype;
                continue;
            }
            bool outside_use = false;
            for (int c : b.consumers[id]) {
                const pf_op cop = g.nodes[c].op;
                if (is_view(n.op)) {
                    // readers of a view go to its root, except a transpose, which needs the window in memory
                    if (cop == PF_OP_TRANSPOSE) outside_use = true;
                    continue;
                }
                const bool stored_through = cop == PF_OP_TRANSPOSE && b.group_of[c] == (int)gi && b.kind_of[c] == 4;    // leaves from registers
                if (b.group_of[c] != (int)gi || !b.usable_in_kernel(id) || (cop == PF_OP_TRANSPOSE && !stored_through) || is_view(cop)) outside_use = true;
                for (size_t k = 0; k < g.nodes[c].in.size(); ++k)
                    if (g.nodes[c].in[k] == id && g.nodes[c].reads_alias(k)) outside_use = true;
            }
            // anything downstream of a view chain rooted here reads this node from memory
            if (!is_view(n.op))
                for (size_t q = 0; q < g.nodes.size() && !outside_use; ++q)
                    if (is_view(g.nodes[q].op) && b.root_of((int)q) == id) outside_use = true;
            if (!n.is_output && !outside_use) continue;
            const bool col_uniform = is_col && bg.kinds[m] == 3;
            const bool row_scalar = !is_col && (is_reduction(n.op) || (b.kind_in(n, bg.domain) == 1));
            if (n.is_output) {
                Store s;
                s.node = id;
                s.dtype = n.dtype;
                s.shape = n.shape;
                s.row_scalar = row_scalar;
                s.col_uniform = col_uniform;
                s.graph_output = output_slot[id];
                for (size_t k = 0; k < g.outputs.size(); ++k)
                    if (g.outputs[k] == id && (int)k != output_slot[id]) s.also_outputs.push_back((int)k);
                grp.stores.push_back(s);
                mem_dtype[id] = n.dtype;
            }
            // Later kernels read a value in fp32 (a second copy beside a 16-bit output: averaging the rounded values of
            // an output instead fails the tolerance where the average nearly cancels), unless every reader is a
            // transpose that is a graph output of this node's own 16-bit dtype: rounding before or after the move gives
            // the same bits.
            bool only_moved = n.dtype != PF_F32 && n.dtype != PF_F64;
            for (int c : b.consumers[id]) {
                const Node& cn = g.nodes[c];
                if (b.group_of[c] == (int)gi && b.usable_in_kernel(id) && cn.op != PF_OP_TRANSPOSE && !is_view(cn.op)) continue;   // reads it in-kernel
                // (a transpose that is a graph output and nothing else: no arithmetic ever sees the moved value)
                if (cn.op != PF_OP_TRANSPOSE || cn.dtype != n.dtype || !cn.is_output || !b.consumers[c].empty()) only_moved = false;
            }
            const bool need_ws = outside_use && (!n.is_output || (opt.intermediates_f32 && n.dtype != PF_F32 && !only_moved));
            if (need_ws) {
                Store s;
                s.node = id;
                s.dtype = (opt.intermediates_f32 && !only_moved) ? PF_F32 : n.dtype;
                s.shape = n.shape;
                s.row_scalar = row_scalar;
                s.col_uniform = col_uniform;
                s.ws_offset = (int64_t)ws;
                ws_off[id] = (int64_t)ws;
                mem_dtype[id] = s.dtype;
                ws = align_up(ws + (uint64_t)numel(n.shape) * itemsize(s.dtype), 256);
                grp.stores.push_back(s);
            }
        }
        if (grp.stores.empty()) continue;   // dead code: nothing observes this group
        if (is_col) {
            // will the kernel generator split the rows over workgroups (few column tiles, many rows)?  Then the
            // group is two launches.  (The same test as in the column-reduction template, on the default tiling.)
            int min_item = 4;
            for (auto& o : grp.operands)
                if (!o.coluni && o.stride[rd - 1] != 0) min_item = std::min(min_item, itemsize(o.dtype));
            for (auto& st : grp.stores)
                if (!st.col_uniform) min_item = std::min(min_item, itemsize(st.dtype));
            const int64_t S = bg.domain[rd - 2], DD = bg.domain[rd - 1];
            int64_t lead = 1;
            for (int k = 0; k < rd - 2; ++k) lead *= bg.domain[k];
            int vec = 16 / min_item;
            while (vec > 1 && vec > DD) vec >>= 1;
            const int64_t vcols = (DD + vec - 1) / vec;
            int tx = 1;
            while (tx < 16 && tx < vcols) tx <<= 1;
            bool any_var = false;
            for (int id : bg.nodes) any_var |= g.nodes[id].op == PF_OP_VAR;
            if (lead * ((vcols + tx - 1) / tx) < 128 && S >= 8 * (1024 / tx) && !any_var) grp.extra_launches = 1;
        }
        for (auto& o : grp.operands) grp.bytes_read += (uint64_t)numel(o.shape) * itemsize(o.dtype);
        for (auto& s : grp.stores)
            grp.bytes_written += (uint64_t)numel(s.shape) * itemsize(s.dtype) * (1 + s.also_outputs.size());
        plan.groups.push_back(std::move(grp));
    }
    plan.workspace_bytes = ws;
}

}  // namespace

uint64_t plan_cost(const Plan& plan) {
    uint64_t c = 0;
    for (auto& grp : plan.groups) {
        // Bytes that cross an LDS transpose move slower than streamed ones, the more so the more tensors a tile
        // kernel stages (measured on 100 - 200 MB kernels: one staged tensor 5.0 - 5.3 TB/s against 6.4 for a flat
        // kernel, four 4.6 TB/s, eight 3.2 TB/s, where four and more no longer fit 64-wide tiles in 64 KB of LDS)
        int staged = 0;
        for (auto& o : grp.operands) staged += o.transposed ? 1 : 0;
        for (auto& st : grp.stores) staged += st.tstore ? 1 : 0;
        const double f = staged == 0 ? 1.0 : std::max(1.2, 0.8 + 0.15 * staged);
        c += (uint64_t)((double)(grp.bytes_read + grp.bytes_written) * f) + kLaunchCostBytes * (uint64_t)(1 + grp.extra_launches);
    }
    return c;
}

void make_plan(const pf_graph& g, const pf_options& opt, Plan& plan) {
    if (g.outputs.empty()) fail(PF_E_COMPILE, "graph has no outputs");
    for (int o : g.outputs)
        if (g.nodes[o].op == PF_OP_INPUT) fail(PF_E_COMPILE, "output %%%d is a graph input; nothing to compute", o);
    // The grouping is greedy, so no way of choosing a node's group is always ahead: letting it join the group of any
    // of its operands saves a kernel or a round trip in most graphs and costs one in a few, and so does keeping the
    // prologue of a column reduction out of flat groups.  Plan each way, keep the cheapest.
    plan_with(g, opt, true, true, plan);
    if (!opt.fuse) return;
    bool any_prologue = false;
    for (auto& n : g.nodes) any_prologue |= n.col_prologue;
    for (int policy = 1; policy < 4; ++policy) {
        if ((policy & 2) && !any_prologue) continue;
        Plan other;
        plan_with(g, opt, !(policy & 1), !(policy & 2), other);
        if (plan_cost(other) < plan_cost(plan)) plan = std::move(other);
    }
}

}  // namespace pf
