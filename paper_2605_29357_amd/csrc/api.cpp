// The C boundary.  Every entry point catches, records the message in a
// thread-local string and returns a pf_status.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <memory>
#include <new>
#include <set>

#include "exec.h"
#include "pf_internal.h"
#include "metric.h"
#include "score_dev.h"

namespace {

thread_local std::string g_last_error;

template <typename F>
pf_status guarded(F&& f) {
    try {
        f();
        return PF_OK;
    } catch (const pf::Error& e) {
        g_last_error = e.what();
        return e.status;
    } catch (const std::bad_alloc&) {
        g_last_error = "out of host memory";
        return PF_E_NOMEM;
    } catch (const std::exception& e) {
        g_last_error = e.what();
        return PF_E_INVALID;
    }
}

void need(const void* p, const char* what) {
    if (!p) pf::fail(PF_E_INVALID, "%s is NULL", what);
}

pf_status copy_out(const std::string& s, char* buf, size_t cap, size_t* needed) {
    if (needed) *needed = s.size() + 1;
    if (buf && cap) {
        size_t n = s.size() < cap - 1 ? s.size() : cap - 1;
        memcpy(buf, s.data(), n);
        buf[n] = '\0';
        if (n < s.size()) {
            g_last_error = "buffer too small";
            return PF_E_INVALID;
        }
    }
    return PF_OK;
}

}  // namespace

extern "C" {

const char* pf_last_error(void) { return g_last_error.c_str(); }
const char* pf_version(void) { return "pf 0.1 (gfx950)"; }

pf_status pf_graph_create(pf_graph** g) {
    return guarded([&] {
        need(g, "g");
        *g = new pf_graph();
    });
}

void pf_graph_destroy(pf_graph* g) { delete g; }

pf_status pf_graph_input(pf_graph* g, pf_dtype dtype, int rank, const int64_t* h_shape, int* node_out) {
    return guarded([&] {
        need(g, "g");
        if (rank < 0 || rank > PF_MAX_RANK) pf::fail(PF_E_COMPILE, "rank %d out of range", rank);
        if (rank) need(h_shape, "h_shape");
        int id = pf::graph_add_input(*g, dtype, pf::Shape(h_shape, h_shape + rank));
        if (node_out) *node_out = id;
    });
}

pf_status pf_graph_node(pf_graph* g, pf_op op, const int* h_in_nodes, int n_in, const pf_attr* h_attrs, int n_attr,
                        pf_dtype out_dtype, int* node_out) {
    return guarded([&] {
        need(g, "g");
        if (n_in < 0 || n_in > 2) pf::fail(PF_E_COMPILE, "operators take at most two operands");
        if (n_in) need(h_in_nodes, "h_in_nodes");
        if (n_attr < 0) pf::fail(PF_E_INVALID, "n_attr < 0");
        if (n_attr) need(h_attrs, "h_attrs");
        std::vector<std::pair<std::string, std::string>> attrs;
        for (int i = 0; i < n_attr; ++i) {
            need(h_attrs[i].key, "attr key");
            need(h_attrs[i].value, "attr value");
            attrs.emplace_back(h_attrs[i].key, h_attrs[i].value);
        }
        int id = pf::graph_add_node(*g, op, std::vector<int>(h_in_nodes, h_in_nodes + n_in), attrs, out_dtype);
        if (node_out) *node_out = id;
    });
}

pf_status pf_graph_output(pf_graph* g, int node) {
    return guarded([&] {
        need(g, "g");
        pf::graph_add_output(*g, node);
    });
}

pf_status pf_graph_parse(const char* h_text, size_t len, pf_graph** g) {
    return guarded([&] {
        need(h_text, "h_text");
        need(g, "g");
        *g = nullptr;
        pf_graph* ng = new pf_graph();
        try {
            pf::graph_parse(std::string(h_text, len), *ng);
        } catch (...) {
            delete ng;
            throw;
        }
        *g = ng;
    });
}

pf_status pf_graph_variant(const pf_graph* g, const int* h_ranks, const int64_t* h_shapes, int from_dtype, int to_dtype,
                           pf_graph** out) {
    return guarded([&] {
        need(g, "g");
        need(out, "out");
        *out = nullptr;
        if (!g->inputs.empty()) {
            need(h_ranks, "h_ranks");
            need(h_shapes, "h_shapes");
        }
        if ((from_dtype < 0) != (to_dtype < 0)) pf::fail(PF_E_INVALID, "from_dtype and to_dtype must both be given or both be -1");
        for (int d : {from_dtype, to_dtype})
            if (d >= 0 && d != PF_F32 && d != PF_BF16 && d != PF_F16) pf::fail(PF_E_INVALID, "dtype %d is not a tensor dtype", d);
        pf_graph* ng = new pf_graph();
        try {
            pf::graph_variant(*g, h_ranks, h_shapes, from_dtype, to_dtype, *ng);
        } catch (...) {
            delete ng;
            throw;
        }
        *out = ng;
    });
}

pf_status pf_graph_print(const pf_graph* g, char* h_buf, size_t cap, size_t* needed) {
    pf_status st = PF_OK;
    pf_status outer = guarded([&] {
        need(g, "g");
        st = copy_out(pf::graph_print(*g), h_buf, cap, needed);
    });
    return outer != PF_OK ? outer : st;
}

pf_status pf_graph_size(const pf_graph* g, int* n_nodes, int* n_inputs, int* n_outputs) {
    return guarded([&] {
        need(g, "g");
        if (n_nodes) *n_nodes = (int)g->nodes.size();
        if (n_inputs) *n_inputs = (int)g->inputs.size();
        if (n_outputs) *n_outputs = (int)g->outputs.size();
    });
}

pf_status pf_graph_node_info(const pf_graph* g, int node, pf_node_info* h_info) {
    return guarded([&] {
        need(g, "g");
        need(h_info, "h_info");
        if (node < 0 || node >= (int)g->nodes.size()) pf::fail(PF_E_INVALID, "node %d out of range", node);
        const pf::Node& n = g->nodes[node];
        memset(h_info, 0, sizeof *h_info);
        h_info->op = n.op;
        h_info->dtype = n.dtype;
        h_info->rank = (int)n.shape.size();
        for (size_t i = 0; i < n.shape.size(); ++i) h_info->shape[i] = n.shape[i];
        h_info->n_in = (int)n.in.size();
        for (size_t i = 0; i < n.in.size() && i < 2; ++i) h_info->in_nodes[i] = n.in[i];
        h_info->is_output = n.is_output ? 1 : 0;
    });
}

void pf_options_default(pf_options* h_opt) {
    if (!h_opt) return;
    memset(h_opt, 0, sizeof *h_opt);
    h_opt->fuse = 1;
    h_opt->intermediates_f32 = 1;
}

pf_status pf_compile(const pf_graph* g, const pf_options* h_opt, pf_exec** e) {
    return guarded([&] {
        need(g, "g");
        need(e, "e");
        *e = nullptr;
        pf_options opt;
        pf_options_default(&opt);
        if (h_opt) opt = *h_opt;
        for (int r : opt.reserved)
            if (r) pf::fail(PF_E_INVALID, "pf_options.reserved must be zero");
        std::unique_ptr<pf_exec> ex(new pf_exec());
        ex->opt = opt;
        // Fused plans work on a rewritten copy (transposes of computed values pushed down to the operands).  The
        // rewrite has optional parts, its sites: reductions that could run in their sources' orientation instead of
        // behind a transpose, and transposes whose kernel could take over the results of the kernel before it.  Plan
        // with none, with all, and with each toggled in turn, and keep what the traffic model prefers.
        std::vector<int> best;
        if (opt.fuse) {
            const std::vector<int> sites = pf::rewrite_sites(*g, opt);
            auto cost_of = [&](const std::vector<int>& chosen) -> uint64_t {
                try {
                    pf_graph w;
                    pf::Plan p;
                    pf::sink_transposes(*g, opt, chosen, w);
                    pf::make_plan(w, opt, p);
                    return pf::plan_cost(p);
                } catch (const pf::Error&) {
                    return ~uint64_t(0);        // this choice does not plan: any other is cheaper
                }
            };
            if (!sites.empty()) {
                uint64_t best_cost = cost_of(best);
                const uint64_t all_cost = cost_of(sites);
                if (all_cost < best_cost) { best = sites; best_cost = all_cost; }
                for (int s : sites) {              // one site at a time, from whichever end is ahead
                    std::vector<int> trial = best;
                    auto it = std::find(trial.begin(), trial.end(), s);
                    if (it == trial.end()) trial.push_back(s);
                    else trial.erase(it);
                    std::sort(trial.begin(), trial.end());
                    const uint64_t c = cost_of(trial);
                    if (c < best_cost) { best = trial; best_cost = c; }
                }
            }
        }
        auto build = [&](const std::vector<int>& chosen) {
            pf_graph work;
            if (opt.fuse) pf::sink_transposes(*g, opt, chosen, work);
            else work = *g;
            ex->plan = pf::Plan();
            pf::make_plan(work, opt, ex->plan);
            int idx = 0;
            for (auto& grp : ex->plan.groups) {
                for (int id : grp.nodes) {
                    const int user = opt.fuse ? work.nodes[id].orig : id;
                    if (user >= 0) grp.user_nodes.push_back(user);
                }
                size_t n_args = grp.operands.size() + 2;
                for (auto& st : grp.stores) n_args += 1 + st.also_outputs.size();
                if (n_args > (size_t)pf::kMaxKernelArgs)
                    pf::fail(PF_E_COMPILE, "a fused group would take %zu kernel arguments (limit %d)", n_args, pf::kMaxKernelArgs);
                pf::generate_source(work, opt, grp, idx++);
                if (grp.grid > 0x7fffffffLL || grp.grid2 > 0x7fffffffLL)
                    pf::fail(PF_E_COMPILE, "kernel %s would need %lld workgroups; a launch holds at most 2^31 - 1", grp.kernel_name.c_str(),
                             (long long)std::max(grp.grid, grp.grid2));
                if (grp.scratch_bytes) {     // partial results of a split reduction live at the end of the workspace
                    const uint64_t at = (ex->plan.workspace_bytes + 255) / 256 * 256;
                    grp.scratch_offset = (int64_t)at;
                    ex->plan.workspace_bytes = at + grp.scratch_bytes;
                    grp.bytes_written += grp.scratch_bytes;
                    grp.bytes_read += grp.scratch_bytes;
                }
            }
            // Two kernels of a plan that do not depend on each other, directly or through others, need not be two
            // launches: the smaller one rides on the other (attach_rider) wherever the merged kernel can stand in
            // the execution order - after everything either of them reads, before everything that reads either.
            if (opt.fuse) {
                auto& groups = ex->plan.groups;
                struct Touch {
                    std::set<int> reads, writes;       // nodes read from memory other kernels wrote; nodes written
                };
                auto touch_of = [&](const pf::Group& grp) {
                    Touch t;
                    auto add = [&](const std::vector<pf::Operand>& ops, const std::vector<pf::Store>& sts) {
                        for (auto& o : ops)
                            if (o.graph_input < 0) t.reads.insert(o.node);
                        for (auto& st : sts) t.writes.insert(st.node);
                    };
                    add(grp.operands, grp.stores);
                    for (auto& rd : grp.riders) add(rd.operands, rd.stores);
                    return t;
                };
                auto needs = [](const Touch& b, const Touch& a) {          // does b read something a writes?
                    for (int n : b.reads)
                        if (a.writes.count(n)) return true;
                    return false;
                };
                for (bool again = true; again && groups.size() > 1;) {
                    again = false;
                    const size_t n = groups.size();
                    std::vector<Touch> tch;
                    for (auto& grp : groups) tch.push_back(touch_of(grp));
                    // reach[b][a]: b needs a, directly or through others (the groups are in execution order)
                    std::vector<std::vector<char>> reach(n, std::vector<char>(n, 0));
                    for (size_t b = 0; b < n; ++b)
                        for (size_t a = 0; a < b; ++a)
                            if (needs(tch[b], tch[a])) {
                                reach[b][a] = 1;
                                for (size_t c = 0; c < a; ++c) reach[b][c] |= reach[a][c];
                            }
                    std::vector<size_t> order(n);
                    for (size_t k = 0; k < n; ++k) order[k] = k;
                    std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return groups[a].grid < groups[b].grid; });
                    // the smallest kernel first, onto the largest kernel that takes it
                    for (size_t oi = 0; oi < n && !again; ++oi) {
                        const size_t r = order[oi];
                        if (!groups[r].riders.empty()) continue;
                        for (auto it = order.rbegin(); it != order.rend() && !again; ++it) {
                            const size_t h = *it;
                            if (h == r || reach[r][h] || reach[h][r]) continue;
                            // the host is the larger of the two, or the one with the larger workgroups
                            if (groups[h].block < groups[r].block || (groups[h].block == groups[r].block && groups[h].grid < groups[r].grid)) continue;
                            // where may the merged kernel stand?  At the later of the two places if nothing in between
                            // reads the earlier one; at the earlier if the later one reads nothing in between.
                            const size_t lo = std::min(r, h), hi = std::max(r, h);
                            bool at_hi = true, at_lo = true;
                            for (size_t k = lo + 1; k < hi; ++k) {
                                at_hi &= !reach[k][lo];
                                at_lo &= !reach[hi][k];
                            }
                            if (!at_hi && !at_lo) continue;
                            size_t n_args = groups[h].operands.size() + groups[r].operands.size() + 2;
                            for (auto& st : groups[h].stores) n_args += 1 + st.also_outputs.size();
                            for (auto& st : groups[r].stores) n_args += 1 + st.also_outputs.size();
                            for (auto& rd : groups[h].riders) {
                                n_args += rd.operands.size();
                                for (auto& st : rd.stores) n_args += 1 + st.also_outputs.size();
                            }
                            if (n_args > (size_t)pf::kMaxKernelArgs) continue;
                            if (!pf::attach_rider(groups[h], groups[r])) continue;
                            again = true;
                            pf::Group merged = std::move(groups[h]);
                            const size_t place = at_hi ? hi : lo;
                            // rebuild the order: everything but the two, with the merged kernel where it may stand
                            std::vector<pf::Group> next;
                            for (size_t k = 0; k < n; ++k) {
                                if (k == place) next.push_back(std::move(merged));
                                else if (k != r && k != h) next.push_back(std::move(groups[k]));
                            }
                            groups.swap(next);
                        }
                    }
                }
            }
            for (auto& grp : ex->plan.groups) pf::jit_compile(grp);
        };
        try {
            build(best);
        } catch (const pf::Error&) {
            // a limit of the kernel generator (kernel arguments, LDS) that the plain rewrite may stay within
            if (best.empty()) throw;
            build({});
        }
        ex->n_inputs = (int)g->inputs.size();
        ex->n_outputs = (int)g->outputs.size();
        for (int i : g->inputs) ex->input_bytes.push_back((uint64_t)pf::numel(g->nodes[i].shape) * pf::itemsize(g->nodes[i].dtype));
        for (int o : g->outputs) ex->output_bytes.push_back((uint64_t)pf::numel(g->nodes[o].shape) * pf::itemsize(g->nodes[o].dtype));
        *e = ex.release();
    });
}

void pf_exec_destroy(pf_exec* e) {
    if (!e) return;
    pf::exec_unload(*e);
    delete e;
}

pf_status pf_exec_info(const pf_exec* e, pf_plan_info* h_info) {
    return guarded([&] {
        need(e, "e");
        need(h_info, "h_info");
        memset(h_info, 0, sizeof *h_info);
        h_info->n_groups = (int)e->plan.groups.size();
        h_info->reserved_ = 0;
        h_info->n_kernels = 0;
        for (auto& grp : e->plan.groups) h_info->n_kernels += grp.kernel2_name.empty() ? 1 : 2;
        h_info->n_inputs = e->n_inputs;
        h_info->n_outputs = e->n_outputs;
        h_info->algorithmic_bytes = e->plan.algorithmic_bytes;
        h_info->workspace_bytes = e->plan.workspace_bytes;
        for (auto& grp : e->plan.groups) h_info->planned_bytes += grp.bytes_read + grp.bytes_written;
    });
}

pf_status pf_exec_group_info(const pf_exec* e, int group, pf_group_info* h_info) {
    return guarded([&] {
        need(e, "e");
        need(h_info, "h_info");
        if (group < 0 || group >= (int)e->plan.groups.size()) pf::fail(PF_E_INVALID, "group %d out of range", group);
        const pf::Group& grp = e->plan.groups[group];
        memset(h_info, 0, sizeof *h_info);
        h_info->tmpl = grp.tmpl;
        h_info->n_nodes = (int)std::min<size_t>(grp.user_nodes.size(), 64);
        for (size_t i = 0; i < grp.user_nodes.size() && i < 64; ++i) h_info->nodes[i] = grp.user_nodes[i];
        h_info->rows = grp.rows;
        h_info->cols = grp.cols;
        h_info->block_threads = grp.block;
        h_info->grid_blocks = grp.grid;
        h_info->lanes_per_row = grp.lanes_per_row;
        h_info->bytes_read = grp.bytes_read;
        h_info->bytes_written = grp.bytes_written;
    });
}

pf_status pf_exec_source(const pf_exec* e, int group, char* h_buf, size_t cap, size_t* needed) {
    pf_status st = PF_OK;
    pf_status outer = guarded([&] {
        need(e, "e");
        if (group < 0 || group >= (int)e->plan.groups.size()) pf::fail(PF_E_INVALID, "group %d out of range", group);
        st = copy_out(e->plan.groups[group].source, h_buf, cap, needed);
    });
    return outer != PF_OK ? outer : st;
}

pf_status pf_exec_kernel_name(const pf_exec* e, int group, char* h_buf, size_t cap, size_t* needed) {
    pf_status st = PF_OK;
    pf_status outer = guarded([&] {
        need(e, "e");
        if (group < 0 || group >= (int)e->plan.groups.size()) pf::fail(PF_E_INVALID, "group %d out of range", group);
        st = copy_out(e->plan.groups[group].kernel_name, h_buf, cap, needed);
    });
    return outer != PF_OK ? outer : st;
}

pf_status pf_jit_stats_get(pf_jit_stats* h_out) {
    return guarded([&] {
        need(h_out, "h_out");
        pf::jit_stats(h_out);
    });
}

static void check_execute_args(pf_exec* e, const void* const* d_inputs, int n_in, void* const* d_outputs, int n_out,
                               void* d_workspace, size_t workspace_bytes) {
    need(e, "e");
    if (n_in != e->n_inputs) pf::fail(PF_E_RUNTIME, "expected %d input buffers, got %d", e->n_inputs, n_in);
    if (n_out != e->n_outputs) pf::fail(PF_E_RUNTIME, "expected %d output buffers, got %d", e->n_outputs, n_out);
    if (n_in) need(d_inputs, "d_inputs");
    need(d_outputs, "d_outputs");
    for (int i = 0; i < n_in; ++i) {
        if (!d_inputs[i]) pf::fail(PF_E_RUNTIME, "input buffer %d is NULL", i);
        if ((uintptr_t)d_inputs[i] & 15) pf::fail(PF_E_INVALID, "input buffer %d is not 16-byte aligned", i);
    }
    for (int i = 0; i < n_out; ++i) {
        if (!d_outputs[i]) pf::fail(PF_E_RUNTIME, "output buffer %d is NULL", i);
        if ((uintptr_t)d_outputs[i] & 15) pf::fail(PF_E_INVALID, "output buffer %d is not 16-byte aligned", i);
    }
    if (e->plan.workspace_bytes) {
        if (!d_workspace || workspace_bytes < e->plan.workspace_bytes)
            pf::fail(PF_E_RUNTIME, "workspace of %llu bytes needed, %zu given", (unsigned long long)e->plan.workspace_bytes,
                     workspace_bytes);
        if ((uintptr_t)d_workspace & 255) pf::fail(PF_E_INVALID, "workspace is not 256-byte aligned");
    }
}

pf_status pf_execute(pf_exec* e, const void* const* d_inputs, int n_in, void* const* d_outputs, int n_out, void* d_workspace,
                     size_t workspace_bytes, void* stream) {
    return guarded([&] {
        check_execute_args(e, d_inputs, n_in, d_outputs, n_out, d_workspace, workspace_bytes);
        pf::exec_run(*e, d_inputs, d_outputs, d_workspace, stream, nullptr, nullptr);
    });
}

pf_status pf_execute_outer(pf_exec* e, int64_t outer_extent, const void* const* d_inputs, int n_in, void* const* d_outputs, int n_out,
                           void* stream) {
    return guarded([&] {
        need(e, "e");
        if (e->plan.groups.size() != 1 || e->plan.workspace_bytes != 0)
            pf::fail(PF_E_INVALID, "another outermost extent needs a subgraph that is one kernel without scratch");
        const pf::Group& grp = e->plan.groups[0];
        if (grp.rt_per_block <= 0 || grp.domain.size() < 2)
            pf::fail(PF_E_INVALID, "this kernel is specialised for its outermost extent (template %d)", (int)grp.tmpl);
        for (auto& o : grp.operands)
            if (o.mapped(0)) pf::fail(PF_E_INVALID, "an operand is rolled or sliced along the outermost dim");
        check_execute_args(e, d_inputs, n_in, d_outputs, n_out, nullptr, 0);
        if (outer_extent < 1 || outer_extent > grp.domain[0])
            pf::fail(PF_E_INVALID, "outermost extent %lld outside 1 .. %lld (the compiled one)", (long long)outer_extent, (long long)grp.domain[0]);
        if ((outer_extent * grp.rt_rows_per_outer) % grp.rt_row_multiple)
            pf::fail(PF_E_INVALID, "this kernel needs a multiple of %lld rows", (long long)grp.rt_row_multiple);
        pf::exec_run(*e, d_inputs, d_outputs, nullptr, stream, nullptr, nullptr, outer_extent);
    });
}

pf_status pf_execute_timed(pf_exec* e, const void* const* d_inputs, int n_in, void* const* d_outputs, int n_out,
                           void* d_workspace, size_t workspace_bytes, void* stream, void* start_event, void* stop_event) {
    return guarded([&] {
        check_execute_args(e, d_inputs, n_in, d_outputs, n_out, d_workspace, workspace_bytes);
        pf::exec_run(*e, d_inputs, d_outputs, d_workspace, stream, start_event, stop_event);
    });
}

}  // extern "C"

namespace {

void check_pair(const pf_pair& p, int i) {
    if (p.cand_dtype != PF_F32 && p.cand_dtype != PF_BF16 && p.cand_dtype != PF_F16)
        pf::fail(PF_E_INVALID, "pair %d: candidate dtype must be f32, bf16 or f16", i);
    if (!pf::score_combo_supported(p.cand_dtype, p.ref_dtype))
        pf::fail(PF_E_INVALID, "pair %d: unsupported dtype combination (candidate %d, reference %d)", i, p.cand_dtype, p.ref_dtype);
    if (p.n && (!p.d_cand || !p.d_ref)) pf::fail(PF_E_INVALID, "pair %d: NULL buffer", i);
    if (((uintptr_t)p.d_cand | (uintptr_t)p.d_ref) & 15) pf::fail(PF_E_INVALID, "pair %d: buffers must be 16-byte aligned", i);
    if (!(p.rtol >= 0.0) || !(p.atol >= 0.0)) pf::fail(PF_E_INVALID, "pair %d: tolerances must be >= 0", i);
}

pf::PairDev descriptor(const pf_pair& p, int orig, unsigned long long chunk) {
    pf::PairDev d;
    memset(&d, 0, sizeof d);
    d.cand = p.d_cand;
    d.ref = p.d_ref;
    d.n = p.n;
    d.cand_dtype = p.cand_dtype;
    d.ref_dtype = p.ref_dtype;
    d.rtol = p.rtol;
    d.atol = p.atol;
    d.equal_nan = p.equal_nan;
    d.orig = orig;
    d.chunk = chunk;
    return d;
}

// Workspace: descriptors, workgroup prefix, tickets and seeds of the pairs, then 64 partial-result slots per pair
// for each result wanted.  Every part is written by the staging launch before it is read: a workspace needs
// no initialisation.
struct WsLayout {
    size_t pairs, start, wg_pair, tickets, seeds, sslots, lslots, total;
};
WsLayout ws_layout(int n_pairs, bool score, bool ladder) {
    const size_t n = n_pairs < 0 ? 0 : (size_t)n_pairs;
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    WsLayout w;
    size_t at = 0;
    w.pairs = at; at += up(n * sizeof(pf::PairDev));
    w.start = at; at += up((n + 1) * sizeof(unsigned long long));
    w.wg_pair = at; at += up((n + pf::kScoreMaxTargetWGs) * sizeof(int));      // a call has at most target + n workgroups      // a call has at most target + n workgroups
    w.tickets = at; at += up(n * (pf::kScoreSlots + 1) * sizeof(unsigned int));
    w.seeds = at; at += up(n * pf::kScoreSeedParts * 2 * sizeof(double));
    w.sslots = at; if (score) at += up(n * pf::kScoreSlots * sizeof(pf_score_result));
    w.lslots = at; if (ladder) at += up(n * pf::kScoreSlots * sizeof(pf_ladder_result));
    w.total = at;
    return w;
}

// One pass over the pairs for either result or both (d_score / d_ladder: NULL = not wanted).
void score_impl(const pf_pair* h_pairs, int n_pairs, pf_score_result* d_score, pf_ladder_result* d_ladder, void* d_workspace,
                size_t workspace_bytes, void* stream) {
    if (n_pairs < 0) pf::fail(PF_E_INVALID, "n_pairs < 0");
    if (n_pairs == 0) return;
    need(h_pairs, "h_pairs");
    if (!d_score && !d_ladder) pf::fail(PF_E_INVALID, "d_results is NULL");
    for (int i = 0; i < n_pairs; ++i) check_pair(h_pairs[i], i);      // nothing is enqueued for an invalid batch
    need(d_workspace, "d_workspace");
    const WsLayout lay = ws_layout(n_pairs, d_score != nullptr, d_ladder != nullptr);
    if (workspace_bytes < lay.total) pf::fail(PF_E_RUNTIME, "score workspace too small (%zu < %zu bytes)", workspace_bytes, lay.total);
    if ((uintptr_t)d_workspace & 255) pf::fail(PF_E_INVALID, "workspace is not 256-byte aligned");
    const hipStream_t hs = (hipStream_t)stream;
    pf::LadderTable table;
    memset(&table, 0, sizeof table);
    for (int dt : {(int)PF_F32, (int)PF_BF16, (int)PF_F16})
        for (int k = 0; k < PF_LADDER_LEVELS; ++k) pf::tolerance_at((pf_dtype)dt, k - (PF_LADDER_LEVELS - 1), &table.rtol[dt][k], &table.atol[dt][k]);

    // Small pairs take one workgroup each and a single launch per dtype combination; the others are staged
    // (descriptors, cleared slots, seeds) and then walked by one launch per dtype combination.
    std::vector<int> big, small[4][4];
    const unsigned long long small_max = pf::score_small_pair_elems();
    unsigned long long call_elems = 0;
    for (int i = 0; i < n_pairs; ++i) {
        const pf_pair& p = h_pairs[i];
        if (p.n <= small_max) small[p.cand_dtype][p.ref_dtype].push_back(i);
        else {
            big.push_back(i);
            call_elems += p.n;
        }
    }
    if (!big.empty()) {
        // ordered by dtype combination: each kernel instantiation then owns a contiguous range of workgroups
        auto combo = [&](int i) { return h_pairs[i].cand_dtype * 4 + h_pairs[i].ref_dtype; };
        std::stable_sort(big.begin(), big.end(), [&](int a, int b) { return combo(a) < combo(b); });
        const int nb = (int)big.size();
        const unsigned long long chunk = pf::score_chunk_elems(call_elems, d_ladder != nullptr);
        unsigned long long call_chunks = 0;
        for (int i : big) call_chunks += (h_pairs[i].n + chunk - 1) / chunk;
        const unsigned long long target = pf::score_target_wgs(d_ladder != nullptr, nb);
        const unsigned long long chunks_per_wg = (call_chunks + target - 1) / target;
        char* base = (char*)d_workspace;
        pf::ScoreSpace sp;
        sp.pairs = (pf::PairDev*)(base + lay.pairs);
        sp.start = (unsigned long long*)(base + lay.start);
        sp.wg_pair = (int*)(base + lay.wg_pair);
        sp.tickets = (unsigned int*)(base + lay.tickets);
        sp.seeds = (double*)(base + lay.seeds);
        sp.sslots = d_score ? (pf_score_result*)(base + lay.sslots) : nullptr;
        sp.lslots = d_ladder ? (pf_ladder_result*)(base + lay.lslots) : nullptr;
        pf::ScoreRanges ranges;
        memset(&ranges, 0, sizeof ranges);
        unsigned long long total = 0;
        pf::PairBatch b;
        for (int first = 0; first < nb; first += pf::kPairBatch) {
            memset(&b, 0, sizeof b);
            b.first = first;
            b.count = nb - first < pf::kPairBatch ? nb - first : pf::kPairBatch;
            b.last = first + b.count == nb;
            for (int k = 0; k < b.count; ++k) {
                const pf_pair& p = h_pairs[big[first + k]];
                b.pairs[k] = descriptor(p, big[first + k], chunk);
                b.start[k] = total;
                const unsigned long long nw = ((p.n + chunk - 1) / chunk + chunks_per_wg - 1) / chunks_per_wg;
                b.pairs[k].wgs = nw;
                if (ranges.count[p.cand_dtype][p.ref_dtype] == 0) ranges.first[p.cand_dtype][p.ref_dtype] = total;
                ranges.count[p.cand_dtype][p.ref_dtype] += nw;
                total += nw;
            }
            b.start[b.count] = total;
            if (total > pf::kScoreMaxTargetWGs + (unsigned long long)n_pairs) pf::fail(PF_E_INVALID, "internal: %llu workgroups", total);
            hipError_t err = pf::launch_stage(b, sp, hs);
            if (err != hipSuccess) pf::fail(PF_E_RUNTIME, "staging launch failed: %s", hipGetErrorString(err));
        }
        hipError_t err = pf::launch_pairs(sp, ranges, table, d_score, d_ladder, hs);
        if (err != hipSuccess) pf::fail(PF_E_RUNTIME, "score launch failed: %s", hipGetErrorString(err));
    }
    for (int cd = 0; cd < 4; ++cd)
        for (int rd = 0; rd < 4; ++rd) {
            const std::vector<int>& idx = small[cd][rd];
            for (size_t first = 0; first < idx.size(); first += pf::kPairBatch) {
                pf::PairBatch b;
                memset(&b, 0, sizeof b);
                b.count = (int)std::min<size_t>(pf::kPairBatch, idx.size() - first);
                for (int k = 0; k < b.count; ++k) b.pairs[k] = descriptor(h_pairs[idx[first + k]], idx[first + k], 0);
                hipError_t err = pf::launch_small(b, cd, rd, table, d_score, d_ladder, hs);
                if (err != hipSuccess) pf::fail(PF_E_RUNTIME, "score launch failed: %s", hipGetErrorString(err));
            }
        }
}

}  // namespace

extern "C" {

size_t pf_score_workspace_bytes(int n_pairs) { return ws_layout(n_pairs, true, false).total; }
size_t pf_score_ladder_workspace_bytes(int n_pairs) { return ws_layout(n_pairs, false, true).total; }
size_t pf_score_all_workspace_bytes(int n_pairs) { return ws_layout(n_pairs, true, true).total; }

pf_status pf_score(const pf_pair* h_pairs, int n_pairs, pf_score_result* d_results, void* d_workspace, size_t workspace_bytes,
                   void* stream) {
    return guarded([&] {
        if (n_pairs > 0) need(d_results, "d_results");
        score_impl(h_pairs, n_pairs, d_results, nullptr, d_workspace, workspace_bytes, stream);
    });
}

pf_status pf_score_ladder(const pf_pair* h_pairs, int n_pairs, pf_ladder_result* d_results, void* d_workspace,
                          size_t workspace_bytes, void* stream) {
    return guarded([&] {
        if (n_pairs > 0) need(d_results, "d_results");
        score_impl(h_pairs, n_pairs, nullptr, d_results, d_workspace, workspace_bytes, stream);
    });
}

pf_status pf_score_all(const pf_pair* h_pairs, int n_pairs, pf_score_result* d_score_results, pf_ladder_result* d_ladder_results,
                       void* d_workspace, size_t workspace_bytes, void* stream) {
    return guarded([&] {
        if (n_pairs > 0) {
            need(d_score_results, "d_score_results");
            need(d_ladder_results, "d_ladder_results");
        }
        score_impl(h_pairs, n_pairs, d_score_results, d_ladder_results, d_workspace, workspace_bytes, stream);
    });
}

pf_status pf_score_static(const pf_pair* h_pairs, int n_pairs, pf_score_result* d_results, void* stream) {
    return guarded([&] {
        if (n_pairs < 0) pf::fail(PF_E_INVALID, "n_pairs < 0");
        if (n_pairs > PF_SCORE_STATIC_MAX_PAIRS)
            pf::fail(PF_E_INVALID, "pf_score_static takes at most %d pairs per call (%d given); use pf_score with a workspace", PF_SCORE_STATIC_MAX_PAIRS,
                     n_pairs);
        if (n_pairs == 0) return;
        need(d_results, "d_results");
        void* d_scratch = nullptr;
        size_t bytes = 0;
        hipError_t err = pf::static_scratch(&d_scratch, &bytes);
        if (err != hipSuccess) pf::fail(PF_E_RUNTIME, "address of the library's scratch array: %s", hipGetErrorString(err));
        const size_t want = ws_layout(n_pairs, true, false).total;
        if (want > bytes) pf::fail(PF_E_INVALID, "internal: %d pairs need %zu bytes of scratch, the library holds %zu", n_pairs, want, bytes);
        score_impl(h_pairs, n_pairs, d_results, nullptr, d_scratch, bytes, stream);
    });
}

pf_status pf_tolerance(pf_dtype dtype, int t, double* h_rtol, double* h_atol) {
    return guarded([&] {
        need(h_rtol, "h_rtol");
        need(h_atol, "h_atol");
        pf::tolerance_at(dtype, t, h_rtol, h_atol);
    });
}

pf_status pf_aggregate(const pf_case* h_cases, int n_cases, double b, double p, pf_metrics* h_out) {
    return guarded([&] {
        need(h_cases, "h_cases");
        need(h_out, "h_out");
        if (n_cases <= 0) pf::fail(PF_E_INVALID, "need at least one case");
        pf::aggregate(h_cases, n_cases, b, p, h_out);
    });
}

pf_status pf_fast_p(const pf_case* h_cases, int n_cases, double threshold, int t, double* h_out) {
    return guarded([&] {
        need(h_cases, "h_cases");
        need(h_out, "h_out");
        if (n_cases <= 0) pf::fail(PF_E_INVALID, "need at least one case");
        *h_out = pf::fast_p(h_cases, n_cases, threshold, t);
    });
}

pf_status pf_copy_bytes(void* d_dst, const void* d_src, size_t bytes, void* stream) {
    return guarded([&] {
        need(d_dst, "d_dst");
        need(d_src, "d_src");
        if ((bytes & 15) || (((uintptr_t)d_dst | (uintptr_t)d_src) & 15)) pf::fail(PF_E_INVALID, "copy needs 16-byte granularity");
        hipError_t err = pf::launch_copy(d_dst, d_src, bytes, (hipStream_t)stream);
        if (err != hipSuccess) pf::fail(PF_E_RUNTIME, "copy launch failed: %s", hipGetErrorString(err));
    });
}

}  // extern "C"
