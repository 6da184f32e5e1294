// Kernel specialisation: emits the HIP source of one fused group.
//
// Each template is a hand-written skeleton (how elements map to lanes, how
// they are loaded, reduced and stored); the operators of the group become a
// straight-line body over per-lane register arrays.  All shapes are static, so
// every extent, stride and divisor is a literal in the emitted source.
//
//   EW_FLAT       elementwise chains, broadcast operands; flat 16-byte vectors
//   ROW_RESIDENT  last-dim reductions + epilogue; a team of T lanes holds one
//                 row in registers: one HBM read, one write (the paper's Case 1
//                 kernel makes three passes over the row instead)
//   TILE          groups that read a tensor through a swap of its last two
//                 dims; 64x64 tiles staged through LDS
//   COL_REDUCE    reductions over the second-to-last dim (pooling over the
//                 sequence dim, the paper's Case 2) with an elementwise
//                 prologue and an epilogue on the reduced shape
#include <cmath>
#include <cstring>
#include <functional>
#include <set>

#include "device_prelude.h"
#include "pf_internal.h"

namespace pf {

namespace {

struct Emit {
    const pf_graph& g;
    const pf_options& opt;
    Group& grp;
    std::string s;                       // source being built
    std::map<int, int> operand_of;       // node -> operand index (plain reads)
    std::map<int, int> toperand_of;      // node -> operand index (transposed reads)
    std::map<int, int> voperand_of;      // roll / slice node -> operand index (reads through its index map)
    std::map<int, int> coperand_of;      // node -> operand index (reads of a column reduction's epilogue)
    std::map<int, int> plan_kind;        // member node -> kind the planner gave it (3: column-uniform)
    std::set<int> members;
    std::map<int, int> kind;             // member/operand node -> 2 full, 1 row-uniform
    bool precise = false;
    bool wide = false;                   // 64-bit indexing
    int rd = 0;                          // domain rank

    Emit(const pf_graph& gr, const pf_options& o, Group& gp) : g(gr), opt(o), grp(gp) {}

    void line(const std::string& t) { s += t; s += '\n'; }

    static std::string lit(double v) {
        if (std::isnan(v)) return "__builtin_nanf(\"\")";
        if (std::isinf(v)) return v > 0 ? "__builtin_inff()" : "(-__builtin_inff())";
        return strf("((float)%a)", v);
    }
    const char* ctype(pf_dtype d) const { return d == PF_BF16 ? "u16" : d == PF_F16 ? "f16" : "float"; }
    const char* idx_t() const { return wide ? "long long" : "unsigned"; }

    bool in_kernel(int p) const {
        if (!members.count(p)) return false;
        const Node& n = g.nodes[p];
        return !(is_reduction(n.op) && !n.keepdim && n.red_dim == -1);
    }
    bool epilogue_node(int id) const {
        return grp.tmpl == PF_T_COL_REDUCE && plan_kind.at(id) == 3 && !is_reduction(g.nodes[id].op);
    }

    // Register layout of a value inside a lane: RU rows ("u") times NN slots ("j").
    int RU = 1, NN = 1;
    std::set<int> hoisted;               // operand indices loaded once for all RU rows

    std::string slot(const std::string& j) const { return RU == 1 ? j : strf("u * %d + %s", NN, j.c_str()); }

    // expression for the value of node p at row u, register slot j (a string like "j" or "j + 1")
    std::string ref(int consumer, int p, const std::string& j) const {
        const Node& n = g.nodes[p];
        if (n.op == PF_OP_CONST) return lit(n.value);
        if (in_kernel(p) && !reads_alias(consumer, p)) return kind.at(p) == 2 ? strf("v%d[%s]", p, slot(j).c_str()) : strf("s%d[u]", p);
        int oi = is_view(n.op) ? voperand_of.at(p) : epilogue_node(consumer) ? coperand_of.at(p) : reads_alias(consumer, p) ? toperand_of.at(p) : operand_of.at(p);
        const bool h = hoisted.count(oi) != 0;
        if (operand_kind(oi) == 2) return h ? strf("x%d[%s]", oi, j.c_str()) : strf("x%d[%s]", oi, slot(j).c_str());
        return h ? strf("x%d[0]", oi) : strf("x%d[u]", oi);
    }

    // does the consumer read p through an orientation change that moves no data?
    bool reads_alias(int consumer, int p) const {
        const Node& c = g.nodes[consumer];
        for (size_t k = 0; k < c.in.size(); ++k)
            if (c.in[k] == p && c.reads_alias(k)) return true;
        return false;
    }

    // 2: varies along the last dim (array per lane); 1: uniform along it (scalar per row)
    int operand_kind(int oi) const {
        const Operand& o = grp.operands[oi];
        if (o.coluni) return 1;               // one value per epilogue lane
        if (grp.tmpl == PF_T_TILE) return 2;
        if (grp.tmpl == PF_T_EW_FLAT && straddle) return 2;
        if (rd == 0) return 1;
        if (grp.cols == 1) return 2;          // last dim of size 1: "full" and "row-uniform" coincide
        return o.stride[rd - 1] != 0 ? 2 : 1;
    }

    bool straddle = false;

    int node_kind(int id) const {
        const Node& n = g.nodes[id];
        if (is_reduction(n.op)) return 1;
        if (is_view(n.op)) return 2;
        if (grp.tmpl == PF_T_COL_REDUCE) return plan_kind.at(id) == 3 ? 1 : 2;
        if (grp.tmpl != PF_T_ROW_RESIDENT && grp.tmpl != PF_T_ROW_LOOP) return 2;
        if (grp.cols == 1) return 2;
        // row-uniform iff every operand is
        for (int p : n.in) {
            if (g.nodes[p].op == PF_OP_CONST) continue;
            int k = in_kernel(p) && !reads_alias(id, p) ? kind.at(p)
                    : operand_kind(is_view(g.nodes[p].op) ? voperand_of.at(p) : reads_alias(id, p) ? toperand_of.at(p) : operand_of.at(p));
            if (k == 2) return 2;
        }
        return 1;
    }

    // ---- body: one statement (or loop) per member node over N register slots ----
    void emit_elementwise(int id, int N) {
        const Node& n = g.nodes[id];
        const int k = kind.at(id);
        auto expr = [&](const std::string& j) -> std::string {
            auto a = [&](int i) { return ref(id, n.in[i], j); };
            switch (n.op) {
                case PF_OP_ADD: return a(0) + " + " + a(1);
                case PF_OP_SUB: return a(0) + " - " + a(1);
                case PF_OP_MUL: return a(0) + " * " + a(1);
                case PF_OP_DIV: return "pf_div(" + a(0) + ", " + a(1) + ")";
                case PF_OP_EXP: return "pf_exp(" + a(0) + ")";
                case PF_OP_TANH: return "pf_tanh(" + a(0) + ")";
                case PF_OP_SIGMOID: return "pf_sigmoid(" + a(0) + ")";
                case PF_OP_GELU: return std::string(n.gelu_erf ? "pf_gelu_erf(" : "pf_gelu_tanh(") + a(0) + ")";
                case PF_OP_RSQRT: return "pf_rsqrt(" + a(0) + ")";
                case PF_OP_MAXIMUM: return "pf_max_nan(" + a(0) + ", " + a(1) + ")";
                case PF_OP_MINIMUM: return "pf_min_nan(" + a(0) + ", " + a(1) + ")";
                default: fail(PF_E_COMPILE, "internal: %s is not elementwise", op_name(n.op));
            }
        };
        const std::string loops = strf("    _Pragma(\"unroll\") for (int u = 0; u < %d; ++u) _Pragma(\"unroll\") for (int j = 0; j < %d; %s)", RU,
                                       N, n.op == PF_OP_ROT_PAIRS ? "j += 2" : "++j");
        if (n.op == PF_OP_TRANSPOSE || is_view(n.op)) {
            // value arrives through the transposed / index-mapped operand
            int oi = is_view(n.op) ? voperand_of.at(id) : toperand_of.at(n.in[0]);
            line(strf("    float v%d[%d];", id, RU * N));
            line(loops + strf(" v%d[%s] = x%d[%s];", id, slot("j").c_str(), oi, slot("j").c_str()));
            return;
        }
        if (n.op == PF_OP_ROT_PAIRS) {
            if (k != 2) fail(PF_E_COMPILE, "rot_pairs of a row-uniform value");
            std::string a0 = ref(id, n.in[0], "j + 1"), a1 = ref(id, n.in[0], "j");
            line(strf("    float v%d[%d];", id, RU * N));
            line(loops + strf(" { v%d[%s] = -(%s); v%d[%s] = %s; }", id, slot("j").c_str(), a0.c_str(), id, slot("j + 1").c_str(),
                              a1.c_str()));
            return;
        }
        if (k == 2) {
            line(strf("    float v%d[%d];", id, RU * N));
            line(loops + strf(" v%d[%s] = %s;", id, slot("j").c_str(), expr("j").c_str()));
        } else {
            line(strf("    float s%d[%d];", id, RU));
            line(strf("    _Pragma(\"unroll\") for (int u = 0; u < %d; ++u) s%d[u] = %s;", RU, id, expr("0").c_str()));
        }
    }

    // ================================================================ ROW_RESIDENT
    // A team of T lanes (a slice of a wave, a wave, or several waves) owns RU
    // consecutive rows at a time.  Lane l holds chunks l, l+T, l+2T, ... of VEC
    // contiguous elements of each row, so every load instruction of a team
    // covers T*VEC contiguous elements.  Operands that do not change along the
    // innermost leading dim (tables, weights) are loaded once for all RU rows.
    void gen_row() {
        const int64_t C = grp.cols, R = grp.rows;
        int min_item = 4;
        for (auto& o : grp.operands)
            if (operand_kind_pre(o) == 2) min_item = std::min(min_item, itemsize(o.dtype));
        for (auto& st : grp.stores)
            if (!st.row_scalar) min_item = std::min(min_item, itemsize(st.dtype));
        // Rows whose length is not a multiple of the vector still use full 16-byte
        // accesses (merely element-aligned); only the last chunk of a row is ragged.
        int vec = 16 / min_item;
        while (vec > 1 && vec > C) vec >>= 1;
        const bool ragged = C % vec != 0;
        const int64_t chunks = (C + vec - 1) / vec;
        const int per_lane_max = 32 / vec > 0 ? 32 / vec : 1;      // keep <= 32 floats per value per lane
        // Lanes per row.  Every lane of a team pays the cross-lane reductions (log2 T shuffle steps per
        // reduction, doubled for fp64 accumulators), so the smallest team that still issues whole cache
        // lines per load is the cheapest: about 16 elements per lane and value (measured over rows of
        // 24 ... 11008 elements, fp32 and bf16: 16-element lanes are up to 2x faster than 8-element
        // ones on fp32 LayerNorm rows of 96 ... 768 and never more than 10% slower).
        const int k_target = std::max(1, 16 / vec);
        int T = 1;
        while (T < 8 && T < chunks) T <<= 1;        // a team's load covers at least one 128-byte line
        while (T < 1024 && (chunks + T - 1) / T > std::min(per_lane_max, k_target)) T <<= 1;
        while ((chunks + T - 1) / T > per_lane_max && T < 1024) T <<= 1;
        int64_t K = (chunks + T - 1) / T;
        if (K * vec > 64) {          // the row does not fit in the registers of 1024 lanes: stream it
            gen_loop(vec, ragged);
            return;
        }
        // Padding: K * T chunk slots for `chunks` chunks.  When more than a tenth of the slots is empty,
        // half or twice the lanes may fit better (17 chunks: 8 x 3 instead of 16 x 2; 1376 chunks:
        // 512 x 3 instead of 1024 x 2, measured 15% faster).
        auto slots = [&](int t) { return ((chunks + t - 1) / t) * t; };
        if (slots(T) * 10 > chunks * 11) {
            int best = T;
            if (T >= 16 && (chunks + T / 2 - 1) / (T / 2) <= per_lane_max && slots(T / 2) < slots(best)) best = T / 2;
            if (T < 1024 && slots(T * 2) < slots(best)) best = T * 2;
            T = best;
            K = (chunks + T - 1) / T;
        }
        // few rows: spread each row over more lanes until about six waves per CU exist
        while (K > 1 && T < 1024 && R * T < 256 * 64 * 6) {
            T <<= 1;
            K = (chunks + T - 1) / T;
        }
        // (Spreading few long rows over still more, lighter lanes once tens of MB cross the kernel paid while the fp32
        // operators were the library's: 556 x 4096 fp32 rows with three divisions, two tanh and an exp ran 20% faster
        // with 1024 lanes x 4 elements than with 256 x 16.  With the estimate-based operators it is the other way
        // round, 20.4 us against 13.4 us, so the rule is gone.)
        // A workgroup of 1024 lanes leaves each lane 128 registers, one of 512 lanes 256: rows that fit 512 lanes with
        // at most 32 elements per lane and value run there (96 rows of 11008 fp32 elements with eleven full-size
        // operands and results spilled 28 registers at 1024 x 12 and ran in 18.6 us, 16.3 us at 512 x 24)
        if (T == 1024 && (chunks + 511) / 512 <= per_lane_max) {
            T = 512;
            K = (chunks + T - 1) / T;
        }
        if (opt.tune_row_lanes > 0) {
            T = opt.tune_row_lanes;
            if (T & (T - 1) || T > 1024) fail(PF_E_INVALID, "tune_row_lanes must be a power of two <= 1024");
            K = (chunks + T - 1) / T;
            if (K * vec > 64) fail(PF_E_COMPILE, "tune_row_lanes=%d leaves %lld elements per lane", T, (long long)(K * vec));
        }
        const int N = (int)K * vec;
        // rows in flight per team: short rows leave registers free, and more
        // independent loads per lane are what keeps HBM busy
        const int nlead = rd > 0 ? rd - 1 : 0;
        scan_decomp(nlead);
        // Rows in flight per team.  More independent loads per lane help only while enough waves remain
        // to fill the chip twice over: one extra row per 262144 lanes (4096 waves), at most four, and
        // at most 32 elements per lane and value.  (Measured: 2 rows on 16384 x 512 bf16 rows and 4 on
        // 262144 x 128 are 8% and 3% faster than one; on 2M-element problems any more than one row is
        // 10 ... 100% slower.)
        int ru = 1;
        if (T <= 64 && !ragged) {      // ragged rows measured 15% slower with a second row in flight
            while (ru < 4 && R * T >= (int64_t)262144 * ru * 2) ru <<= 1;
            while (ru > 1 && ru * N > 32) ru >>= 1;
        }
        if (opt.tune_row_unroll > 0) ru = T <= 64 ? opt.tune_row_unroll : 1;
        const int64_t inner = nlead > 0 ? grp.domain[nlead - 1] : 1;
        if (need_decomp)
            while (ru > 1 && inner % ru) ru >>= 1;   // all RU rows must share their outer indices
        if (ru > R) ru = 1;
        RU = ru;
        NN = N;
        const bool groups_exact = R % RU == 0;
        const int block = T > 256 ? T : 256;
        const int teams = block / T;
        const bool mask = (int64_t)K * T * vec != C && !ragged;   // whole chunks beyond the row end
        const int64_t row_groups = (R + RU - 1) / RU;
        grp.block = block;
        grp.grid = (row_groups + teams - 1) / teams;
        if (rd >= 2) {
            grp.rt_per_outer = grp.rt_rows_per_outer = inner_rows();
            grp.rt_per_block = (int64_t)RU * teams;
            grp.rt_row_multiple = groups_exact ? RU : 1;      // a kernel compiled for whole row groups has no partial-group code
        }
        grp.lanes_per_row = T;
        grp.vec = vec;
        grp.chunks_per_lane = (int)K;
        const char* acc = precise ? "double" : "float";
        hoisted.clear();
        if (RU > 1)
            for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
                const Operand& o = grp.operands[oi];
                const bool inner_const = nlead == 0 || (o.stride[nlead - 1] == 0 && !o.mapped(nlead - 1));
                if (lead_zero(o, nlead) || (inner_const && inner % RU == 0)) hoisted.insert((int)oi);
            }

        int n_red = 0;
        for (int id : grp.nodes)
            if (is_reduction(g.nodes[id].op)) n_red += g.nodes[id].op == PF_OP_VAR ? 2 : 1;

        // the outermost extent is a kernel argument: problems that differ only there (and lead to the
        // same tiling decisions) generate the same source text and share one code object
        set_outer_runtime();
        signature(outer_param());
        line(strf("    constexpr int T = %d, K = %d, VEC = %d, N = %d, RU = %d, TEAMS = %d;", T, (int)K, vec, N, RU, teams));
        if (grp.outer_runtime) {
            line(strf("    constexpr %s C = %lld;", idx_t(), (long long)C));
            line(strf("    const %s ROWS = (%s)pf_d0 * %lld, GROUPS = (ROWS + RU - 1) / RU;", idx_t(), idx_t(), (long long)inner_rows()));
        } else
        line(strf("    constexpr %s C = %lld, ROWS = %lld, GROUPS = %lld;", idx_t(), (long long)C, (long long)R, (long long)row_groups));
        if (T > 64) line(strf("    __shared__ %s red_lds[%d][%d];", acc, std::max(n_red, 1), block / 64));
        if (T > 64 && precise) line(strf("    __shared__ float redf_lds[%d][%d];", std::max(n_red, 1), block / 64));
        line("    const int team = threadIdx.x / T, lane = threadIdx.x % T;");
        line(strf("    const %s grp_raw = (%s)blockIdx.x * TEAMS + team;", idx_t(), idx_t()));
        line("    const bool grp_ok = grp_raw < GROUPS;");
        // lanes of a team past the end stay alive (shuffles, barriers) on the last group
        line(strf("    const %s row0 = (grp_ok ? grp_raw : GROUPS - 1) * RU;", idx_t()));
        line(strf("    %s row[RU]; bool row_ok[RU];", idx_t()));
        if (groups_exact) line("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) { row[u] = row0 + u; row_ok[u] = grp_ok; }");
        else line("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) { row_ok[u] = grp_ok && row0 + u < ROWS; row[u] = row0 + u < ROWS ? row0 + u : ROWS - 1; }");
        emit_lead_decomposition("row0", nlead);
        // loads
        for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
            const Operand& o = grp.operands[oi];
            const bool h = hoisted.count((int)oi) != 0;
            const int reps = h ? 1 : RU;
            // offset of row u: outer part from row0 (or the row itself when strides nest)
            std::string base;
            if (lead_zero(o, nlead)) base = strf("(%s)0", idx_t());
            else if (lead_mergeable(o, nlead)) base = strf("row[u] * %lld", (long long)o.stride[nlead - 1]);
            else base = lead_offset_row_u(o, nlead);
            if (operand_kind((int)oi) == 1) {
                line(strf("    float x%zu[%d];", oi, reps));
                line(strf("    _Pragma(\"unroll\") for (int u = 0; u < %d; ++u) x%zu[u] = pf_ld1(p%zu + %s);", reps, oi, oi, base.c_str()));
                continue;
            }
            const bool nt = numel(o.shape) * itemsize(o.dtype) >= (int64_t(1) << 22);
            line(strf("    float x%zu[%d];", oi, reps * N));
            line(strf("    _Pragma(\"unroll\") for (int u = 0; u < %d; ++u) _Pragma(\"unroll\") for (int k = 0; k < K; ++k) {", reps));
            emit_chunk_start(ragged);
            if (last_mapped(o)) {     // rolled / sliced along the row: gather element by element
                line(strf("        _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) x%zu[u * N + k * VEC + j] = (c0 + j < C) ? pf_ld1(p%zu + %s + %s * %lld) : 0.0f;",
                          oi, oi, base.c_str(), mapexpr(o, rd - 1, "(c0 + j)").c_str(), (long long)o.stride[rd - 1]));
            } else if (ragged) {
                line(strf("        pf_ld<VEC, %s, true>(p%zu + %s + c0, &x%zu[u * N + k * VEC]);", nt ? "true" : "false", oi, base.c_str(), oi));
            } else if (mask) {
                line(strf("        if (c0 < C) pf_ld<VEC, %s>(p%zu + %s + c0, &x%zu[u * N + k * VEC]);", nt ? "true" : "false", oi,
                          base.c_str(), oi));
                line(strf("        else { _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) x%zu[u * N + k * VEC + j] = 0.0f; }", oi));
            } else {
                line(strf("        pf_ld<VEC, %s>(p%zu + %s + c0, &x%zu[u * N + k * VEC]);", nt ? "true" : "false", oi, base.c_str(), oi));
            }
            line("    }");
        }
        // body
        int red_slot = 0;
        for (int id : grp.nodes) {
            const Node& n = g.nodes[id];
            if (!is_reduction(n.op)) {
                emit_elementwise(id, N);
                continue;
            }
            const int src = n.in[0];
            auto valid_open = [&]() {
                line("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) _Pragma(\"unroll\") for (int k = 0; k < K; ++k) {");
                emit_chunk_start(ragged);
                line("        _Pragma(\"unroll\") for (int jj = 0; jj < VEC; ++jj) {");
                line("            const int j = k * VEC + jj;");
                line(strf("            if (%s) {", ragged ? "jj >= skip" : mask ? "c0 < C" : "true"));
            };
            auto valid_close = [&]() { line("            }"); line("        }"); line("    }"); };
            std::string xj = ref(id, src, "j");
            const std::string lds = T > 64 ? strf("red_lds[%d]", red_slot) : "nullptr";
            if (n.op == PF_OP_MAX) {
                line(strf("    float m%d[RU]; bool nan%d[RU];", id, id));
                line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) { m%d[u] = -__builtin_inff(); nan%d[u] = false; }", id, id));
                valid_open();
                line(strf("                const float t = %s; m%d[u] = fmaxf(m%d[u], t); nan%d[u] |= (t != t);", xj.c_str(), id, id, id));
                valid_close();
                line(strf("    float s%d[RU];", id));
                line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) s%d[u] = pf_team_max<T>(nan%d[u] ? __builtin_nanf(\"\") : m%d[u], %s);",
                          id, id, id, T > 64 ? strf(precise ? "redf_lds[%d]" : "red_lds[%d]", red_slot).c_str() : "nullptr"));
                ++red_slot;
                continue;
            }
            // sum, mean, var
            line(strf("    %s a%d[RU];", acc, id));
            line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) a%d[u] = 0;", id));
            valid_open();
            line(strf("                a%d[u] += (%s)(%s);", id, acc, xj.c_str()));
            valid_close();
            line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) a%d[u] = pf_team_sum<T, %s>(a%d[u], %s);", id, acc, id, lds.c_str()));
            ++red_slot;
            line(strf("    float s%d[RU];", id));
            if (n.op == PF_OP_SUM) {
                line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) s%d[u] = (float)a%d[u];", id, id));
            } else if (n.op == PF_OP_MEAN) {
                line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) s%d[u] = (float)(a%d[u] / (%s)%lld);", id, id, acc, (long long)C));
            } else {
                line(strf("    %s q%d[RU];", acc, id));
                line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) { a%d[u] = a%d[u] / (%s)%lld; q%d[u] = 0; }", id, id, acc,
                          (long long)C, id));
                valid_open();
                line(strf("                const %s d = (%s)(%s) - a%d[u]; q%d[u] += d * d;", acc, acc, xj.c_str(), id, id));
                valid_close();
                line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) s%d[u] = (float)(pf_team_sum<T, %s>(q%d[u], %s) / (%s)%lld);", id,
                          acc, id, T > 64 ? strf("red_lds[%d]", red_slot).c_str() : "nullptr", acc, (long long)(C - n.correction)));
                ++red_slot;
            }
        }
        // stores
        int sp = 0;
        for (auto& st : grp.stores) {
            std::vector<int> ptrs;
            ptrs.push_back(sp++);
            for (size_t k = 0; k < st.also_outputs.size(); ++k) ptrs.push_back(sp++);
            for (int q : ptrs) {
                if (st.row_scalar) {
                    line(strf("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) if (row_ok[u] && lane == 0) pf_st1(q%d + row[u], s%d[u]);", q,
                              st.node));
                } else if (kind.at(st.node) == 1) {
                    // a row-uniform value stored at full shape cannot occur: its shape has last dim 1
                    fail(PF_E_COMPILE, "internal: full store of a row-uniform value");
                } else {
                    const bool nt = numel(st.shape) * itemsize(st.dtype) >= (int64_t(1) << 22);
                    line("    _Pragma(\"unroll\") for (int u = 0; u < RU; ++u) _Pragma(\"unroll\") for (int k = 0; k < K; ++k) {");
                    emit_chunk_start(ragged);
                    if (ragged) {
                        // the shifted last chunk stores the elements it shares with the chunk before a second time, with the same values
                        line(strf("        if (row_ok[u] && c0n < C) pf_st<VEC, %s, true>(q%d + row[u] * C + c0, &v%d[u * N + k * VEC]);",
                                  nt ? "true" : "false", q, st.node));
                    } else
                    line(strf("        if (row_ok[u]%s) pf_st<VEC, %s>(q%d + row[u] * C + c0, &v%d[u * N + k * VEC]);", mask ? " && c0 < C" : "",
                              nt ? "true" : "false", q, st.node));
                    line("    }");
                }
            }
        }
        line("}");
    }

    // Where a lane's chunk k starts in its row.  Rows whose length is no multiple of the vector end in a partial
    // chunk; that chunk is moved back so that it ends with the row: every access stays a full vector inside the
    // row, and the `skip` elements it shares with the chunk before it are left out of reductions (they are
    // computed twice, with identical results, and stored twice).  A chunk that lies wholly past the row
    // (c0n >= C) reads the same last vector and contributes nothing.
    void emit_chunk_start(bool ragged) {
        if (!ragged) {
            line(strf("        const %s c0 = (%s)(k * T + lane) * VEC;", idx_t(), idx_t()));
            return;
        }
        line(strf("        const %s c0n = (%s)(k * T + lane) * VEC;", idx_t(), idx_t()));
        line(strf("        const %s c0 = c0n + VEC <= C ? c0n : C - VEC;", idx_t()));
        line("        const int skip = (int)(c0n - c0); (void)skip;");
    }

    // ================================================================ ROW_LOOP
    // Rows too long to hold on chip.  One workgroup of T lanes walks its row in
    // steps of T*VEC elements, once per "pass": pass p recomputes every value whose
    // inputs are available by then and accumulates the reductions that read them,
    // so a chain of k dependent reductions costs k+1 passes over the inputs (the
    // repeats are served by L2 when the row fits there).  The paper's Case 1
    // kernel has this same structure (mean pass, variance pass, write pass).
    void gen_loop(int vec, bool ragged) {
        grp.tmpl = PF_T_ROW_LOOP;
        const int64_t C = grp.cols, R = grp.rows;
        const int T = 1024;
        const int nlead = rd > 0 ? rd - 1 : 0;
        RU = 1;
        NN = vec;
        hoisted.clear();
        grp.block = T;
        grp.grid = R;
        if (rd >= 2) {
            grp.rt_per_outer = grp.rt_rows_per_outer = inner_rows();
            grp.rt_per_block = 1;
        }
        grp.lanes_per_row = T;
        grp.vec = vec;
        grp.chunks_per_lane = (int)(((C + vec - 1) / vec + T - 1) / T);
        const char* acc = precise ? "double" : "float";
        // stage of every value: the first pass in which it can be computed
        std::map<int, int> stage, rpass;     // node -> stage; reduction -> pass in which it accumulates
        auto avail = [&](int p) -> int {
            const Node& n = g.nodes[p];
            if (n.op == PF_OP_CONST || !in_kernel(p)) return 0;
            if (is_reduction(n.op)) return rpass.at(p) + (n.op == PF_OP_VAR ? 2 : 1);
            return stage.at(p);
        };
        int last_pass = 0;
        for (int id : grp.nodes) {
            const Node& n = g.nodes[id];
            int st = 0;
            for (int p : n.in) st = std::max(st, avail(p));
            if (is_reduction(n.op)) {
                rpass[id] = st;
                last_pass = std::max(last_pass, st + (n.op == PF_OP_VAR ? 1 : 0));
            } else {
                stage[id] = st;
            }
        }
        for (auto& st : grp.stores)
            if (!st.row_scalar) last_pass = std::max(last_pass, stage.at(st.node));
        int n_red = 0;
        for (int id : grp.nodes)
            if (is_reduction(g.nodes[id].op)) n_red += g.nodes[id].op == PF_OP_VAR ? 2 : 1;

        signature();
        line(strf("    constexpr int T = %d, VEC = %d;", T, vec));
        line(strf("    constexpr %s C = %lld, CHUNKS = %lld;", idx_t(), (long long)C, (long long)((C + vec - 1) / vec)));
        line(strf("    __shared__ %s red_lds[%d][%d];", acc, std::max(n_red, 1), T / 64));
        if (precise) line(strf("    __shared__ float redf_lds[%d][%d];", std::max(n_red, 1), T / 64));
        line("    const int lane = threadIdx.x;");
        line(strf("    %s row[1]; row[0] = blockIdx.x;", idx_t()));
        line("    constexpr int u = 0;");
        emit_lead_decomposition("row[0]", nlead);
        // row-uniform operands are loaded once
        for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
            if (operand_kind((int)oi) != 1) continue;
            const Operand& o = grp.operands[oi];
            std::string base = lead_zero(o, nlead) ? strf("(%s)0", idx_t())
                               : lead_mergeable(o, nlead) ? strf("row[0] * %lld", (long long)o.stride[nlead - 1])
                                                          : lead_offset(o, "row[0]");
            line(strf("    float x%zu[1]; x%zu[0] = pf_ld1(p%zu + %s);", oi, oi, oi, base.c_str()));
        }
        auto emit_uniform_nodes = [&](int st) {
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (is_reduction(n.op) || kind.at(id) != 1 || stage.at(id) != st) continue;
                emit_elementwise(id, vec);
            }
        };
        emit_uniform_nodes(0);
        int red_slot = 0;
        std::map<int, int> slot_of;
        for (int id : grp.nodes)
            if (is_reduction(g.nodes[id].op)) {
                slot_of[id] = red_slot;
                red_slot += g.nodes[id].op == PF_OP_VAR ? 2 : 1;
            }
        for (int pass = 0; pass <= last_pass; ++pass) {
            // accumulators of this pass
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (!is_reduction(n.op)) continue;
                if (rpass.at(id) == pass) {
                    if (n.op == PF_OP_MAX) line(strf("    float m%d = -__builtin_inff(); bool nan%d = false;", id, id));
                    else line(strf("    %s a%d = 0;", acc, id));
                }
                if (n.op == PF_OP_VAR && rpass.at(id) + 1 == pass) line(strf("    %s q%d = 0;", acc, id));
            }
            line(strf("    for (%s k = lane; k < CHUNKS; k += T) {   // pass %d", idx_t(), pass));
            line(strf("        const %s c0 = k * VEC;", idx_t()));
            for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
                if (operand_kind((int)oi) != 2) continue;
                const Operand& o = grp.operands[oi];
                std::string base = lead_zero(o, nlead) ? strf("(%s)0", idx_t())
                                   : lead_mergeable(o, nlead) ? strf("row[0] * %lld", (long long)o.stride[nlead - 1])
                                                              : lead_offset(o, "row[0]");
                if (last_mapped(o)) {
                    line(strf("        float x%zu[VEC];", oi));
                    line(strf("        _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) x%zu[j] = (c0 + j < C) ? pf_ld1(p%zu + %s + %s * %lld) : 0.0f;", oi,
                              oi, base.c_str(), mapexpr(o, rd - 1, "(c0 + j)").c_str(), (long long)o.stride[rd - 1]));
                } else if (ragged) {
                    line(strf("        float x%zu[VEC];", oi));
                    line(strf("        if (c0 + VEC <= C) pf_ld<VEC, false, true>(p%zu + %s + c0, x%zu);", oi, base.c_str(), oi));
                    line(strf("        else { _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) x%zu[j] = (c0 + j < C) ? pf_ld1(p%zu + %s + c0 + j) : 0.0f; }",
                              oi, oi, base.c_str()));
                } else
                line(strf("        float x%zu[VEC]; pf_ld<VEC, false>(p%zu + %s + c0, x%zu);", oi, oi, base.c_str(), oi));
            }
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (is_reduction(n.op)) {
                    std::string xj = ref(id, n.in[0], "j");
                    if (rpass.at(id) == pass) {
                        if (n.op == PF_OP_MAX)
                            line(strf("        _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) if (%s) { const float t = %s; m%d = fmaxf(m%d, t); nan%d |= (t != t); }",
                                      ragged ? "c0 + j < C" : "true", xj.c_str(), id, id, id));
                        else
                            line(strf("        _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) if (%s) a%d += (%s)(%s);", ragged ? "c0 + j < C" : "true", id,
                                      acc, xj.c_str()));
                    }
                    if (n.op == PF_OP_VAR && rpass.at(id) + 1 == pass)
                        line(strf("        _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) if (%s) { const %s d = (%s)(%s) - a%d; q%d += d * d; }",
                                  ragged ? "c0 + j < C" : "true", acc, acc, xj.c_str(), id, id));
                    continue;
                }
                if (kind.at(id) == 2 && stage.at(id) <= pass) emit_elementwise(id, vec);
            }
            int sp = 0;
            for (auto& st : grp.stores) {
                const int cnt = 1 + (int)st.also_outputs.size();
                if (!st.row_scalar && stage.at(st.node) == pass)
                    for (int c = 0; c < cnt; ++c)
                        if (ragged) {
                            line(strf("        if (c0 + VEC <= C) pf_st<VEC, false, true>(q%d + row[0] * C + c0, v%d);", sp + c, st.node));
                            line(strf("        else { _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) if (c0 + j < C) pf_st1(q%d + row[0] * C + c0 + j, v%d[j]); }",
                                      sp + c, st.node));
                        } else
                        line(strf("        pf_st<VEC, false>(q%d + row[0] * C + c0, v%d);", sp + c, st.node));
                sp += cnt;
            }
            line("    }");
            // finish the reductions of this pass
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (!is_reduction(n.op)) continue;
                const int sl = slot_of.at(id);
                if (rpass.at(id) == pass) {
                    if (n.op == PF_OP_MAX) {
                        line(strf("    float s%d[1]; s%d[0] = pf_team_max<T>(nan%d ? __builtin_nanf(\"\") : m%d, %s[%d]);", id, id, id, id,
                                  precise ? "redf_lds" : "red_lds", sl));
                    } else {
                        line(strf("    a%d = pf_team_sum<T, %s>(a%d, red_lds[%d]);", id, acc, id, sl));
                        if (n.op == PF_OP_SUM) line(strf("    float s%d[1]; s%d[0] = (float)a%d;", id, id, id));
                        else if (n.op == PF_OP_MEAN) line(strf("    float s%d[1]; s%d[0] = (float)(a%d / (%s)%lld);", id, id, id, acc, (long long)C));
                        else line(strf("    a%d = a%d / (%s)%lld;", id, id, acc, (long long)C));
                    }
                }
                if (n.op == PF_OP_VAR && rpass.at(id) + 1 == pass)
                    line(strf("    float s%d[1]; s%d[0] = (float)(pf_team_sum<T, %s>(q%d, red_lds[%d]) / (%s)%lld);", id, id, acc, id, sl + 1, acc,
                              (long long)(C - n.correction)));
            }
            emit_uniform_nodes(pass + 1);
        }
        int sp = 0;
        for (auto& st : grp.stores) {
            const int cnt = 1 + (int)st.also_outputs.size();
            if (st.row_scalar)
                for (int c = 0; c < cnt; ++c) line(strf("    if (lane == 0) pf_st1(q%d + row[0], s%d[0]);", sp + c, st.node));
            sp += cnt;
        }
        line("}");
    }

    // ================================================================ COL_REDUCE
    // Domain [lead..., S, DD]; reductions run over S.  A workgroup of TX x TY
    // lanes owns one leading index and W = TX*VEC adjacent columns: lane (tx, ty)
    // walks rows ty, ty+TY, ... with 16-byte loads along DD (U rows in flight),
    // applies the prologue and accumulates VEC columns in registers.  Partial
    // sums meet by wave shuffles across ty, then in LDS across waves; lane c < W
    // finishes column c: it evaluates the epilogue once and stores one element.
    // A variance takes a second walk over the rows (mean first).
    void gen_col() {
        if (rd < 2) fail(PF_E_COMPILE, "internal: column reduction of rank < 2");
        const int64_t S = grp.domain[rd - 2], DD = grp.domain[rd - 1];
        int64_t L = 1;
        for (int k = 0; k < rd - 2; ++k) L *= grp.domain[k];
        const int nlead = rd - 2;
        int min_item = 4, n_vec_ops = 0;
        for (auto& o : grp.operands)
            if (!o.coluni && o.stride[rd - 1] != 0) {
                min_item = std::min(min_item, itemsize(o.dtype));
                ++n_vec_ops;
            }
        for (auto& st : grp.stores)
            if (!st.col_uniform) min_item = std::min(min_item, itemsize(st.dtype));
        int vec = 16 / min_item;
        while (vec > 1 && vec > DD) vec >>= 1;
        const bool ragged = DD % vec != 0;
        const int64_t vcols = (DD + vec - 1) / vec;
        int TX = 1;
        while (TX < 16 && TX < vcols) TX <<= 1;
        if (opt.tune_row_lanes > 0) {
            TX = opt.tune_row_lanes;
            if (TX & (TX - 1) || TX > 64) fail(PF_E_INVALID, "tune_row_lanes must be a power of two <= 64 for column reductions");
        }
        const int64_t CT = (vcols + TX - 1) / TX;
        const int64_t tiles = L * CT;
        bool any_var = false;
        for (int id : grp.nodes) any_var |= g.nodes[id].op == PF_OP_VAR;
        // Few (leading index, column tile) pairs and many rows: split the rows over SP workgroups per
        // tile.  Each writes its partial results to scratch memory; a second, small kernel combines
        // them and runs the epilogue.  (No waiting between workgroups anywhere.)
        int SP = 1;
        // (worth a second launch once an unsplit workgroup of 1024 lanes would walk eight or more rows per lane)
        if (tiles < 128 && S >= 8 * (1024 / TX) && !any_var)
            while (tiles * SP < 512 && S / (SP * 2) >= 32 && SP < 256) SP <<= 1;
        const int64_t SB = (S + SP - 1) / SP;          // rows per workgroup
        const int64_t blocks = tiles * SP;
        // lanes along S: enough workgroups x lanes to fill the chip, never more than rows
        int TY = 1024 / TX;
        while (TY > 1 && (TY / 2) * TX >= 64 && (TY > SB || blocks * TX * TY > (int64_t)512 * 1024)) TY >>= 1;
        if (opt.tune_col_block > 0) {
            if (opt.tune_col_block & (opt.tune_col_block - 1) || opt.tune_col_block > 1024 || opt.tune_col_block < 64 || opt.tune_col_block < TX)
                fail(PF_E_INVALID, "tune_col_block must be a power of two in [64, 1024], at least the lanes per row");
            TY = opt.tune_col_block / TX;
        }
        auto lds_bytes = [&](int ty) { return (int64_t)n_red_slots() * ((int64_t)(TX * ty / 64) + 1) * TX * vec * (precise ? 8 : 4); };
        while (TY > 1 && (TY / 2) * TX >= 64 && lds_bytes(TY) > 60 * 1024) TY >>= 1;
        if (lds_bytes(TY) > 64 * 1024) fail(PF_E_COMPILE, "column reduction group needs %lld bytes of LDS", (long long)lds_bytes(TY));
        const int block = TX * TY;
        // rows in flight per lane; at least four trips of the row loop measured best (B=32, S=512, D=1024:
        // 18.0 us with U = 2 against 18.9 us with U = 4 at 16 x 64 lanes)
        int U = 4;
        while (U > 1 && ((int64_t)U * TY * 4 > SB || U * vec * std::max(n_vec_ops, 1) > 64)) U >>= 1;
        if (opt.tune_row_unroll > 0) U = opt.tune_row_unroll;
        RU = U;
        NN = vec;
        const int W = TX * vec, NW = block / 64;
        grp.block = block;
        grp.grid = blocks;
        grp.lanes_per_row = TX;
        grp.vec = vec;
        grp.chunks_per_lane = U;
        const char* acc = precise ? "double" : "float";

        // reduction slots in LDS (a variance takes two: sum, then squared deviations)
        std::map<int, int> slot_of;
        int n_red = 0;
        for (int id : grp.nodes)
            if (is_reduction(g.nodes[id].op)) {
                slot_of[id] = n_red;
                n_red += g.nodes[id].op == PF_OP_VAR ? 2 : 1;
            }
        const bool split = SP > 1;
        if (split) {
            grp.scratch_bytes = (uint64_t)blocks * n_red * W * (precise ? 8 : 4);
            grp.kernel2_name = grp.kernel_name + "_fin";
            grp.grid2 = tiles;
            // the combining kernel: W columns x KP lanes along the partial results (all powers of two)
            int KP = 1;
            while (KP * 2 <= SP && W * KP * 2 <= 1024) KP <<= 1;
            while (W * KP < 64) KP <<= 1;
            grp.block2 = W * KP;
        }
        // operands that do not change along S are loaded once
        hoisted.clear();
        for (size_t oi = 0; oi < grp.operands.size(); ++oi)
            if (!grp.operands[oi].coluni && grp.operands[oi].stride[rd - 2] == 0) hoisted.insert((int)oi);

        const std::string extra = split ? strf("%s* __restrict__ scratch", acc) : "";
        signature(extra);
        line(strf("    constexpr int TX = %d, TY = %d, VEC = %d, U = %d, W = %d, NW = %d, BLOCK = %d, SP = %d, NRED = %d;", TX, TY, vec, U, W, NW, block,
                  SP, n_red));
        line(strf("    constexpr %s S = %lld, DD = %lld, CT = %lld, SB = %lld;", idx_t(), (long long)S, (long long)DD, (long long)CT, (long long)SB));
        line(strf("    __shared__ %s part[%d][NW][W];", acc, n_red));
        line(strf("    __shared__ %s tot[%d][W];", acc, n_red));
        line("    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX, wave = threadIdx.x >> 6;");
        if (split) {
            line(strf("    const %s seg = blockIdx.x %% SP, tile = blockIdx.x / SP;", idx_t()));
            line(strf("    const %s ct = tile %% CT, lead = tile / CT;", idx_t()));
            line(strf("    const %s s_begin = seg * SB, s_end = s_begin + SB < S ? s_begin + SB : S;   // may be empty for the last segments", idx_t()));
        } else {
            line(strf("    const %s ct = blockIdx.x %% CT, lead = blockIdx.x / CT;", idx_t()));
            line(strf("    constexpr %s s_begin = 0, s_end = S;", idx_t()));
        }
        line(strf("    const %s d0 = ct * W + (%s)tx * VEC;", idx_t(), idx_t()));
        // lanes whose columns lie outside still take part in shuffles and barriers; they read column block 0
        line(strf("    const bool col_ok = d0 < DD;"));
        line(strf("    const %s dc = col_ok ? d0 : 0;", idx_t()));
        emit_lead_decomposition("lead", nlead);
        auto load_vec = [&](size_t oi, const std::string& off, const std::string& dst, const char* ind) {
            const Operand& o = grp.operands[oi];
            const bool nt = numel(o.shape) * itemsize(o.dtype) >= (int64_t(1) << 22);
            if (ragged) {
                line(strf("%sif (dc + VEC <= DD) pf_ld<VEC, %s, true>(p%zu + %s + dc, %s);", ind, nt ? "true" : "false", oi, off.c_str(), dst.c_str()));
                line(strf("%selse { _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) (%s)[j] = pf_ld1(p%zu + %s + (dc + j < DD ? dc + j : DD - 1)); }", ind,
                          dst.c_str(), oi, off.c_str()));
            } else {
                line(strf("%spf_ld<VEC, %s>(p%zu + %s + dc, %s);", ind, nt ? "true" : "false", oi, off.c_str(), dst.c_str()));
            }
        };
        for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
            if (!hoisted.count((int)oi)) continue;
            const Operand& o = grp.operands[oi];
            std::string base = lead_offset_n(o, nlead);
            if (o.stride[rd - 1] == 0) line(strf("    float x%zu[1]; x%zu[0] = pf_ld1(p%zu + %s);", oi, oi, oi, base.c_str()));
            else {
                line(strf("    float x%zu[VEC];", oi));
                load_vec(oi, base, strf("x%zu", oi), "    ");
            }
        }
        for (int pass = 0; pass < (any_var ? 2 : 1); ++pass) {
            // accumulators of this pass
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (!is_reduction(n.op)) continue;
                if (pass == 0) {
                    if (n.op == PF_OP_MAX) line(strf("    float a%d[VEC]; _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) a%d[j] = -__builtin_inff();", id, id));
                    else line(strf("    %s a%d[VEC]; _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) a%d[j] = 0;", acc, id, id));
                } else if (n.op == PF_OP_VAR) {
                    line(strf("    %s mu%d[VEC], q%d[VEC];", acc, id, id));
                    line(strf("    _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) { mu%d[j] = tot[%d][tx * VEC + j] / (%s)%lld; q%d[j] = 0; }", id,
                              slot_of.at(id), acc, (long long)S, id));
                }
            }
            line(strf("    for (%s sb = s_begin + ty; sb < s_end; sb += (%s)TY * U) {   // pass %d", idx_t(), idx_t(), pass));
            line(strf("        %s row[U]; bool row_ok[U];", idx_t()));
            line(strf("        _Pragma(\"unroll\") for (int u = 0; u < U; ++u) { const %s t = sb + (%s)u * TY; row_ok[u] = t < s_end; row[u] = row_ok[u] ? t : s_end - 1; }",
                      idx_t(), idx_t()));
            for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
                const Operand& o = grp.operands[oi];
                if (o.coluni || hoisted.count((int)oi)) continue;
                std::string base = lead_offset_n(o, nlead);
                if (o.stride[rd - 1] == 0) {
                    line(strf("        float x%zu[U];", oi));
                    line(strf("        _Pragma(\"unroll\") for (int u = 0; u < U; ++u) x%zu[u] = pf_ld1(p%zu + %s + row[u] * %lld);", oi, oi, base.c_str(),
                              (long long)o.stride[rd - 2]));
                } else {
                    line(strf("        float x%zu[U * VEC];", oi));
                    line("        _Pragma(\"unroll\") for (int u = 0; u < U; ++u) {");
                    load_vec(oi, strf("%s + row[u] * %lld", base.c_str(), (long long)o.stride[rd - 2]), strf("&x%zu[u * VEC]", oi), "            ");
                    line("        }");
                }
            }
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (is_reduction(n.op)) {
                    const std::string xj = ref(id, n.in[0], "j");
                    const std::string open = "        _Pragma(\"unroll\") for (int u = 0; u < U; ++u) if (row_ok[u]) _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j)";
                    if (pass == 0) {
                        if (n.op == PF_OP_MAX) line(open + strf(" a%d[j] = pf_max_nan(a%d[j], %s);", id, id, xj.c_str()));
                        else line(open + strf(" a%d[j] += (%s)(%s);", id, acc, xj.c_str()));
                    } else if (n.op == PF_OP_VAR) {
                        line(open + strf(" { const %s d = (%s)(%s) - mu%d[j]; q%d[j] += d * d; }", acc, acc, xj.c_str(), id, id));
                    }
                    continue;
                }
                if (plan_kind.at(id) == 2) emit_elementwise(id, vec);
            }
            if (pass == 0) {
                int sp = 0;
                for (auto& st : grp.stores) {
                    const int cnt = 1 + (int)st.also_outputs.size();
                    if (!st.col_uniform)
                        for (int c = 0; c < cnt; ++c) {
                            const bool nt = numel(st.shape) * itemsize(st.dtype) >= (int64_t(1) << 22);
                            line("        _Pragma(\"unroll\") for (int u = 0; u < U; ++u) if (row_ok[u] && col_ok) {");
                            line(strf("            const %s o = (lead * S + row[u]) * DD + d0;", idx_t()));
                            if (ragged) {
                                line(strf("            if (d0 + VEC <= DD) pf_st<VEC, %s, true>(q%d + o, &v%d[u * VEC]);", nt ? "true" : "false", sp + c, st.node));
                                line(strf("            else { _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) if (d0 + j < DD) pf_st1(q%d + o + j, v%d[u * VEC + j]); }",
                                          sp + c, st.node));
                            } else {
                                line(strf("            pf_st<VEC, %s>(q%d + o, &v%d[u * VEC]);", nt ? "true" : "false", sp + c, st.node));
                            }
                            line("        }");
                        }
                    sp += cnt;
                }
            }
            line("    }");
            // combine: across ty inside a wave by shuffles, across waves in LDS
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (!is_reduction(n.op)) continue;
                if (pass == 1 && n.op != PF_OP_VAR) continue;
                const int sl = slot_of.at(id) + pass;
                const std::string a = strf(pass == 0 ? "a%d" : "q%d", id);
                const bool mx = n.op == PF_OP_MAX;
                line("    _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) {");
                line(strf("        %s t = %s[j];", mx ? "float" : acc, a.c_str()));
                if (TX < 64) {
                    if (mx) line("        _Pragma(\"unroll\") for (int m = TX; m < 64; m <<= 1) t = pf_max_nan(t, __shfl_xor(t, m, 64));");
                    else line("        _Pragma(\"unroll\") for (int m = TX; m < 64; m <<= 1) t += __shfl_xor(t, m, 64);");
                }
                line(strf("        if ((threadIdx.x & 63) < TX) part[%d][wave][tx * VEC + j] = t;", sl));
                line("    }");
            }
            line("    __syncthreads();");
            line("    for (int c = threadIdx.x; c < W; c += BLOCK) {");
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (!is_reduction(n.op)) continue;
                if (pass == 1 && n.op != PF_OP_VAR) continue;
                const int sl = slot_of.at(id) + pass;
                // with TX == 64 a wave holds one ty; otherwise 64 / TX of them, already combined
                if (n.op == PF_OP_MAX) {
                    line(strf("        { float t = (float)part[%d][0][c]; for (int w = 1; w < NW; ++w) t = pf_max_nan(t, (float)part[%d][w][c]); tot[%d][c] = t; }",
                              sl, sl, sl));
                } else {
                    line(strf("        { %s t = part[%d][0][c]; for (int w = 1; w < NW; ++w) t += part[%d][w][c]; tot[%d][c] = t; }", acc, sl, sl, sl));
                }
            }
            line("    }");
            line("    __syncthreads();");
        }
        // epilogue: lane c finishes column c of this workgroup's W columns
        RU = 1;
        auto emit_epilogue = [&](const std::function<std::string(int)>& total) {
            line(strf("        const %s col = ct * W + c;", idx_t()));
            line("        if (col >= DD) continue;");
            line("        constexpr int u = 0; (void)u;");
            for (int id : grp.nodes) {
                const Node& n = g.nodes[id];
                if (!is_reduction(n.op)) continue;
                const int sl = slot_of.at(id);
                if (n.op == PF_OP_SUM || n.op == PF_OP_MAX) line(strf("        float s%d[1]; s%d[0] = (float)%s;", id, id, total(sl).c_str()));
                else if (n.op == PF_OP_MEAN) line(strf("        float s%d[1]; s%d[0] = (float)(%s / (%s)%lld);", id, id, total(sl).c_str(), acc, (long long)S));
                else line(strf("        float s%d[1]; s%d[0] = (float)(%s / (%s)%lld);", id, id, total(sl + 1).c_str(), acc, (long long)(S - n.correction)));
            }
            for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
                const Operand& o = grp.operands[oi];
                if (!o.coluni) continue;
                line(strf("        float x%zu[1]; x%zu[0] = pf_ld1(p%zu + %s + col * %lld);", oi, oi, oi, lead_offset_n(o, nlead).c_str(),
                          (long long)o.stride[rd - 1]));
            }
            for (int id : grp.nodes)
                if (epilogue_node(id)) emit_elementwise(id, 1);
            int sp = 0;
            for (auto& st : grp.stores) {
                const int cnt = 1 + (int)st.also_outputs.size();
                if (st.col_uniform)
                    for (int c = 0; c < cnt; ++c) line(strf("        pf_st1(q%d + lead * DD + col, s%d[0]);", sp + c, st.node));
                sp += cnt;
            }
        };
        if (!split) {
            line("    for (int c = threadIdx.x; c < W; c += BLOCK) {");
            emit_epilogue([](int sl) { return strf("tot[%d][c]", sl); });
            line("    }");
            line("}");
            return;
        }
        // split rows: publish this workgroup's partial results ...
        line("    for (int c = threadIdx.x; c < W; c += BLOCK)");
        line(strf("        _Pragma(\"unroll\") for (int r = 0; r < NRED; ++r) scratch[(((%s)tile * SP + seg) * NRED + r) * W + c] = tot[r][c];", idx_t()));
        line("}");
        // ... and combine them, one workgroup per (leading index, column tile), one lane per column
        const std::string name1 = grp.kernel_name;
        grp.kernel_name = grp.kernel2_name;
        const int block1 = grp.block;
        grp.block = grp.block2;
        signature(strf("const %s* __restrict__ scratch", acc));
        grp.kernel_name = name1;
        grp.block = block1;
        line(strf("    constexpr int W = %d, SP = %d, NRED = %d, BLOCK = %d, KP = BLOCK / W;", W, SP, n_red, grp.block2));
        line(strf("    constexpr %s DD = %lld, CT = %lld;", idx_t(), (long long)DD, (long long)CT));
        line(strf("    const %s tile = blockIdx.x, ct = tile %% CT, lead = tile / CT;", idx_t()));
        emit_lead_decomposition("lead", nlead);
        // lane (kk, c) folds partial results kk, kk + KP, ... of column c; LDS then folds the KP lanes of a column
        line(strf("    __shared__ %s red[NRED][KP][W];", acc));
        line("    {");
        line("        const int c = threadIdx.x % W, kk = threadIdx.x / W;");
        for (int id : grp.nodes) {
            const Node& n = g.nodes[id];
            if (!is_reduction(n.op)) continue;
            const int sl = slot_of.at(id);
            const std::string at = strf("scratch[(((%s)tile * SP + k) * NRED + %d) * W + c]", idx_t(), sl);
            if (n.op == PF_OP_MAX)
                line(strf("        { float t = -__builtin_inff(); _Pragma(\"unroll 4\") for (int k = kk; k < SP; k += KP) t = pf_max_nan(t, (float)%s); red[%d][kk][c] = t; }",
                          at.c_str(), sl));
            else
                line(strf("        { %s t = 0; _Pragma(\"unroll 4\") for (int k = kk; k < SP; k += KP) t += %s; red[%d][kk][c] = t; }", acc, at.c_str(), sl));
        }
        line("    }");
        line("    __syncthreads();");
        line("    for (int c = threadIdx.x; c < W; c += BLOCK) {");
        line(strf("        %s fin[NRED];", acc));
        for (int id : grp.nodes) {
            const Node& n = g.nodes[id];
            if (!is_reduction(n.op)) continue;
            const int sl = slot_of.at(id);
            if (n.op == PF_OP_MAX)
                line(strf("        { float t = (float)red[%d][0][c]; for (int q = 1; q < KP; ++q) t = pf_max_nan(t, (float)red[%d][q][c]); fin[%d] = t; }", sl, sl, sl));
            else
                line(strf("        { %s t = red[%d][0][c]; for (int q = 1; q < KP; ++q) t += red[%d][q][c]; fin[%d] = t; }", acc, sl, sl, sl));
        }
        emit_epilogue([](int sl) { return strf("fin[%d]", sl); });
        line("    }");
        line("}");
    }

    int n_red_slots() const {
        int n = 0;
        for (int id : grp.nodes)
            if (is_reduction(g.nodes[id].op)) n += g.nodes[id].op == PF_OP_VAR ? 2 : 1;
        return n;
    }
    int operand_kind_pre(const Operand& o) const { return rd > 0 && (o.stride[rd - 1] != 0 || grp.cols == 1) ? 2 : 1; }

    // ================================================================ EW_FLAT
    void gen_flat() {
        const int64_t C = grp.cols, R = grp.rows, N = C * R;
        int min_item = 4;
        for (auto& o : grp.operands) min_item = std::min(min_item, itemsize(o.dtype));
        for (auto& st : grp.stores) min_item = std::min(min_item, itemsize(st.dtype));
        const int vec = 16 / min_item;
        // aligned: a vector never crosses a row, so broadcast operands are uniform or
        // contiguous inside it; otherwise vectors run over the flat index and
        // operands that are not plain contiguous are gathered per element
        bool all_flat = true;
        for (auto& o : grp.operands)
            if (!is_contiguous_full(o) && numel(o.shape) != 1) all_flat = false;
        straddle = (C % vec) != 0;
        const bool tail = straddle && (N % vec) != 0;
        // one vector per lane and many small workgroups measured fastest on MI355X (80% of
        // peak HBM bandwidth on bf16 [8192,11008] against 73% with four vectors per lane)
        const int U = opt.tune_flat_unroll > 0 ? opt.tune_flat_unroll : 1;
        const int block = 256;
        const int64_t nvec = (N + vec - 1) / vec;
        grp.block = block;
        grp.grid = (nvec + (int64_t)block * U - 1) / ((int64_t)block * U);
        if (rd >= 2 && !straddle) {                           // whole vectors per row: no tail code to depend on the element count
            grp.rt_per_outer = inner_rows() * C;
            grp.rt_per_block = (int64_t)vec * block * U;
            grp.rt_rows_per_outer = inner_rows();
        }
        grp.vec = vec;
        grp.chunks_per_lane = U;
        grp.lanes_per_row = 0;
        (void)all_flat;

        // re-evaluate kinds now that straddle is known
        recompute_kinds();
        RU = 1;
        NN = vec;

        // body as a device function of the vector index
        // the outermost extent is a kernel argument (see the row template)
        set_outer_runtime();
        line(strf("template <bool TAIL> PF_DEV void body(%s, %s v, const %s NEL) {", param_list().c_str(), idx_t(), idx_t()));
        line(strf("    constexpr int VEC = %d;", vec));
        line(strf("    constexpr %s C = %lld;", idx_t(), (long long)C));
        line(strf("    const %s e0 = v * VEC;", idx_t()));
        if (!straddle) {
            line(strf("    const %s row = e0 / C, col0 = e0 %% C;", idx_t()));
            emit_row_decomposition("row");
        }
        for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
            const Operand& o = grp.operands[oi];
            const bool nt = numel(o.shape) * itemsize(o.dtype) >= (int64_t(1) << 22);
            if (!straddle) {
                std::string base = lead_offset(o, "row");
                if (operand_kind((int)oi) == 1) line(strf("    const float x%zu[1] = {pf_ld1(p%zu + %s)};", oi, oi, base.c_str()));
                else if (last_mapped(o)) {
                    line(strf("    float x%zu[VEC];", oi));
                    line(strf("    _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) x%zu[j] = pf_ld1(p%zu + %s + %s * %lld);", oi, oi, base.c_str(),
                              mapexpr(o, rd - 1, "(col0 + j)").c_str(), (long long)o.stride[rd - 1]));
                } else {
                    line(strf("    float x%zu[VEC];", oi));
                    line(strf("    pf_ld<VEC, %s>(p%zu + %s + col0, x%zu);", nt ? "true" : "false", oi, base.c_str(), oi));
                }
                continue;
            }
            line(strf("    float x%zu[VEC];", oi));
            if (is_contiguous_full(o)) {
                line(strf("    if (!TAIL) pf_ld<VEC, %s>(p%zu + e0, x%zu);", nt ? "true" : "false", oi, oi));
                line(strf("    else { _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) x%zu[j] = (e0 + j < NEL) ? pf_ld1(p%zu + e0 + j) : 0.0f; }",
                          oi, oi));
            } else {
                line("    _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) {");
                line(strf("        const %s e = (TAIL && e0 + j >= NEL) ? NEL - 1 : e0 + j;", idx_t()));
                line(strf("        const %s row = e / C, col = e %% C;", idx_t()));
                std::string off = element_offset(o, "row", "col");
                line(strf("        x%zu[j] = pf_ld1(p%zu + %s);", oi, oi, off.c_str()));
                line("    }");
            }
        }
        for (int id : grp.nodes) emit_elementwise(id, vec);
        int sp = 0;
        for (auto& st : grp.stores) {
            const bool nt = numel(st.shape) * itemsize(st.dtype) >= (int64_t(1) << 22);
            int cnt = 1 + (int)st.also_outputs.size();
            for (int c = 0; c < cnt; ++c, ++sp) {
                line(strf("    if (!TAIL) pf_st<VEC, %s>(q%d + e0, v%d);", nt ? "true" : "false", sp, st.node));
                line(strf("    else { _Pragma(\"unroll\") for (int j = 0; j < VEC; ++j) if (e0 + j < NEL) pf_st1(q%d + e0 + j, v%d[j]); }",
                          sp, st.node));
            }
        }
        line("}");
        signature(outer_param());
        line(strf("    constexpr int U = %d, BLOCK = %d;", U, block));
        if (grp.outer_runtime) {
            line(strf("    const %s NEL = (%s)pf_d0 * %lld, NVEC = (NEL + %d) / %d;", idx_t(), idx_t(), (long long)(inner_rows() * C), vec - 1, vec));
        } else
        line(strf("    constexpr %s NEL = %lld, NVEC = %lld;", idx_t(), (long long)N, (long long)nvec));
        line(strf("    const %s v0 = (%s)blockIdx.x * (BLOCK * U) + threadIdx.x;", idx_t(), idx_t()));
        std::string args = arg_list();
        if (tail) {
            line("    _Pragma(\"unroll\") for (int u = 0; u < U; ++u) {");
            line(strf("        const %s v = v0 + (%s)u * BLOCK;", idx_t(), idx_t()));
            line(strf("        if (v + 1 < NVEC) body<false>(%s, v, NEL); else if (v < NVEC) body<true>(%s, v, NEL);", args.c_str(), args.c_str()));
            line("    }");
        } else {
            line(strf("    if (v0 + (%s)(U - 1) * BLOCK < NVEC) {", idx_t()));
            line(strf("        _Pragma(\"unroll\") for (int u = 0; u < U; ++u) body<false>(%s, v0 + (%s)u * BLOCK, NEL);", args.c_str(), idx_t()));
            line("    } else {");
            line("        _Pragma(\"unroll\") for (int u = 0; u < U; ++u) {");
            line(strf("            const %s v = v0 + (%s)u * BLOCK;", idx_t(), idx_t()));
            line(strf("            if (v < NVEC) body<false>(%s, v, NEL);", args.c_str()));
            line("        }");
            line("    }");
        }
        line("}");
    }

    // ================================================================ TILE
    void gen_tile() {
        if (rd < 2) fail(PF_E_COMPILE, "internal: tiled group of rank < 2");
        const int64_t C = grp.domain[rd - 1], R = grp.domain[rd - 2];
        int64_t L = 1;
        for (int k = 0; k < rd - 2; ++k) L *= grp.domain[k];
        // Tile edge: 64 (16 elements per lane: long contiguous runs on both sides), or 32 (4 elements per
        // lane) while 64-wide tiles would leave the chip short of waves: a small problem is bound by the
        // chain of instructions each wave runs on its own, and four times as many waves with a quarter
        // of the work each cut that chain (heavy epilogues on 1.5 M elements: 21 us -> 16 us measured).
        int64_t t64 = L * ((R + 63) / 64) * ((C + 63) / 64);
        int n_compute = 0;
        for (int id : grp.nodes) n_compute += g.nodes[id].op != PF_OP_TRANSPOSE;
        // plain transposes of 5 MB and more run up to 25% faster with 64-wide tiles; with an epilogue of several
        // operators the shorter instruction chain per wave still wins at four times that size
        const int64_t few_tiles = n_compute <= 1 ? 512 : n_compute <= 3 ? 2048 : n_compute <= 6 ? 4096 : 8192;
        int n_t = 0;
        for (auto& o : grp.operands) n_t += o.transposed ? 1 : 0;
        // every transposed operand is staged through a padded LDS tile of its own; a workgroup may declare 64 KB
        auto lds_bytes = [&](int ts) { return (int64_t)std::max(n_t, 1) * ts * (ts + 1) * 4; };
        int TS = (t64 < few_tiles || lds_bytes(64) > 64 * 1024) ? 32 : 64;
        if (opt.tune_tile_edge > 0) {
            if (opt.tune_tile_edge != 32 && opt.tune_tile_edge != 64) fail(PF_E_INVALID, "tune_tile_edge must be 32 or 64");
            if (lds_bytes(opt.tune_tile_edge) <= 64 * 1024) TS = opt.tune_tile_edge;
        }
        if (lds_bytes(TS) > 64 * 1024)
            fail(PF_E_COMPILE, "a tiled group with %d transposed operands needs %lld bytes of LDS", n_t, (long long)lds_bytes(TS));
        // 16-byte accesses on both sides: four fp32 elements per lane and row, eight when every tensor of the
        // group holds 16-bit elements (64-wide tiles only: a 32-wide tile of eight-element vectors has no
        // whole pass of 256 lanes); 8192 x 8192 bf16 went from 4.4 to 4.7 TB/s
        int min_item = 4;
        for (auto& o : grp.operands) min_item = std::min(min_item, itemsize(o.dtype));
        for (auto& st : grp.stores) min_item = std::min(min_item, itemsize(st.dtype));
        bool all_16bit = min_item == 2;
        for (auto& o : grp.operands) if (numel(o.shape) > 1 && itemsize(o.dtype) != 2 && o.stride[rd - 1] != 0) all_16bit = false;
        for (auto& st : grp.stores) if (itemsize(st.dtype) != 2) all_16bit = false;
        const int VW = (TS == 64 && all_16bit) ? 8 : 4;
        const int TXN = TS / VW, TYN = 256 / TXN, NI = TS / TYN, EPL = NI * VW;  // lanes along a row, rows per pass, passes, elements per lane
        const int64_t tr = (R + TS - 1) / TS, tc = (C + TS - 1) / TS;
        grp.block = 256;
        // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Runs of G consecutive
        // tiles go to the same XCD, so tiles that share cache lines (rows whose length is no multiple
        // of a line) meet in one L2 instead of being fetched and written back twice, while the XCDs
        // still work on neighbouring regions (one long run per XCD put them a power-of-two stride
        // apart on square shapes and cost 15%).
        const int64_t tiles = L * tr * tc;
        const int G = opt.tune_flat_unroll > 0 ? opt.tune_flat_unroll : 16;   // 8...32 measured within 4% of each other
        const bool xcd_remap = tiles >= 64 && G > 1;
        const int64_t rounds = (tiles + 8 * G - 1) / (8 * G);
        grp.grid = xcd_remap ? rounds * 8 * G : tiles;
        grp.vec = VW;
        grp.chunks_per_lane = NI;
        grp.lanes_per_row = 0;
        RU = 1;
        NN = EPL;

        signature();
        line(strf("    constexpr %s C = %lld, R = %lld, TR = %lld, TC = %lld;", idx_t(), (long long)C, (long long)R, (long long)tr,
                  (long long)tc));
        line(strf("    constexpr int TS = %d, TXN = %d, TYN = %d, NI = %d, VW = %d;", TS, TXN, TYN, NI, VW));
        line(strf("    __shared__ float tile[%d][TS][TS + 1];", std::max(n_t, 1)));
        if (xcd_remap) {
            line(strf("    const %s slot = blockIdx.x / 8;", idx_t()));
            line(strf("    const %s b = ((slot / %d) * 8 + blockIdx.x %% 8) * %d + slot %% %d;", idx_t(), G, G, G));
            line(strf("    if (b >= %lld) return;", (long long)tiles));
        } else {
            line(strf("    const %s b = blockIdx.x;", idx_t()));
        }
        line(strf("    const %s tcol = b %% TC, trow = (b / TC) %% TR, lead = b / (TC * TR);", idx_t()));
        line(strf("    const %s r0 = trow * TS, c0 = tcol * TS;", idx_t()));
        line("    const int tx = threadIdx.x % TXN, ty = threadIdx.x / TXN;");
        emit_lead_decomposition("lead", rd - 2);
        // stage transposed operands through LDS: memory is [.., C, R] with R contiguous
        int ti = 0;
        for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
            const Operand& o = grp.operands[oi];
            if (!o.transposed) continue;
            std::string base = lead_offset_n(o, rd - 2);
            const bool vec_ok = (R % VW == 0) && lead_strides_multiple_of(o, VW, rd - 2);
            line("    _Pragma(\"unroll\") for (int i = 0; i < NI; ++i) {");
            line(strf("        const %s cc = c0 + ty + TYN * i, rr = r0 + tx * VW;", idx_t()));
            line("        float t4[VW];");
            line("        _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) t4[j] = 0.0f;");
            if (vec_ok) {
                line(strf("        if (cc < C && rr < R) pf_ld<VW, false>(p%zu + %s + cc * R + rr, t4);", oi, base.c_str()));
            } else {
                // rows of a length that is no multiple of four: full vectors at element alignment, scalars at the row end
                line(strf("        if (cc < C && rr + VW <= R) pf_ld<VW, false, true>(p%zu + %s + cc * R + rr, t4);", oi, base.c_str()));
                line(strf("        else if (cc < C) { _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) if (rr + j < R) t4[j] = pf_ld1(p%zu + %s + cc * R + rr + j); }",
                          oi, base.c_str()));
            }
            line(strf("        _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) tile[%d][ty + TYN * i][tx * VW + j] = t4[j];", ti));
            line("    }");
            ++ti;
        }
        if (n_t) line("    __syncthreads();");
        ti = 0;
        for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
            const Operand& o = grp.operands[oi];
            line(strf("    float x%zu[%d];", oi, EPL));
            if (o.transposed) {
                line("    _Pragma(\"unroll\") for (int i = 0; i < NI; ++i)");
                line(strf("        _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) x%zu[i * VW + j] = tile[%d][tx * VW + j][ty + TYN * i];", oi, ti));
                ++ti;
                continue;
            }
            std::string base = lead_offset_n(o, rd - 2);
            const int64_t sr = o.stride[rd - 2], sc = o.stride[rd - 1];
            const bool vec_ok = sc == 1 && (C % VW == 0) && (sr % VW == 0) && lead_strides_multiple_of(o, VW, rd - 2) && !o.mapped(rd - 1) &&
                                o.const_offset % VW == 0;
            line("    _Pragma(\"unroll\") for (int i = 0; i < NI; ++i) {");
            line(strf("        const %s rr = r0 + ty + TYN * i, cc = c0 + tx * VW;", idx_t()));
            line(strf("        const %s rc = rr < R ? rr : R - 1;", idx_t()));
            if (vec_ok) {
                line(strf("        if (cc < C) pf_ld<VW, false>(p%zu + %s + %s * %lld + cc, &x%zu[i * VW]);", oi, base.c_str(),
                          mapexpr(o, rd - 2, "rc").c_str(), (long long)sr, oi));
                line(strf("        else { _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) x%zu[i * VW + j] = 0.0f; }", oi));
            } else {
                const bool ua_ok = sc == 1 && !o.mapped(rd - 1);     // contiguous along the row, merely not 16-byte aligned
                if (ua_ok)
                    line(strf("        if (cc + VW <= C) pf_ld<VW, false, true>(p%zu + %s + %s * %lld + cc, &x%zu[i * VW]); else", oi, base.c_str(),
                              mapexpr(o, rd - 2, "rc").c_str(), (long long)sr, oi));
                line("        _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) {");
                line(strf("            const %s cj = cc + j < C ? cc + j : C - 1;", idx_t()));
                line(strf("            x%zu[i * VW + j] = pf_ld1(p%zu + %s + %s * %lld + %s * %lld);", oi, oi, base.c_str(),
                          mapexpr(o, rd - 2, "rc").c_str(), (long long)sr, mapexpr(o, rd - 1, "cj").c_str(), (long long)sc));
                line("        }");
            }
            line("    }");
        }
        for (int id : grp.nodes)
            if (plan_kind.at(id) != 4) emit_elementwise(id, EPL);
        int sp = 0;
        const bool st_vec = C % VW == 0;
        for (auto& st : grp.stores) {
            int cnt = 1 + (int)st.also_outputs.size();
            if (st.tstore) {
                // A result of the other orientation: memory is [.., C, R] with R contiguous.  The lanes' values go through
                // the LDS tile the other way round from a transposed load: written as computed, read back transposed,
                // stored coalesced along R.  (The tile is free by now: every staged operand sits in registers; the
                // barriers keep the uses of the tile apart.)
                const bool tv_ok = R % VW == 0;
                line("    __syncthreads();");
                line("    _Pragma(\"unroll\") for (int i = 0; i < NI; ++i)");
                line(strf("        _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) tile[0][tx * VW + j][ty + TYN * i] = v%d[i * VW + j];", st.value_node));
                line("    __syncthreads();");
                for (int c = 0; c < cnt; ++c, ++sp) {
                    line("    _Pragma(\"unroll\") for (int i = 0; i < NI; ++i) {");
                    line(strf("        const %s cc = c0 + ty + TYN * i, rr = r0 + tx * VW;", idx_t()));
                    line("        float t4[VW];");
                    line("        _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) t4[j] = tile[0][ty + TYN * i][tx * VW + j];");
                    line(strf("        const %s o = (lead * C + cc) * R + rr;", idx_t()));
                    if (tv_ok) line(strf("        if (cc < C && rr < R) pf_st<VW, false>(q%d + o, t4);", sp));
                    else {
                        line(strf("        if (cc < C && rr + VW <= R) pf_st<VW, false, true>(q%d + o, t4);", sp));
                        line(strf("        else if (cc < C) { _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) if (rr + j < R) pf_st1(q%d + o + j, t4[j]); }", sp));
                    }
                    line("    }");
                }
                continue;
            }
            for (int c = 0; c < cnt; ++c, ++sp) {
                line("    _Pragma(\"unroll\") for (int i = 0; i < NI; ++i) {");
                line(strf("        const %s rr = r0 + ty + TYN * i, cc = c0 + tx * VW;", idx_t()));
                line(strf("        const %s o = (lead * R + rr) * C + cc;", idx_t()));
                if (st_vec) line(strf("        if (rr < R && cc < C) pf_st<VW, false>(q%d + o, &v%d[i * VW]);", sp, st.node));
                else {
                    line(strf("        if (rr < R && cc + VW <= C) pf_st<VW, false, true>(q%d + o, &v%d[i * VW]);", sp, st.node));
                    line(strf("        else if (rr < R) { _Pragma(\"unroll\") for (int j = 0; j < VW; ++j) if (cc + j < C) pf_st1(q%d + o + j, v%d[i * VW + j]); }",
                              sp, st.node));
                }
                line("    }");
            }
        }
        line("}");
    }

    // ---------------------------------------------------------------- addressing
    bool is_contiguous_full(const Operand& o) const {
        if (o.transposed || any_mapped(o, rd)) return false;
        int64_t st = 1;
        for (int k = rd - 1; k >= 0; --k) {
            if (grp.domain[k] != 1 && o.stride[k] != st) return false;
            st *= grp.domain[k];
        }
        return true;
    }
    bool lead_strides_multiple_of(const Operand& o, int m, int nlead) const {
        for (int k = 0; k < nlead; ++k)
            if (o.stride[k] % m) return false;
        return true;
    }
    bool need_decomp = false;
    int decomp_dims = 0;

    // index of dim k as the source tensor sees it: roll / slice steps applied to the consumer's index
    std::string mapexpr(const Operand& o, int k, const std::string& idx) const {
        std::string e = idx;
        for (auto& st : o.steps[k]) {
            if (st.mod) e = strf("((%s + %lld) %% %lld)", e.c_str(), (long long)st.add, (long long)st.mod);
            else e = strf("(%s + %lld)", e.c_str(), (long long)st.add);
        }
        return e;
    }
    bool any_mapped(const Operand& o, int nlead) const {
        for (int k = 0; k < nlead; ++k)
            if (o.mapped(k)) return true;
        return false;
    }
    bool last_mapped(const Operand& o) const { return rd > 0 && o.mapped(rd - 1); }

    // can the leading offset be written as row * stride? (strides nest like the domain)
    bool lead_mergeable(const Operand& o, int nlead) const {
        if (any_mapped(o, nlead)) return false;
        for (int k = 0; k + 1 < nlead; ++k)
            if (o.stride[k] != o.stride[k + 1] * grp.domain[k + 1]) return false;
        return true;
    }
    bool lead_zero(const Operand& o, int nlead) const {
        for (int k = 0; k < nlead; ++k)
            if (o.stride[k] != 0) return false;
        return true;
    }
    void scan_decomp(int nlead) {
        need_decomp = false;
        for (auto& o : grp.operands)
            if (!lead_zero(o, nlead) && !lead_mergeable(o, nlead)) need_decomp = true;
        decomp_dims = nlead;
    }
    // emits i0..i{n-1} from a flat index over the leading dims
    void emit_lead_decomposition(const std::string& var, int nlead) {
        scan_decomp(nlead);
        if (!need_decomp) return;
        std::string cur = var;
        for (int k = nlead - 1; k >= 0; --k) {
            if (k == 0) {
                line(strf("    const %s i0 = %s;", idx_t(), cur.c_str()));
            } else {
                line(strf("    const %s i%d = %s %% %lld; const %s t%d = %s / %lld;", idx_t(), k, cur.c_str(), (long long)grp.domain[k],
                          idx_t(), k, cur.c_str(), (long long)grp.domain[k]));
                cur = strf("t%d", k);
            }
        }
    }
    void emit_row_decomposition(const std::string& var) { emit_lead_decomposition(var, rd > 0 ? rd - 1 : 0); }

    std::string lead_offset_n(const Operand& o, int nlead) const {
        if (lead_zero(o, nlead)) return strf("(%s)0", idx_t());
        if (lead_mergeable(o, nlead)) return strf("%s * %lld", nlead == rd - 1 ? row_var.c_str() : "lead", (long long)o.stride[nlead - 1]);
        std::string e;
        for (int k = 0; k < nlead; ++k) {
            if (!o.stride[k]) continue;
            if (!e.empty()) e += " + ";
            e += strf("%s * %lld", mapexpr(o, k, strf("i%d", k)).c_str(), (long long)o.stride[k]);
        }
        return "(" + e + ")";
    }
    // row template: offset of row u of the team's row group (outer indices shared, inner index + u)
    std::string lead_offset_row_u(const Operand& o, int nlead) const {
        std::string e;
        for (int k = 0; k < nlead; ++k) {
            if (!o.stride[k]) continue;
            if (!e.empty()) e += " + ";
            const std::string idx = k == nlead - 1 ? strf("(i%d + (%s)u)", k, idx_t()) : strf("i%d", k);
            e += strf("%s * %lld", mapexpr(o, k, idx).c_str(), (long long)o.stride[k]);
        }
        return e.empty() ? strf("(%s)0", idx_t()) : "(" + e + ")";
    }
    std::string row_var = "row";
    std::string lead_offset(const Operand& o, const std::string& rv) {
        row_var = rv;
        return lead_offset_n(o, rd > 0 ? rd - 1 : 0);
    }
    // offset of one element from (row, col) without pre-computed indices (gather path)
    std::string element_offset(const Operand& o, const std::string& rv, const std::string& cv) const {
        const int nlead = rd > 0 ? rd - 1 : 0;
        std::string e = strf("%s * %lld", rd > 0 ? mapexpr(o, rd - 1, cv).c_str() : cv.c_str(), rd > 0 ? (long long)o.stride[rd - 1] : 0LL);
        if (lead_zero(o, nlead)) return e;
        if (lead_mergeable(o, nlead)) return e + strf(" + %s * %lld", rv.c_str(), (long long)o.stride[nlead - 1]);
        // decompose inline
        std::string cur = rv;
        for (int k = nlead - 1; k >= 0; --k) {
            if (k == 0) e += strf(" + %s * %lld", mapexpr(o, 0, "(" + cur + ")").c_str(), (long long)o.stride[0]);
            else {
                e += strf(" + %s * %lld", mapexpr(o, k, strf("((%s) %% %lld)", cur.c_str(), (long long)grp.domain[k])).c_str(),
                          (long long)o.stride[k]);
                cur = strf("((%s) / %lld)", cur.c_str(), (long long)grp.domain[k]);
            }
        }
        return e;
    }

    // ---------------------------------------------------------------- signature
    std::string param_list() const {
        std::string p;
        for (size_t oi = 0; oi < grp.operands.size(); ++oi)
            p += strf("%sconst %s* __restrict__ p%zu", oi ? ", " : "", ctype(grp.operands[oi].dtype), oi);
        int sp = 0;
        for (auto& st : grp.stores)
            for (size_t c = 0; c < 1 + st.also_outputs.size(); ++c, ++sp)
                p += strf("%s%s* __restrict__ q%d", p.empty() ? "" : ", ", ctype(st.dtype), sp);
        return p;
    }
    std::string arg_list() const {
        std::string p;
        for (size_t oi = 0; oi < grp.operands.size(); ++oi) p += strf("%sp%zu", oi ? ", " : "", oi);
        int sp = 0;
        for (auto& st : grp.stores)
            for (size_t c = 0; c < 1 + st.also_outputs.size(); ++c, ++sp) p += strf("%sq%d", p.empty() ? "" : ", ", sp);
        return p;
    }
    // Flat and row kernels take the outermost extent of their domain as an argument when the domain
    // has leading dims at all; everything else stays literal.
    void set_outer_runtime() {
        grp.outer_runtime = rd >= 2;
        grp.outer_extent = rd >= 2 ? grp.domain[0] : 0;
    }
    int64_t inner_rows() const {       // rows per index of the outermost dim
        int64_t r = 1;
        for (int k = 1; k + 1 < rd; ++k) r *= grp.domain[k];
        return r;
    }
    std::string outer_param() const { return grp.outer_runtime ? "const long long pf_d0" : ""; }
    void signature(const std::string& extra = "") {
        std::string params = param_list();
        if (!extra.empty()) params += (params.empty() ? "" : ", ") + extra;
        line(strf("extern \"C\" __global__ void __launch_bounds__(%d) %s(%s) {", grp.block, grp.kernel_name.c_str(), params.c_str()));
        for (size_t oi = 0; oi < grp.operands.size(); ++oi)     // source dims a sliced window pins to one index
            if (grp.operands[oi].const_offset) line(strf("    p%zu += %lld;", oi, (long long)grp.operands[oi].const_offset));
    }

    void recompute_kinds() {
        kind.clear();
        for (int id : grp.nodes) kind[id] = node_kind(id);
    }

    void run(int index) {
        rd = (int)grp.domain.size();
        for (int id : grp.nodes) members.insert(id);
        for (size_t m = 0; m < grp.nodes.size(); ++m) plan_kind[grp.nodes[m]] = m < grp.node_kind.size() ? grp.node_kind[m] : 2;
        for (size_t oi = 0; oi < grp.operands.size(); ++oi) {
            if (grp.operands[oi].coluni) coperand_of[grp.operands[oi].node] = (int)oi;
            else if (grp.operands[oi].view >= 0) voperand_of[grp.operands[oi].view] = (int)oi;
            else if (grp.operands[oi].via_transpose) toperand_of[grp.operands[oi].node] = (int)oi;
            else operand_of[grp.operands[oi].node] = (int)oi;
        }
        // a transpose that moves no data is planned as a plain operand
        int64_t maxel = numel(grp.domain);
        for (auto& o : grp.operands) maxel = std::max(maxel, numel(o.shape));
        wide = maxel >= (int64_t(1) << 30);
        for (int o : g.outputs)
            if (g.nodes[o].dtype == PF_F32) precise = true;
        for (auto& st : grp.stores)
            if (st.tstore && grp.tmpl != PF_T_TILE) fail(PF_E_COMPILE, "internal: a transposed store outside a tiled group");
        if (grp.tmpl == PF_T_TILE) {
            bool any_t = false;
            for (auto& o : grp.operands) any_t |= o.transposed;
            for (auto& st : grp.stores) any_t |= st.tstore;
            if (!any_t) grp.tmpl = PF_T_EW_FLAT;
        }
        // name: template + operators (+ a hash of the specialised source, added below), so
        // that a profile tells kernels of different subgraphs apart
        grp.kernel_name = "PFKNAME";
        (void)index;
        recompute_kinds();
        s.clear();
        s += strf("// group %d: %s over domain [PFDOMAIN0", index, grp.kernel_name.c_str());
        for (size_t k = 1; k < grp.domain.size(); ++k) s += strf(",%lld", (long long)grp.domain[k]);
        s += "], nodes";
        for (int id : grp.nodes) s += strf(" %%%d=%s", id, op_name(g.nodes[id].op));
        s += "\n";
        s += strf("#define PF_PRECISE %d\n", precise ? 1 : 0);
        s += kDevicePrelude;
        switch (grp.tmpl) {
            case PF_T_EW_FLAT: gen_flat(); break;
            case PF_T_ROW_RESIDENT: gen_row(); break;
            case PF_T_TILE: gen_tile(); break;
            case PF_T_COL_REDUCE: gen_col(); break;
            default: fail(PF_E_COMPILE, "template not implemented");
        }
        std::string nm = grp.tmpl == PF_T_EW_FLAT ? "pf_ew" : grp.tmpl == PF_T_ROW_RESIDENT ? "pf_row" : grp.tmpl == PF_T_TILE ? "pf_tile" : grp.tmpl == PF_T_COL_REDUCE ? "pf_col" : "pf_loop";
        int shown = 0;
        for (int id : grp.nodes) {
            if (shown == 8) { nm += "_etc"; break; }
            nm += "_";
            nm += op_name(g.nodes[id].op);
            ++shown;
        }
        {
            // a row-streaming kernel (one workgroup per row) never mentions the number of rows either
            const bool generic = grp.outer_runtime || (grp.tmpl == PF_T_ROW_LOOP && rd >= 2);
            const std::string d0 = grp.domain.empty() ? "" : generic ? "*" : strf("%lld", (long long)grp.domain[0]);
            const size_t at = s.find("PFDOMAIN0");
            s.replace(at, 9, d0);
        }
        unsigned long long h = 1469598103934665603ull;
        for (unsigned char c : s) { h ^= c; h *= 1099511628211ull; }
        nm += strf("_%08x", (unsigned)(h ^ (h >> 32)));
        size_t pos;
        while ((pos = s.find("PFKNAME")) != std::string::npos) s.replace(pos, 7, nm);
        grp.kernel_name = nm;
        if (!grp.kernel2_name.empty()) grp.kernel2_name = nm + "_fin";
        grp.source = s;
        grp.source_body_at = s.find(kDevicePrelude) + std::string(kDevicePrelude).size();      // the header line above it has just changed length
    }
};

}  // namespace

void generate_source(const pf_graph& g, const pf_options& opt, Group& grp, int index) {
    Emit e(g, opt, grp);
    e.run(index);
}

namespace {

// p12 -> r0_p12, q3 -> r0_q3 (whole identifiers only)
std::string rename_pointer_params(const std::string& text, const std::string& prefix) {
    std::string out;
    out.reserve(text.size() + 64);
    auto ident = [](char c) { return (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || (c >= '0' && c <= '9') || c == '_'; };
    for (size_t i = 0; i < text.size();) {
        if ((text[i] == 'p' || text[i] == 'q') && (i == 0 || !ident(text[i - 1])) && i + 1 < text.size() && text[i + 1] >= '0' && text[i + 1] <= '9') {
            size_t j = i + 1;
            while (j < text.size() && text[j] >= '0' && text[j] <= '9') ++j;
            if (j == text.size() || !ident(text[j])) {
                out += prefix;
                out.append(text, i, j - i);
                i = j;
                continue;
            }
        }
        out += text[i++];
    }
    return out;
}

void replace_all(std::string& s, const std::string& what, const std::string& with) {
    for (size_t at = 0; (at = s.find(what, at)) != std::string::npos; at += with.size()) s.replace(at, what.size(), with);
}

}  // namespace

// A subgraph often has a small side computation (a chain on a weight vector, on per-row scalars) whose kernel is one
// workgroup or a few: a launch of its own costs ~4 us for microseconds of nothing.  Such a kernel rides on another kernel
// of the plan instead: the host is launched with that many workgroups more, and those run the rider's code.  The
// rider's kernel text becomes a device function in a namespace of its own (its pointer parameters renamed, its
// workgroup index counted from the host's grid); the host's kernel gets the rider's pointers after its own parameters
// and one line at its top that sends the workgroups past its own grid to the rider.
bool attach_rider(Group& host, const Group& rider) {
    // (a larger rider must not move much: the launch it saves is worth ~4 us, while sharing one kernel's register and
    // LDS budget with the host cost a 196 MB rider 1.5 us; and it must be light on LDS, or every workgroup of the host
    // pays for it in occupancy: row and flat kernels are, a tile kernel is when host and rider together stage at most
    // three tensors, a column reduction is not)
    int rider_staged = 0;
    for (auto& o : rider.operands) rider_staged += o.transposed ? 1 : 0;
    for (auto& st : rider.stores) rider_staged += st.tstore ? 1 : 0;
    int host_staged = 0;
    for (auto& o : host.operands) host_staged += o.transposed ? 1 : 0;
    for (auto& st : host.stores) host_staged += st.tstore ? 1 : 0;
    const bool light = rider.bytes_read + rider.bytes_written <= (uint64_t(96) << 20) &&
                       (rider.tmpl == PF_T_EW_FLAT || rider.tmpl == PF_T_ROW_RESIDENT || rider.tmpl == PF_T_ROW_LOOP ||
                        (rider.tmpl == PF_T_TILE && rider_staged + host_staged <= 3));
    if (rider.grid < 1 || (rider.grid > 64 && !light) || !rider.kernel2_name.empty() || !host.kernel2_name.empty() || rider.scratch_bytes || !rider.riders.empty() || host.riders.size() >= 4) return false;
    if (host.source_body_at == 0 || rider.source_body_at == 0 || rider.block > host.block) return false;
    // A rider written for fewer lanes than the host's workgroups have: the surplus waves of its workgroups leave at
    // once (a barrier waits for the surviving waves of a workgroup only), which wastes their slots - small riders only.
    const bool narrower = rider.block < host.block;
    if (narrower && (rider.grid > 256 || rider.bytes_read + rider.bytes_written > (uint64_t(8) << 20))) return false;
    // a tile kernel that stages several tensors has little LDS to spare for a rider's own
    if (host_staged > 2) return false;
    const std::string head = "extern \"C\" __global__ void __launch_bounds__(";
    std::string rtext = rider.source.substr(rider.source_body_at);
    const size_t rk = rtext.find(head);
    if (rk == std::string::npos || rtext.find(head, rk + 1) != std::string::npos) return false;
    const size_t rname_at = rtext.find(") ", rk + head.size());
    const size_t rparen = rtext.find('(', rname_at + 2);
    if (rname_at == std::string::npos || rparen == std::string::npos) return false;
    const std::string tag = strf("r%zu_", host.riders.size()), space = strf("pf_rider%zu", host.riders.size());
    rtext.replace(rk, rparen - rk, "__device__ __forceinline__ void pf_rider_kernel");
    replace_all(rtext, "blockIdx.x", strf("(blockIdx.x - %lldu)", (long long)host.grid));      // the rider's workgroups follow the host's
    rtext = rename_pointer_params(rtext, tag);

    std::string htext = host.source.substr(host.source_body_at);
    const size_t hk = htext.find(head);
    if (hk == std::string::npos) return false;
    const size_t hopen = htext.find('(', htext.find(") ", hk + head.size()) + 2);
    const size_t hclose = htext.find(") {", hopen);
    if (hopen == std::string::npos || hclose == std::string::npos) return false;
    // the rider's pointers, as parameters of the host and as arguments of the call
    std::string params, args;
    auto add = [&](const std::string& type, const std::string& name) {
        params += ", " + type + " " + name;
        args += (args.empty() ? "" : ", ") + name;
    };
    auto tn = [](pf_dtype d) { return d == PF_BF16 ? "u16" : d == PF_F16 ? "f16" : "float"; };
    for (size_t oi = 0; oi < rider.operands.size(); ++oi) add(strf("const %s* __restrict__", tn(rider.operands[oi].dtype)), strf("%sp%zu", tag.c_str(), oi));
    int sp = 0;
    for (auto& st : rider.stores)
        for (size_t c = 0; c < 1 + st.also_outputs.size(); ++c, ++sp) add(strf("%s* __restrict__", tn(st.dtype)), strf("%sq%d", tag.c_str(), sp));
    if (rider.outer_runtime) args += strf("%s(long long)%lld", args.empty() ? "" : ", ", (long long)rider.outer_extent);
    const std::string guard = narrower ? strf("if (threadIdx.x < %du) ", rider.block) : "";
    std::string call = strf("\n    if (blockIdx.x >= %lldu && blockIdx.x < %lldu) { %s%s::pf_rider_kernel(%s); return; }", (long long)host.grid,
                            (long long)(host.grid + rider.grid), guard.c_str(), space.c_str(), args.c_str());
    htext.insert(hclose + 3, call);
    htext.insert(hclose, params);
    // (an earlier rider's parameters already follow the host's: this one's go after them, before the closing parenthesis)
    host.source = host.source.substr(0, host.source_body_at) + "namespace " + space + " {\n" + rtext + "}  // namespace " + space + "\n" + htext;
    // the kernel's name ends in a hash of its source: with a rider it is another kernel
    {
        unsigned long long h = 1469598103934665603ull;
        for (unsigned char c : host.source) { h ^= c; h *= 1099511628211ull; }
        const std::string old_name = host.kernel_name;
        const std::string new_name = old_name.substr(0, old_name.rfind('_')) + strf("_%08x", (unsigned)(h ^ (h >> 32)));
        replace_all(host.source, old_name, new_name);
        host.kernel_name = new_name;
    }
    Group::Rider rd;
    rd.operands = rider.operands;
    rd.stores = rider.stores;
    host.riders.push_back(std::move(rd));
    host.grid += rider.grid;
    host.rt_per_block = 0;                  // the rider's workgroup number is literal: no other outermost extent
    host.bytes_read += rider.bytes_read;
    host.bytes_written += rider.bytes_written;
    host.nodes.insert(host.nodes.end(), rider.nodes.begin(), rider.nodes.end());
    host.user_nodes.insert(host.user_nodes.end(), rider.user_nodes.begin(), rider.user_nodes.end());
    host.node_kind.insert(host.node_kind.end(), rider.node_kind.begin(), rider.node_kind.end());
    return true;
}

}  // namespace pf
