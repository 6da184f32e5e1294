// Internal data structures of the fused-subgraph engine (host side).
#pragma once

#include <cstdint>
#include <map>
#include <stdexcept>
#include <string>
#include <vector>

#include "pf.h"

namespace pf {

// Error carrying a pf_status; caught at the C boundary.
struct Error : std::runtime_error {
    pf_status status;
    Error(pf_status s, const std::string& m) : std::runtime_error(m), status(s) {}
};

[[noreturn]] void fail(pf_status s, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
std::string strf(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

using Shape = std::vector<int64_t>;

inline int64_t numel(const Shape& s) {
    int64_t n = 1;
    for (int64_t d : s) n *= d;
    return n;
}
inline int itemsize(pf_dtype d) { return (d == PF_BF16 || d == PF_F16) ? 2 : d == PF_F32 ? 4 : 8; }
const char* dtype_name(pf_dtype d);
const char* op_name(pf_op op);
bool op_from_name(const std::string& name, pf_op* op);
bool is_reduction(pf_op op);
bool is_unary(pf_op op);
bool is_binary(pf_op op);
inline bool is_view(pf_op op) { return op == PF_OP_ROLL || op == PF_OP_SLICE; }

// A node of the computational graph (Def. 3.1): operator type, operands,
// inferred output shape, and the dtype it has when stored.
struct Node {
    pf_op op = PF_OP_INPUT;
    pf_dtype dtype = PF_F32;
    std::vector<int> in;
    Shape shape;
    // attributes
    double value = 0.0;   // const
    int keepdim = 1;      // reductions
    int correction = 0;   // var
    int gelu_erf = 0;     // gelu: 0 tanh form, 1 erf form
    int dim = 0;          // roll, slice: normalised to [0, rank)
    int red_dim = -1;     // reductions: -1 (last dim) or -2 (the dim before it)
    int64_t shift = 0;    // roll
    int64_t start = 0, stop = 0;   // slice
    bool is_output = false;
    // set by the rewrite that runs ahead of planning (never by the parser):
    int orig = -1;                 // the user's node this one computes (a value recomputed in the other orientation keeps it)
    std::vector<char> alias_t;     // per operand: read through a swap of its last two dims that moves no data
    bool reads_alias(size_t k) const { return k < alias_t.size() && alias_t[k]; }
    bool store_t = false;          // a transpose whose operand is computed in its kernel and only written out: a transposed store
    bool col_prologue = false;     // computed for a column reduction in its sources' orientation: belongs in that reduction's kernel
};

}  // namespace pf

struct pf_graph {
    std::vector<pf::Node> nodes;
    std::vector<int> inputs;    // node ids of inputs, in declaration order
    std::vector<int> outputs;   // node ids of outputs, in declaration order
};

namespace pf {

// ---- ir.cpp ----
int graph_add_input(pf_graph& g, pf_dtype dt, const Shape& shape);
int graph_add_node(pf_graph& g, pf_op op, const std::vector<int>& in,
                   const std::vector<std::pair<std::string, std::string>>& attrs, pf_dtype dt);
void graph_add_output(pf_graph& g, int node);
void graph_parse(const std::string& text, pf_graph& g);
std::string graph_print(const pf_graph& g);
void graph_variant(const pf_graph& g, const int* ranks, const int64_t* shapes, int from, int to, pf_graph& out);
Shape broadcast_shapes(const Shape& a, const Shape& b);

// ---- plan.cpp ----

// One step of an index remapping along one dim, applied to the consumer's index:
// slice: idx + add; roll: (idx + add) mod size (add = size - shift mod size).
struct ViewStep {
    int64_t add = 0;
    int64_t mod = 0;   // 0: no wrap
};

// How a kernel reads one external tensor inside its iteration domain.
struct Operand {
    int node = -1;            // producing node (graph input or earlier group's member)
    pf_dtype dtype = PF_F32;  // dtype in memory
    Shape shape;              // its own shape
    // element strides per domain dim (domain rank-aligned; 0 where broadcast)
    int64_t stride[PF_MAX_RANK] = {0, 0, 0, 0};
    bool transposed = false;  // read through a swap of the last two dims (data really moves)
    bool via_transpose = false;  // requested by a transpose node (even when it moves no data)
    bool coluni = false;         // read by the epilogue of a column reduction (stride 0 along dim -2)
    // read through a chain of roll / slice nodes ending in node `view` (-1: read directly):
    // per domain dim the steps that turn the consumer's index into the source index
    int view = -1;
    std::vector<ViewStep> steps[PF_MAX_RANK];
    int64_t const_offset = 0;    // contribution of source dims the domain does not iterate over
    bool mapped(int k) const { return !steps[k].empty(); }
    // where the bytes live
    int graph_input = -1;     // index into d_inputs, or
    int64_t ws_offset = -1;   // byte offset into the workspace, or
    int graph_output = -1;    // an earlier group's graph output buffer
};

struct Store {
    int node = -1;
    pf_dtype dtype = PF_F32;
    Shape shape;
    bool row_scalar = false;   // one value per row of the domain
    bool col_uniform = false;  // one value per (leading index, column): result of a reduction over dim -2
    int graph_output = -1;     // index into d_outputs, or
    int64_t ws_offset = -1;    // byte offset into the workspace
    std::vector<int> also_outputs;  // further graph-output slots receiving the same values
    bool tstore = false;       // written through a swap of the last two dims (tile kernels: an LDS transpose on the store side)
    int value_node = -1;       // the member whose registers are stored (-1: `node` itself)
};

struct Group {
    pf_template tmpl = PF_T_EW_FLAT;
    std::vector<int> nodes;        // members in topological order (const nodes folded in)
    std::vector<int> user_nodes;   // the caller's node ids the members compute (what reports show)
    std::vector<int> node_kind;    // per member: 2 full, 1 row-uniform, 3 column-uniform
    Shape domain;                  // iteration domain, rank-aligned full shape
    int64_t rows = 1, cols = 1;    // product of leading dims, last dim
    std::vector<Operand> operands; // external reads
    // a column reduction whose rows are split over several workgroups: partial results go to scratch
    // memory (a slice of the workspace, passed as the last kernel argument) and a second kernel of
    // the same module combines them
    bool outer_runtime = false;     // the kernel takes the outermost domain extent as its last scalar argument
    int64_t outer_extent = 0;
    // running at another outermost extent than the compiled one: grid = ceil(outer * rt_per_outer / rt_per_block),
    // allowed when rt_per_block > 0 and outer * rt_rows_per_outer is a multiple of rt_row_multiple
    int64_t rt_per_outer = 0, rt_per_block = 0, rt_rows_per_outer = 1, rt_row_multiple = 1;
    uint64_t scratch_bytes = 0;
    int64_t scratch_offset = -1;
    std::string kernel2_name;
    int64_t grid2 = 0;
    int block2 = 0;
    std::vector<Store> stores;     // writes
    int extra_launches = 0;        // plan-time estimate: a column reduction split over workgroups brings a combining kernel
    // launch configuration (filled by codegen)
    int block = 256;
    int64_t grid = 1;
    int lanes_per_row = 0;
    int vec = 1, chunks_per_lane = 1;
    // Small groups that ride on this kernel as extra workgroups (see attach_rider): their pointer arguments follow
    // this group's own
    struct Rider {
        std::vector<Operand> operands;
        std::vector<Store> stores;
    };
    std::vector<Rider> riders;     // in the order of their parameters in the kernel's signature
    size_t source_body_at = 0;     // where the kernel text starts in `source`, after the common prelude
    std::string source;            // generated HIP
    std::string kernel_name;
    std::vector<char> code;        // code object
    uint64_t bytes_read = 0, bytes_written = 0;
};

// pointer arguments of one kernel (operands + stores) plus the outer extent and the scratch pointer
constexpr int kMaxKernelArgs = 160;

struct Plan {
    std::vector<Group> groups;
    uint64_t workspace_bytes = 0;
    uint64_t algorithmic_bytes = 0;
};

void make_plan(const pf_graph& g, const pf_options& opt, Plan& plan);
// What a plan costs under the traffic model: bytes moved (those of kernels that stage tensors through LDS transposes
// weighted by how much slower such kernels run), plus for each kernel what a launch costs at least, expressed in
// bytes (about 4 us at the rate of a plain copy).
constexpr uint64_t kLaunchCostBytes = 24u << 20;
uint64_t plan_cost(const Plan& plan);

// ---- rewrite.cpp ----
// `sites` (caller's node ids, from rewrite_sites): reductions over the last dim to run as reductions over dim -2
// of their operand's cone, evaluated in the orientation its sources have in memory; and transposes of computed
// values whose kernel is to take over what the value's own kernel computes besides (results of that orientation
// are then written through a transposed store); and, listed as -(node + 1), transposes that only the caller reads, to
// be written by the kernel that computes their operand
void sink_transposes(const pf_graph& g, const pf_options& opt, const std::vector<int>& sites, pf_graph& out);
std::vector<int> rewrite_sites(const pf_graph& g, const pf_options& opt);

// ---- codegen.cpp ----
void generate_source(const pf_graph& g, const pf_options& opt, Group& grp, int index);
// Lets the kernel of `rider` (at most 64 workgroups) run as the workgroups past host.grid of the host's kernel (both
// already generated, same workgroup size, independent of each other).  False, and nothing changed, if they do not fit.
bool attach_rider(Group& host, const Group& rider);

// ---- runtime.cpp ----
void jit_compile(Group& grp);
void jit_stats(pf_jit_stats* out);

}  // namespace pf
