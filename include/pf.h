/*
 * pf.h - C ABI of the fused-subgraph engine for AMD MI355X (gfx950).
 *
 * The library takes a computational subgraph in the sense of the paper's
 * Definition 3.1 (a DAG of operator nodes, each with an operator type and an
 * output shape), partitions it into fusible groups, lowers every group to one
 * hand-written HIP kernel skeleton with a generated straight-line body,
 * compiles it once, and executes it on caller-owned device buffers.  The
 * outputs of a candidate execution can then be scored against a reference
 * under the tolerance test of Definition 3.2 / Eq. 1 with the atol/rtol pair
 * of Appendix F.
 *
 * Conventions
 *   - Every function returns a pf_status (0 = PF_OK, < 0 = error).  Nothing
 *     throws across this boundary.  pf_last_error() gives the message of the
 *     last failing call on the calling thread.
 *   - "h_" arguments are host pointers, "d_" arguments are device pointers.
 *   - Tensors are dense, row-major, in the dtype declared in the graph.
 *     Device pointers must be 16-byte aligned.
 *   - The caller owns all device buffers and the stream.  The library owns
 *     pf_graph / pf_exec handles and the code objects behind them.
 *   - pf_execute and pf_score only enqueue work on the given stream; they
 *     never synchronise and never allocate device memory.
 *   - The paper's failure classes (Sec. 3.4: accuracy = 1, compilation = 2,
 *     runtime = 3) map to: PF_E_COMPILE (class 2), PF_E_RUNTIME (class 3); an
 *     accuracy failure is not an error code but allclose == 0 in a
 *     pf_score_result.
 */
#ifndef PF_H
#define PF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PF_OK = 0,
    PF_E_INVALID = -1, /* bad argument, null handle, misaligned pointer            */
    PF_E_COMPILE = -2, /* ill-formed graph, unsupported op/dtype/shape, JIT failed */
    PF_E_RUNTIME = -3, /* wrong buffer count, short workspace, launch failed       */
    PF_E_NOMEM = -4
} pf_status;

/* Storage dtypes.  PF_F16 is IEEE binary16.  PF_F64 is accepted only as the reference side of
 * pf_score / pf_score_ladder.  Scored pairs: a candidate of f32, bf16 or f16 against a reference
 * of the same dtype, f32 or f64; an f32 candidate also against a bf16 or f16 reference. */
typedef enum { PF_F32 = 0, PF_BF16 = 1, PF_F64 = 2, PF_F16 = 3 } pf_dtype;

/*
 * Operator types (the set tau ranges over).  Binary operators broadcast
 * right-aligned, NumPy style.  Reductions act on the last dim and keep it as
 * size 1 unless keepdim=0.  All arithmetic is carried out in fp32 (sums in a
 * wider accumulator for fp32 graphs); a value is rounded to its node dtype
 * only where it is written to memory.
 */
typedef enum {
    PF_OP_INPUT = 0,
    PF_OP_CONST,     /* attr value=<float>; rank-0 scalar                        */
    PF_OP_ADD, PF_OP_SUB, PF_OP_MUL, PF_OP_DIV,
    PF_OP_EXP, PF_OP_TANH,
    PF_OP_SIGMOID,   /* 1 / (1 + exp(-x))                                        */
    PF_OP_GELU,      /* attr approx=tanh (default) | erf                         */
    PF_OP_RSQRT,     /* 1 / sqrt(x)                                              */
    PF_OP_SUM, PF_OP_MAX, PF_OP_MEAN,   /* attrs keepdim=1|0, dim=-1|-2 (which dim is reduced;
                                           -2 is the sequence dim of the paper's Case 2); max propagates NaN */
    PF_OP_VAR,       /* mean((x-mean)^2) * n/(n-correction); attr correction=0   */
    PF_OP_TRANSPOSE, /* swaps the last two dims                                  */
    PF_OP_ROT_PAIRS, /* out[2i] = -x[2i+1], out[2i+1] = x[2i] on the last dim    */
    PF_OP_ROLL,      /* attrs shift=<int>, dim=<int>: out[i] = x[(i - shift) mod S] along dim
                        (the roll of the paper's Case 1); folded into the loads of its consumer */
    PF_OP_SLICE,     /* attrs dim=<int>, start=<int>, stop=<int>: x[start:stop] along dim;
                        folded into the loads of its consumer                     */
    PF_OP_MAXIMUM, PF_OP_MINIMUM,   /* element-wise, NaN-propagating; clamp(x, min=c) = maximum(x, c) */
    PF_OP_COUNT_
} pf_op;

#define PF_MAX_RANK 4

typedef struct pf_graph pf_graph;
typedef struct pf_exec pf_exec;

typedef struct { const char* key; const char* value; } pf_attr;

/* ---- graph construction (Def. 3.1: nodes, edges, operator types, shapes) ---- */

pf_status pf_graph_create(pf_graph** g);
void      pf_graph_destroy(pf_graph* g);

/* Declares an external input tensor; rank in [0, PF_MAX_RANK], dims > 0.
 * Returns the new node id through node_out.  Ids are consecutive from 0. */
pf_status pf_graph_input(pf_graph* g, pf_dtype dtype, int rank, const int64_t* h_shape, int* node_out);

/* Adds an operator node reading earlier nodes.  The output shape is inferred
 * (broadcast / reduction / transposition rules) and never supplied.
 * out_dtype is the dtype the value has whenever it is stored to memory. */
pf_status pf_graph_node(pf_graph* g, pf_op op, const int* h_in_nodes, int n_in,
                        const pf_attr* h_attrs, int n_attr, pf_dtype out_dtype, int* node_out);

/* Marks a node as a graph output (order of calls = order of output buffers). */
pf_status pf_graph_output(pf_graph* g, int node);

/* Text form (one statement per line):
 *     in %0 : bf16[8192,11008]
 *     %2 = add(%0, %1) {key=value} : bf16
 *     out %2
 * pf_graph_print writes a form that pf_graph_parse reads back into an equal
 * graph.  print: buf may be NULL / cap 0 to query *needed (bytes incl. NUL). */
pf_status pf_graph_parse(const char* h_text, size_t len, pf_graph** g);
pf_status pf_graph_print(const pf_graph* g, char* h_buf, size_t cap, size_t* needed);

/* A member G_i of a task instance (Sec. 3.1: subgraphs sharing the operator-type sequence but
 * varying in shape and dtype): a new graph with the operators of g, input k given shape
 * h_shapes[k*PF_MAX_RANK .. +h_ranks[k]) (host arrays, one entry per graph input in order), and every
 * tensor of dtype from_dtype re-typed to to_dtype (both -1: dtypes unchanged).  All shapes are
 * inferred again; attributes that do not fit the new shapes (slice bounds, variance sizes) and
 * operands that no longer broadcast are PF_E_COMPILE.  The caller owns *out. */
pf_status pf_graph_variant(const pf_graph* g, const int* h_ranks, const int64_t* h_shapes, int from_dtype, int to_dtype,
                           pf_graph** out);

typedef struct {
    pf_op    op;
    pf_dtype dtype;
    int      rank;
    int64_t  shape[PF_MAX_RANK];
    int      n_in;
    int      in_nodes[2];
    int      is_output;
} pf_node_info;

pf_status pf_graph_size(const pf_graph* g, int* n_nodes, int* n_inputs, int* n_outputs);
pf_status pf_graph_node_info(const pf_graph* g, int node, pf_node_info* h_info);

/* ---- compilation: fusion planning + kernel specialisation ---- */

typedef struct {
    int fuse;              /* 1: group nodes into fused kernels (default); 0: one kernel per node */
    int intermediates_f32; /* 1: values crossing a kernel boundary are kept in fp32 (default for
                              fuse=1); 0: stored in their node dtype, as op-by-op execution would */
    /* tiling overrides for experiments; 0 = let the planner choose from the shape */
    int tune_row_lanes;    /* row templates: lanes per row (power of two)                         */
    int tune_row_unroll;   /* row templates: rows in flight per team of lanes                     */
    int tune_flat_unroll;  /* ew_flat: 16-byte vectors per lane; tile: consecutive tiles per XCD  */
    int tune_col_block;    /* col_reduce: lanes per workgroup (power of two, 64..1024)             */
    int tune_tile_edge;    /* tile: edge of the LDS tile, 32 or 64                                 */
    int reserved[1];       /* must be zero */
} pf_options;

void pf_options_default(pf_options* h_opt);

/* Plans and JIT-compiles for gfx950.  Needs no GPU: code objects are loaded
 * onto the device at the first pf_execute. */
pf_status pf_compile(const pf_graph* g, const pf_options* h_opt, pf_exec** e);
void      pf_exec_destroy(pf_exec* e);

typedef enum { PF_T_EW_FLAT = 0, PF_T_ROW_RESIDENT = 1, PF_T_TILE = 2, PF_T_ROW_LOOP = 3, PF_T_COL_REDUCE = 4 } pf_template;

typedef struct {
    int      n_kernels;          /* number of kernel launches per pf_execute              */
    int      n_inputs, n_outputs;
    uint64_t algorithmic_bytes;  /* external inputs once + outputs once                   */
    uint64_t workspace_bytes;    /* device scratch pf_execute needs (may be 0)            */
    uint64_t planned_bytes;      /* bytes the planned kernels read + write, incl. scratch */
    int      n_groups;           /* launches' worth of fused groups; pf_exec_group_info / pf_exec_source index
                                    them.  A group is one kernel, except a column reduction over few column
                                    tiles, which runs a partial and a combining kernel (n_kernels counts both).
                                    Groups of a plan that do not depend on each other may share one kernel: the
                                    smaller ones ride on the largest as extra workgroups and are reported with it
                                    (its nodes, bytes and grid include theirs) */
    int      reserved_;
} pf_plan_info;

typedef struct {
    pf_template tmpl;
    int      n_nodes;            /* operator nodes computed by this kernel, in the caller's numbering: a value
                                    behind a transpose may be recomputed in the reader's kernel (then it shows
                                    in both, or only there), transposes that cancel show nowhere */
    int      nodes[64];
    int64_t  rows, cols;         /* iteration domain: product of leading dims, last dim   */
    int      block_threads;
    int64_t  grid_blocks;
    int      lanes_per_row;      /* row templates: lanes cooperating on one row           */
    uint64_t bytes_read, bytes_written;
} pf_group_info;

pf_status pf_exec_info(const pf_exec* e, pf_plan_info* h_info);
pf_status pf_exec_group_info(const pf_exec* e, int group, pf_group_info* h_info);
/* Generated HIP source of one kernel, for inspection (same buffer protocol as print). */
pf_status pf_exec_source(const pf_exec* e, int group, char* h_buf, size_t cap, size_t* needed);
/* Name of the group's kernel: template, operators and a hash of the whole generated source, so two
 * groups with the same name run the same code object (same buffer protocol as print). */
pf_status pf_exec_kernel_name(const pf_exec* e, int group, char* h_buf, size_t cap, size_t* needed);

/* Code objects are cached by source text, in the process and (PF_CACHE_DIR) on disk.  A task
 * instance (Sec. 3.1) holds the same operators at several shapes: elementwise and row kernels take
 * the outermost extent of their domain as an argument, so members that differ only there and get the
 * same tiling generate the same text and share one code object.  Counters of this process:
 * compilations, hits in memory, hits on disk, distinct code objects held. */
typedef struct {
    uint64_t compiled, memory_hits, disk_hits, code_objects;
} pf_jit_stats;
pf_status pf_jit_stats_get(pf_jit_stats* h_out);

/* Thread safety: a pf_exec may be shared by several host threads (its lazy module load is guarded);
 * each call in flight needs its own workspace.  pf_graph objects are not synchronised.
 *
 * Runs the compiled subgraph once.  d_inputs / d_outputs follow the order of
 * the graph's `in` declarations and pf_graph_output calls.  d_workspace must
 * hold workspace_bytes (256-byte aligned) and is private to this call while it
 * is in flight.  Enqueues n_kernels launches on `stream` (a hipStream_t; NULL
 * is the default stream). */
pf_status pf_execute(pf_exec* e, const void* const* d_inputs, int n_in, void* const* d_outputs, int n_out,
                     void* d_workspace, size_t workspace_bytes, void* stream);

/* Runs a compiled subgraph at another outermost extent than the one it was compiled for (a smaller
 * batch: the last member of a task instance, Sec. 3.1, need not be compiled at all).  Every tensor that
 * carries the outermost dim of the kernel's domain is taken to have outer_extent there; tensors that
 * broadcast along it are unchanged.  Only for subgraphs that are one kernel of the elementwise or row
 * templates without scratch, 1 <= outer_extent <= the compiled extent (the index width and the tiling
 * were chosen for that one); otherwise PF_E_INVALID and nothing is enqueued. */
pf_status pf_execute_outer(pf_exec* e, int64_t outer_extent, const void* const* d_inputs, int n_in, void* const* d_outputs,
                           int n_out, void* stream);

/* As pf_execute, with two caller-owned hipEvent_t handles (either may be NULL):
 * start_event is recorded when the first kernel begins executing and
 * stop_event when the last kernel has finished, so that
 * hipEventElapsedTime(start, stop) is the device time of the kernels without
 * the launch overhead around them.  Used by the benchmark (paper Sec. 4.1
 * protocol: warm-up runs, then timed trials). */
pf_status pf_execute_timed(pf_exec* e, const void* const* d_inputs, int n_in, void* const* d_outputs, int n_out,
                           void* d_workspace, size_t workspace_bytes, void* stream, void* start_event, void* stop_event);

/* ---- error scoring (Def. 3.2 / Eq. 1 with atol, rtol of Appendix F) ---- */

typedef struct {
    const void* d_cand;   /* candidate output                      */
    const void* d_ref;    /* reference output                      */
    uint64_t    n;        /* elements                              */
    int32_t     cand_dtype, ref_dtype;   /* pf_dtype               */
    double      rtol, atol;
    int32_t     equal_nan; /* 1: NaN vs NaN at the same index passes */
    int32_t     reserved;
} pf_pair;

/* One element passes when a == b, or |a-b| is finite and <= atol + rtol*|b|
 * (b = reference); NaN on either side fails unless equal_nan and both are NaN.
 * max_abs / max_rel range over elements where neither side is NaN; relative
 * error is 0 when a == b, +inf when b == 0 or |a-b| is infinite, else
 * |a-b|/|b|.  All comparisons are made in fp64 on exactly widened values. */
typedef struct {
    double   max_abs, max_rel;
    uint64_t n, n_viol;
    uint64_t nan_cand, nan_ref, inf_cand, inf_ref;
    uint32_t allclose;       /* n_viol == 0                                   */
    uint32_t bit_identical;  /* same dtype and every element has the same bits */
    uint64_t reserved_;      /* internal progress counter; ignore              */
} pf_score_result;

/* Bytes of device scratch pf_score needs for n_pairs pairs (about 5.5 KB per pair).  A workspace
 * needs no initialisation, holds nothing of value after the call, and is private to the call while
 * it runs. */
size_t pf_score_workspace_bytes(int n_pairs);

/* Scores n_pairs pairs in one pass over their elements.  h_pairs is read
 * before the call returns.  d_results receives n_pairs structs once the
 * stream has run. */
pf_status pf_score(const pf_pair* h_pairs, int n_pairs, pf_score_result* d_results,
                   void* d_workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): pf_score with the library's own scratch in place of a workspace
 * argument.  The scratch is an array of 1.5 MiB inside the library's code object; each GPU the
 * library runs on holds one copy until the process ends.  At most PF_SCORE_STATIC_MAX_PAIRS pairs per
 * call (more is PF_E_INVALID and nothing is enqueued); results, arguments and error behaviour are
 * those of pf_score.  The call allocates and frees no device memory and does not synchronise; the
 * first call on a device looks the array's address up there.  All calls on one GPU share that
 * GPU's array: each call clears what it needs first, and two calls whose kernels may overlap on
 * one GPU (different streams, or threads without ordering) race - order them on one stream. */
#define PF_SCORE_STATIC_MAX_PAIRS 256
pf_status pf_score_static(const pf_pair* h_pairs, int n_pairs, pf_score_result* d_results, void* stream);

/* ---- tolerance ladder and error-aware speedup scores (Sec. 3.4, App. D-F) ---- */

#define PF_LADDER_LEVELS 11   /* tolerance indices t = -10 .. 0 */
#define PF_ES_LEVELS 15       /* t = -10 .. 4 (|E| = 3 error categories, t up to |E|+1) */

/* rtol(t), atol(t) = 10^(k t) with the per-dtype slopes of Appendix F (bf16, f16, f32, f64);
 * t > 0 gives the values of t = 0. */
pf_status pf_tolerance(pf_dtype dtype, int t, double* h_rtol, double* h_atol);

typedef struct {
    uint64_t n;
    uint64_t n_viol[PF_LADDER_LEVELS];   /* [k]: elements failing at t = k - 10, tolerances of the candidate's dtype */
} pf_ladder_result;

/* As pf_score, but counts the violations at all 11 numerical tolerance levels
 * in one pass over the data.  The rtol / atol fields of the pairs are ignored;
 * equal_nan is honoured. */
size_t    pf_score_ladder_workspace_bytes(int n_pairs);
pf_status pf_score_ladder(const pf_pair* h_pairs, int n_pairs, pf_ladder_result* d_results,
                          void* d_workspace, size_t workspace_bytes, void* stream);

/* Both results from a single read of every pair: what the evaluation of Sec. 3.4 needs per output (the
 * verdict of Eq. 1 at all eleven numerical tolerance levels for ES_t / AS, and the error maxima and counts
 * at the pair's own rtol / atol).  d_score_results and d_ladder_results receive n_pairs structs each;
 * arguments, workspace (pf_score_all_workspace_bytes) and error behaviour as for pf_score. */
size_t    pf_score_all_workspace_bytes(int n_pairs);
pf_status pf_score_all(const pf_pair* h_pairs, int n_pairs, pf_score_result* d_score_results, pf_ladder_result* d_ladder_results,
                       void* d_workspace, size_t workspace_bytes, void* stream);

/* One evaluated subgraph: measured speedup over the reference execution, how it
 * failed if it did (0: ran; 2: compilation, 3: runtime failure; an accuracy
 * failure, class 1, follows from the counts) and the ladder counts summed over
 * its outputs. */
typedef struct {
    double   speedup;
    int32_t  error_class;
    int32_t  reserved;
    uint64_t n_viol[PF_LADDER_LEVELS];
} pf_case;

typedef struct {
    double es[PF_ES_LEVELS];   /* ES_t, Eq. 3, [k]: t = k - 10 */
    double as;                 /* AS, Eq. 4 */
} pf_metrics;

/* Host-side aggregation: rectified speedups (Eq. 2, base penalty b, slowdown
 * exponent p), their geometric mean per t and the weighted geometric mean AS. */
pf_status pf_aggregate(const pf_case* h_cases, int n_cases, double b, double p, pf_metrics* h_out);
/* Fraction of all cases that are correct at tolerance index t and faster than threshold. */
pf_status pf_fast_p(const pf_case* h_cases, int n_cases, double threshold, int t, double* h_out);

/* ---- misc ---- */

/* Plain device copy of `bytes` bytes (multiple of 16) with the library's
 * streaming load/store path; the practical bandwidth ceiling to quote beside
 * the fused kernels. */
pf_status pf_copy_bytes(void* d_dst, const void* d_src, size_t bytes, void* stream);

const char* pf_last_error(void);
const char* pf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PF_H */
