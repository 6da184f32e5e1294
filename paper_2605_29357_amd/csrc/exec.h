// A compiled subgraph: the plan, its code objects and (once loaded) the
// device modules.
#pragma once
#include <mutex>

#include "pf_internal.h"

struct pf_exec {
    pf::Plan plan;
    pf_options opt;
    int n_inputs = 0, n_outputs = 0;
    std::vector<uint64_t> input_bytes, output_bytes;
    std::mutex load_mu;             // guards the lazy module load (several threads may share one pf_exec)
    bool loaded = false;
    std::vector<void*> modules;     // hipModule_t
    std::vector<void*> functions;   // hipFunction_t
    std::vector<void*> functions2;  // hipFunction_t of a group's second kernel, or null
};

namespace pf {
void exec_load(pf_exec& e);
void exec_unload(pf_exec& e);
void exec_run(pf_exec& e, const void* const* d_inputs, void* const* d_outputs, void* d_ws, void* stream, void* start_event,
              void* stop_event, int64_t outer_override = 0);
}  // namespace pf
