// Runtime: JIT compilation of generated kernels (hipRTC), code-object cache,
// lazy module loading and launches.
#include <hip/hip_runtime_api.h>
#include <hip/hip_ext.h>
#include <hip/hiprtc.h>

#include <dirent.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <mutex>
#include <unordered_map>

#include "exec.h"
#include "pf_internal.h"

namespace pf {

namespace {

std::mutex g_cache_mu;
std::unordered_map<std::string, std::vector<char>> g_code_cache;   // source text -> code object
pf_jit_stats g_stats = {0, 0, 0, 0};                                // guarded by g_cache_mu

uint64_t fnv1a(const std::string& s) {
    uint64_t h = 1469598103934665603ull;
    for (unsigned char c : s) {
        h ^= c;
        h *= 1099511628211ull;
    }
    return h;
}

constexpr const char* kArch = "gfx950";

// What a cached code object depends on besides the source text: the compiler that made it and the
// target it was made for.  Both go into the file name's hash and into the file's header, so an object
// left behind by another ROCm release (or another target) is never picked up.
const std::string& toolchain_tag() {
    static const std::string tag = [] {
        int major = 0, minor = 0;
        if (hiprtcVersion(&major, &minor) != HIPRTC_SUCCESS) major = minor = -1;
        return strf("hiprtc %d.%d %s -O3", major, minor, kArch);
    }();
    return tag;
}

std::string disk_path(const std::string& source) {
    const char* dir = getenv("PF_CACHE_DIR");
    if (!dir || !*dir) return "";
    return strf("%s/pf_%016llx_%zu.pfk", dir, (unsigned long long)fnv1a(toolchain_tag() + "\n" + source), source.size());
}

// file = "PFCACHE2", u64 tag length, u64 source length, tag, source, code object
bool read_cached(const std::string& path, const std::string& source, std::vector<char>& code) {
    std::ifstream f(path, std::ios::binary);
    if (!f) return false;
    std::vector<char> blob((std::istreambuf_iterator<char>(f)), std::istreambuf_iterator<char>());
    const std::string& tag = toolchain_tag();
    uint64_t tlen = 0, slen = 0;
    if (blob.size() <= 24 || memcmp(blob.data(), "PFCACHE2", 8) != 0) return false;
    memcpy(&tlen, blob.data() + 8, 8);
    memcpy(&slen, blob.data() + 16, 8);
    if (tlen != tag.size() || slen != source.size() || blob.size() <= 24 + tlen + slen) return false;
    if (memcmp(blob.data() + 24, tag.data(), tlen) != 0 || memcmp(blob.data() + 24 + tlen, source.data(), slen) != 0) return false;
    code.assign(blob.begin() + 24 + tlen + slen, blob.end());
    return true;
}

// The cache directory is bounded: past PF_CACHE_MAX_MB (default 256) the least recently written files go,
// down to three quarters of the limit.  Checked at a process's first write and every 64th after it.
void trim_cache_dir(const char* dir) {
    static std::atomic<unsigned> writes{0};
    if (writes.fetch_add(1) % 64 != 0) return;
    uint64_t limit = 256;
    if (const char* v = getenv("PF_CACHE_MAX_MB")) limit = strtoull(v, nullptr, 10);
    limit <<= 20;
    DIR* d = opendir(dir);
    if (!d) return;
    struct Ent { std::string path; uint64_t size; time_t mtime; };
    std::vector<Ent> ents;
    uint64_t total = 0;
    while (dirent* de = readdir(d)) {
        const std::string name = de->d_name;
        if (name.size() < 5 || name.compare(name.size() - 4, 4, ".pfk") != 0) continue;
        struct stat st;
        const std::string path = std::string(dir) + "/" + name;
        if (stat(path.c_str(), &st) != 0) continue;
        ents.push_back({path, (uint64_t)st.st_size, st.st_mtime});
        total += (uint64_t)st.st_size;
    }
    closedir(d);
    if (total <= limit) return;
    std::sort(ents.begin(), ents.end(), [](const Ent& a, const Ent& b) { return a.mtime < b.mtime; });
    for (const Ent& e : ents) {
        if (total <= limit / 4 * 3) break;
        if (remove(e.path.c_str()) == 0) total -= e.size;
    }
}

}  // namespace

void jit_compile(Group& grp) {
    {
        std::lock_guard<std::mutex> lk(g_cache_mu);
        auto it = g_code_cache.find(grp.source);
        if (it != g_code_cache.end()) {
            grp.code = it->second;
            ++g_stats.memory_hits;
            return;
        }
    }
    // on-disk cache: a file holds the toolchain tag and the full source text ahead of the code
    // object, and is used only if both match byte for byte
    const std::string path = disk_path(grp.source);
    if (!path.empty() && read_cached(path, grp.source, grp.code)) {
        std::lock_guard<std::mutex> lk(g_cache_mu);
        g_code_cache[grp.source] = grp.code;
        ++g_stats.disk_hits;
        return;
    }
    hiprtcProgram prog;
    if (hiprtcCreateProgram(&prog, grp.source.c_str(), (grp.kernel_name + ".hip").c_str(), 0, nullptr, nullptr) != HIPRTC_SUCCESS)
        fail(PF_E_COMPILE, "hiprtcCreateProgram failed");
    // packed fp32 instructions are kept out of generated code on purpose
    const char* opts[] = {"--offload-arch=gfx950" /* kArch */, "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    hiprtcResult r = hiprtcCompileProgram(prog, (int)(sizeof opts / sizeof opts[0]), opts);
    if (r != HIPRTC_SUCCESS) {
        size_t n = 0;
        hiprtcGetProgramLogSize(prog, &n);
        std::string log(n, '\0');
        if (n) hiprtcGetProgramLog(prog, log.data());
        hiprtcDestroyProgram(&prog);
        if (getenv("PF_DUMP_FAILED")) fprintf(stderr, "%s\n", grp.source.c_str());
        fail(PF_E_COMPILE, "JIT compilation of %s failed: %s\n%.1500s", grp.kernel_name.c_str(), hiprtcGetErrorString(r), log.c_str());
    }
    size_t sz = 0;
    hiprtcGetCodeSize(prog, &sz);
    grp.code.resize(sz);
    hiprtcGetCode(prog, grp.code.data());
    hiprtcDestroyProgram(&prog);
    if (!path.empty()) {
        const std::string tmp = strf("%s.%d.tmp", path.c_str(), (int)getpid());
        std::ofstream f(tmp, std::ios::binary);
        if (f) {
            const std::string& tag = toolchain_tag();
            const uint64_t tlen = tag.size(), slen = grp.source.size();
            f.write("PFCACHE2", 8);
            f.write((const char*)&tlen, 8);
            f.write((const char*)&slen, 8);
            f.write(tag.data(), (std::streamsize)tlen);
            f.write(grp.source.data(), (std::streamsize)slen);
            f.write(grp.code.data(), (std::streamsize)grp.code.size());
            f.close();
            if (f.good()) rename(tmp.c_str(), path.c_str());
            else remove(tmp.c_str());
            trim_cache_dir(getenv("PF_CACHE_DIR"));
        }
    }
    std::lock_guard<std::mutex> lk(g_cache_mu);
    g_code_cache[grp.source] = grp.code;
    ++g_stats.compiled;
}

void jit_stats(pf_jit_stats* out) {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    *out = g_stats;
    out->code_objects = g_code_cache.size();
}

void exec_load(pf_exec& e) {
    std::lock_guard<std::mutex> lk(e.load_mu);
    if (e.loaded) return;
    e.modules.assign(e.plan.groups.size(), nullptr);
    e.functions.assign(e.plan.groups.size(), nullptr);
    e.functions2.assign(e.plan.groups.size(), nullptr);
    for (size_t i = 0; i < e.plan.groups.size(); ++i) {
        Group& grp = e.plan.groups[i];
        // a failure part-way leaves nothing loaded: the modules of the earlier groups are released again
        auto give_up = [&](const char* what, const std::string& name, hipError_t err) {
            for (void*& m : e.modules)
                if (m) {
                    (void)hipModuleUnload((hipModule_t)m);
                    m = nullptr;
                }
            fail(PF_E_RUNTIME, "%s(%s): %s", what, name.c_str(), hipGetErrorString(err));
        };
        hipModule_t mod = nullptr;
        hipError_t err = hipModuleLoadData(&mod, grp.code.data());
        if (err != hipSuccess) give_up("hipModuleLoadData", grp.kernel_name, err);
        e.modules[i] = mod;
        hipFunction_t fn = nullptr;
        err = hipModuleGetFunction(&fn, mod, grp.kernel_name.c_str());
        if (err != hipSuccess) give_up("hipModuleGetFunction", grp.kernel_name, err);
        e.functions[i] = fn;
        if (!grp.kernel2_name.empty()) {
            err = hipModuleGetFunction(&fn, mod, grp.kernel2_name.c_str());
            if (err != hipSuccess) give_up("hipModuleGetFunction", grp.kernel2_name, err);
            e.functions2[i] = fn;
        }
    }
    e.loaded = true;
}

void exec_unload(pf_exec& e) {
    for (void* m : e.modules)
        if (m) (void)hipModuleUnload((hipModule_t)m);
    e.modules.clear();
    e.functions.clear();
    e.functions2.clear();
    e.loaded = false;
}

void exec_run(pf_exec& e, const void* const* d_inputs, void* const* d_outputs, void* d_ws, void* stream, void* start_event,
              void* stop_event, int64_t outer_override) {
    exec_load(e);
    for (size_t i = 0; i < e.plan.groups.size(); ++i) {
        Group& grp = e.plan.groups[i];
        void* ptrs[kMaxKernelArgs];
        void* args[kMaxKernelArgs];
        int n = 0;
        for (auto& o : grp.operands) {
            const void* p = o.graph_input >= 0    ? d_inputs[o.graph_input]
                            : o.ws_offset >= 0    ? (const void*)((const char*)d_ws + o.ws_offset)
                                                  : (const void*)d_outputs[o.graph_output];
            ptrs[n++] = (void*)p;
        }
        for (auto& s : grp.stores) {
            ptrs[n++] = s.graph_output >= 0 ? d_outputs[s.graph_output] : (void*)((char*)d_ws + s.ws_offset);
            for (int k : s.also_outputs) ptrs[n++] = d_outputs[k];
        }
        for (int k = 0; k < n; ++k) args[k] = &ptrs[k];
        long long outer = outer_override > 0 ? outer_override : grp.outer_extent;
        const int64_t grid1 = outer_override > 0 ? (outer * grp.rt_per_outer + grp.rt_per_block - 1) / grp.rt_per_block : grp.grid;
        if (grp.outer_runtime) args[n++] = &outer;
        if (grp.scratch_bytes) {
            ptrs[n] = (char*)d_ws + grp.scratch_offset;
            args[n] = &ptrs[n];
            ++n;
        }
        // the riders' pointers follow the host's own arguments, rider by rider: operands, then results
        for (auto& rd : grp.riders) {
            for (auto& o : rd.operands) {
                ptrs[n] = o.graph_input >= 0 ? (void*)d_inputs[o.graph_input]
                          : o.ws_offset >= 0 ? (void*)((char*)d_ws + o.ws_offset)
                                             : (void*)d_outputs[o.graph_output];
                args[n] = &ptrs[n];
                ++n;
            }
            for (auto& st : rd.stores) {
                ptrs[n] = st.graph_output >= 0 ? d_outputs[st.graph_output] : (void*)((char*)d_ws + st.ws_offset);
                args[n] = &ptrs[n];
                ++n;
                for (int k : st.also_outputs) {
                    ptrs[n] = d_outputs[k];
                    args[n] = &ptrs[n];
                    ++n;
                }
            }
        }
        // events, when given, bracket the kernels themselves (dispatch timestamps), not the
        // launch calls: the first kernel carries the start event, the last one the stop event
        const bool two = e.functions2[i] != nullptr;
        hipEvent_t ev0 = i == 0 ? (hipEvent_t)start_event : nullptr;
        hipEvent_t ev1 = i + 1 == e.plan.groups.size() ? (hipEvent_t)stop_event : nullptr;
        auto launch = [&](void* fn, int64_t grid, int block, hipEvent_t a, hipEvent_t b) -> hipError_t {
            // one-dimensional launches: more workgroups than the grid can count would silently wrap
            if (grid < 1 || grid > 0x7fffffffLL)
                fail(PF_E_RUNTIME, "%s would need %lld workgroups; a launch holds at most 2^31 - 1", grp.kernel_name.c_str(), (long long)grid);
            if ((a || b) && (uint64_t)grid * (uint64_t)block < (1ull << 32))
                return hipExtModuleLaunchKernel((hipFunction_t)fn, (uint32_t)(grid * block), 1, 1, (uint32_t)block, 1, 1, 0, (hipStream_t)stream,
                                                args, nullptr, a, b, 0);
            if (a) (void)hipEventRecord(a, (hipStream_t)stream);
            hipError_t r = hipModuleLaunchKernel((hipFunction_t)fn, (unsigned)grid, 1, 1, (unsigned)block, 1, 1, 0, (hipStream_t)stream, args, nullptr);
            if (b && r == hipSuccess) (void)hipEventRecord(b, (hipStream_t)stream);
            return r;
        };
        hipError_t err = launch(e.functions[i], grid1, grp.block, ev0, two ? nullptr : ev1);
        if (err == hipSuccess && two) err = launch(e.functions2[i], grp.grid2, grp.block2, nullptr, ev1);
        if (err != hipSuccess) fail(PF_E_RUNTIME, "launch of %s failed: %s", grp.kernel_name.c_str(), hipGetErrorString(err));
    }
}

}  // namespace pf
