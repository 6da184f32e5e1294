// Device-visible descriptor of one (candidate, reference) pair and the launch
// entry points of the ahead-of-time compiled kernels.
#pragma once
#include <hip/hip_runtime_api.h>

#include "pf.h"

namespace pf {

struct PairDev {
    const void* cand;
    const void* ref;
    unsigned long long n;
    int cand_dtype, ref_dtype;
    double rtol, atol;
    int equal_nan;
    int orig;               // index of this pair in the caller's array
    unsigned long long chunk;   // elements per chunk (a multiple of 2048)
    unsigned long long wgs;     // workgroups of this pair: workgroup w walks chunks w, w + wgs, w + 2 wgs, ...
};

// blocks of each (candidate dtype, reference dtype) combination, indexed by pf_dtype: a contiguous range
struct ScoreRanges {
    unsigned long long first[4][4];
    unsigned long long count[4][4];
};
// combinations with a kernel instantiation: candidate f32 / bf16 / f16 against a reference of the
// same dtype, f32 or f64; an f32 candidate also against a bf16 or f16 reference
inline bool score_combo_supported(int cd, int rd) {
    if (cd == PF_F64 || cd < 0 || cd > PF_F16 || rd < 0 || rd > PF_F16) return false;
    if (cd == PF_BF16 && rd == PF_F16) return false;
    if (cd == PF_F16 && rd == PF_BF16) return false;
    return true;
}

constexpr int kScoreSlots = 64;       // partial result slots per pair (spread the atomics of its workgroups)
constexpr unsigned long long kScoreMaxTargetWGs = 12288;  // score_target_wgs() never asks for more
constexpr int kScoreSeedParts = 16;   // sampled maxima per pair (two doubles each), folded by every reader
// Where the parts of a call's workspace lie (device pointers; sslots / lslots are NULL when that result is not wanted).
struct ScoreSpace {
    struct PairDev* pairs;            // [n_pairs] descriptors, ordered by dtype combination
    unsigned long long* start;        // [n_pairs + 1] first workgroup of each pair
    int* wg_pair;                     // [workgroups of the call] the pair each workgroup of the walking kernel works on
    unsigned int* tickets;            // [n_pairs][1 + kScoreSlots] finished: slots of the pair, workgroups of each slot
    double* seeds;                    // [n_pairs][kScoreSeedParts][2]
    pf_score_result* sslots;          // [n_pairs][kScoreSlots]
    pf_ladder_result* lslots;         // [n_pairs][kScoreSlots]
};

// up to kPairBatch descriptors passed by value to a kernel (kernel arguments are limited to 4 KB)
constexpr int kPairBatch = 42;
struct PairBatch {
    PairDev pairs[kPairBatch];
    unsigned long long start[kPairBatch + 1];   // first workgroup of each pair (+ total when last)
    int first, count, last, pad_;
};

// tolerances of every ladder level, per candidate dtype (indexed by pf_dtype; the f64 row is unused)
struct LadderTable {
    double rtol[4][PF_LADDER_LEVELS];
    double atol[4][PF_LADDER_LEVELS];
};

// the tolerances of one candidate dtype (what a one-workgroup-per-pair ladder launch carries besides its batch)
struct LadderRow {
    double rtol[PF_LADDER_LEVELS];
    double atol[PF_LADDER_LEVELS];
};

static_assert(sizeof(PairBatch) + sizeof(LadderRow) + 128 <= 4096, "a batch of descriptors, the tolerances and the other kernel arguments must fit in 4 KB");

unsigned long long score_chunk_elems(unsigned long long call_elems, bool ladder);
unsigned long long score_target_wgs(bool ladder, int n_pairs);
// pairs of at most score_small_pair_elems() elements: one workgroup per pair, results written directly
unsigned long long score_small_pair_elems();
// descriptors, cleared slots and tickets, and seeds of one batch of pairs, in one launch
hipError_t launch_stage(const PairBatch& batch, const ScoreSpace& sp, hipStream_t stream);
// the walking kernels (one launch per dtype combination present); d_sres / d_lres: either may be NULL
hipError_t launch_pairs(const ScoreSpace& sp, const ScoreRanges& ranges, const LadderTable& table, pf_score_result* d_sres,
                        pf_ladder_result* d_lres, hipStream_t stream);
hipError_t launch_small(const PairBatch& batch, int cd, int rd, const LadderTable& table, pf_score_result* d_sres, pf_ladder_result* d_lres,
                        hipStream_t stream);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);

// The workspace of pf_score_static: an array inside the library's code object.  Looks its address up
// on the current device the first time it is asked for there; never allocates.
#define PF_STATIC_SCRATCH_BYTES (1536 * 1024)
hipError_t static_scratch(void** d_ptr, size_t* bytes);

}  // namespace pf
