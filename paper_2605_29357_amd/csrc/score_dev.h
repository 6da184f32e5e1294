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
    unsigned long long chunk;   // elements per workgroup
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

constexpr int kScoreSlots = 64;   // partial result slots per pair
constexpr int kScoreSeedParts = 16;   // sampled maxima per pair (two doubles each), folded by every reader

// up to kPairBatch descriptors passed by value to the staging kernel (kernel arguments are limited to 4 KB)
constexpr int kPairBatch = 48;
struct PairBatch {
    PairDev pairs[kPairBatch];
    unsigned long long start[kPairBatch + 1];   // first block of each pair (+ total when last)
    int first, count, last, pad_;
};

static_assert(sizeof(PairBatch) + 64 <= 4096, "a batch of descriptors and the other kernel arguments must fit in 4 KB");

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
static_assert(sizeof(PairBatch) + sizeof(LadderRow) + 64 <= 4096, "batch + tolerances must fit the kernel arguments");

unsigned long long score_chunk_elems(unsigned long long n);
hipError_t launch_ladder_stage(const PairBatch& batch, PairDev* d_pairs, unsigned long long* d_block_start, pf_ladder_result* d_slots,
                               hipStream_t stream);
hipError_t launch_ladder_small(const PairBatch& batch, int cd, int rd, const LadderTable& table, pf_ladder_result* d_results,
                               hipStream_t stream);
hipError_t launch_ladder(const PairDev* d_pairs, const unsigned long long* d_block_start, int n_pairs, const ScoreRanges& ranges,
                         const LadderTable& table, pf_ladder_result* d_results, pf_ladder_result* d_slots, hipStream_t stream);
// descriptor upload, slot clearing and seeding of one batch in a single launch (the single-level scorer)
hipError_t launch_score_stage(const PairBatch& batch, PairDev* d_pairs, unsigned long long* d_block_start, pf_score_result* d_slots,
                              double* d_seeds, hipStream_t stream);
hipError_t launch_score(const PairDev* d_pairs, const unsigned long long* d_block_start, int n_pairs, const ScoreRanges& ranges,
                        pf_score_result* d_results, pf_score_result* d_slots, const double* d_seeds, hipStream_t stream);
// pairs of at most score_small_pair_elems() elements: one workgroup per pair, results written directly
unsigned long long score_small_pair_elems();
hipError_t launch_score_small(const PairBatch& batch, int cd, int rd, pf_score_result* d_results, hipStream_t stream);
// at most kPairBatch pairs of at most kScoreSlots chunks each, descriptors as kernel arguments: main kernels + fold
hipError_t launch_score_direct(const PairBatch& batch, const ScoreRanges& ranges, pf_score_result* d_results, pf_score_result* d_slots,
                               hipStream_t stream);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);

// The workspace of pf_score_static: an array inside the library's code object.  Looks its address up
// on the current device the first time it is asked for there; never allocates.
#define PF_STATIC_SCRATCH_BYTES (1536 * 1024)
hipError_t static_scratch(void** d_ptr, size_t* bytes);

}  // namespace pf
