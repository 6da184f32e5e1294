// Error-scoring kernels (ahead-of-time compiled for gfx950) and the plain copy
// kernel used as the practical bandwidth ceiling.
//
// Scoring follows the validity test of the paper's Definition 3.2 / Eq. 1 with
// the atol/rtol pair of Appendix F: one pass over every (candidate, reference)
// pair computes the largest absolute and relative error, NaN/Inf counts, the
// number of elements outside |a-b| <= atol + rtol*|b|, and whether the two
// buffers are bit-identical.  All comparisons are fp64 on exactly widened
// values and every accumulator is order-independent (max, integer sums), so
// the result does not depend on how the elements are spread over lanes.
#include <hip/hip_runtime.h>

#include "pf.h"
#include "score_dev.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 256;
constexpr int kPerThread = 64;                       // elements per thread per block-chunk
constexpr int kSlots = pf::kScoreSlots;              // partial results per pair (spreads the atomics)
constexpr unsigned long long kChunk = (unsigned long long)kBlock * kPerThread;

template <int DT> struct Elem;                        // DT: pf_dtype
template <> struct Elem<PF_F32> {
    using raw = unsigned int;
    static __device__ __forceinline__ double widen(raw r) { return (double)__uint_as_float(r); }
    // 8 consecutive elements from an address aligned to their size * 8
    static __device__ __forceinline__ void load8(const void* base, unsigned long long i, raw* out) {
        const u32x4* p = (const u32x4*)((const unsigned int*)base + i);
        u32x4 a = __builtin_nontemporal_load(p), b = __builtin_nontemporal_load(p + 1);
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w; out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    }
    static __device__ __forceinline__ raw load1(const void* base, unsigned long long i) { return ((const unsigned int*)base)[i]; }
};
template <> struct Elem<PF_BF16> {
    using raw = unsigned int;                         // bits in the low half
    static __device__ __forceinline__ double widen(raw r) { return (double)__uint_as_float(r << 16); }
    static __device__ __forceinline__ void load8(const void* base, unsigned long long i, raw* out) {
        u32x4 a = __builtin_nontemporal_load((const u32x4*)((const unsigned short*)base + i));
        out[0] = a.x & 0xffffu; out[1] = a.x >> 16; out[2] = a.y & 0xffffu; out[3] = a.y >> 16;
        out[4] = a.z & 0xffffu; out[5] = a.z >> 16; out[6] = a.w & 0xffffu; out[7] = a.w >> 16;
    }
    static __device__ __forceinline__ raw load1(const void* base, unsigned long long i) { return ((const unsigned short*)base)[i]; }
};
template <> struct Elem<PF_F64> {
    using raw = unsigned long long;
    static __device__ __forceinline__ double widen(raw r) { return __longlong_as_double((long long)r); }
    static __device__ __forceinline__ void load8(const void* base, unsigned long long i, raw* out) {
        const u32x4* p = (const u32x4*)((const unsigned long long*)base + i);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            u32x4 a = __builtin_nontemporal_load(p + k);
            out[2 * k] = (unsigned long long)a.x | ((unsigned long long)a.y << 32);
            out[2 * k + 1] = (unsigned long long)a.z | ((unsigned long long)a.w << 32);
        }
    }
    static __device__ __forceinline__ raw load1(const void* base, unsigned long long i) { return ((const unsigned long long*)base)[i]; }
};

// Per-lane accumulators.  The largest relative error needs a correctly rounded
// fp64 division, which is far too slow to run on every element.  Instead each
// lane tracks the running maximum of a cheap fp32 estimate q ~ d/|b| (relative
// error < 1e-6) and keeps the (d, |b|) of that element; only elements whose
// estimate lies within 2e-6 of the running maximum, or whose operands leave
// the range where the estimate is trustworthy, are divided exactly on the
// spot.  An element that is neither kept nor divided is smaller than the kept
// one by more than both estimates can be wrong, so the exact maximum is
// max(exact divisions, kept_d / kept_b), evaluated once per lane at the end.
struct Acc {
    double max_abs = 0.0, max_rel = 0.0;     // max_rel: exact divisions so far
    double keep_d = 0.0, keep_b = 1.0;       // element with the largest estimate (0/1: none yet)
    float keep_q = 0.0f;
    unsigned long long n_viol = 0, bitdiff = 0;
    unsigned int nan_c = 0, nan_r = 0, inf_c = 0, inf_r = 0;
};

__device__ __forceinline__ bool est_range_ok(float x) {   // 1e-18 <= x <= 1e18, false for 0/inf/nan
    return x >= 1e-18f && x <= 1e18f;
}

template <int CD, int RD>
__device__ __forceinline__ void score_one(typename Elem<CD>::raw ra, typename Elem<RD>::raw rb, const pf::PairDev& pr, Acc& acc) {
    const double a = Elem<CD>::widen(ra), b = Elem<RD>::widen(rb);
    if (CD == RD) acc.bitdiff += (ra != rb) ? 1u : 0u;
    const bool na = a != a, nb = b != b;
    acc.nan_c += na;
    acc.nan_r += nb;
    const double inf = __builtin_inf();
    acc.inf_c += (fabs(a) == inf);
    acc.inf_r += (fabs(b) == inf);
    if (na || nb) {
        acc.n_viol += !(pr.equal_nan && na && nb);
        return;
    }
    if (a == b) return;                               // zero error; covers equal infinities and +-0
    const double d = fabs(__dsub_rn(a, b));           // +inf when exactly one side is infinite or signs differ
    const double ab = fabs(b);
    acc.max_abs = fmax(acc.max_abs, d);
    const double allowed = __dadd_rn(pr.atol, __dmul_rn(pr.rtol, ab));
    acc.n_viol += !(d != inf && d <= allowed);
    if (ab == 0.0 || d == inf) {
        acc.max_rel = inf;
        return;
    }
    const float d32 = (float)d, b32 = (float)ab;
    if (est_range_ok(d32) && est_range_ok(b32)) {
        const float q = d32 * __builtin_amdgcn_rcpf(b32);
        if (q > acc.keep_q * 1.000002f) {             // certainly larger than the kept element
            acc.keep_q = q;
            acc.keep_d = d;
            acc.keep_b = ab;
            return;
        }
        if (q < acc.keep_q * 0.999998f) return;       // certainly smaller
    }
    acc.max_rel = fmax(acc.max_rel, __ddiv_rn(d, ab));
}

template <int CD, int RD>
__device__ __forceinline__ void score_chunk(const pf::PairDev& pr, unsigned long long begin, unsigned long long end, Acc& acc) {
    // vectors of 8 elements, lanes interleaved so that a wave reads contiguous memory
    const unsigned long long nvec = (end - begin) / 8;
    for (unsigned long long v = threadIdx.x; v < nvec; v += kBlock) {
        typename Elem<CD>::raw ra[8];
        typename Elem<RD>::raw rb[8];
        Elem<CD>::load8(pr.cand, begin + v * 8, ra);
        Elem<RD>::load8(pr.ref, begin + v * 8, rb);
#pragma unroll
        for (int j = 0; j < 8; ++j) score_one<CD, RD>(ra[j], rb[j], pr, acc);
    }
    for (unsigned long long i = begin + nvec * 8 + threadIdx.x; i < end; i += kBlock)
        score_one<CD, RD>(Elem<CD>::load1(pr.cand, i), Elem<RD>::load1(pr.ref, i), pr, acc);
}

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;
}

// Descriptors travel as kernel arguments (copied at launch), so the host array
// can be released as soon as the call returns and no host-to-device copy has
// to be ordered against the stream.
__global__ void __launch_bounds__(64) score_upload_kernel(pf::PairBatch batch, pf::PairDev* pairs, unsigned long long* block_start) {
    const int i = threadIdx.x;
    if (i < batch.count) {
        pairs[batch.first + i] = batch.pairs[i];
        block_start[batch.first + i] = batch.start[i];
    }
    if (i == 0 && batch.last) block_start[batch.first + batch.count] = batch.start[batch.count];
}

__global__ void __launch_bounds__(kBlock) score_init_kernel(const pf::PairDev* pairs, int n_pairs, pf_score_result* res,
                                                            pf_score_result* slots) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n_pairs * kSlots) {
        pf_score_result z;
        z.max_abs = 0.0; z.max_rel = 0.0; z.n = 0; z.n_viol = 0;
        z.nan_cand = z.nan_ref = z.inf_cand = z.inf_ref = 0;
        z.allclose = 0; z.bit_identical = 0; z.reserved_ = 0;
        slots[p] = z;
    }
    if (p >= n_pairs) return;
    pf_score_result r;
    r.max_abs = 0.0; r.max_rel = 0.0;
    r.n = pairs[p].n; r.n_viol = 0;
    r.nan_cand = r.nan_ref = r.inf_cand = r.inf_ref = 0;
    r.allclose = 0; r.bit_identical = 0; r.reserved_ = 0;
    res[p] = r;
}

__device__ __forceinline__ void raise_max(double* slot, double v) {
    // values only grow, so a stale read can at worst cause a redundant atomic
    const unsigned long long bits = (unsigned long long)__double_as_longlong(v);
    if (bits > __atomic_load_n((unsigned long long*)slot, __ATOMIC_RELAXED)) atomicMax((unsigned long long*)slot, bits);
}

__global__ void __launch_bounds__(kBlock) score_kernel(const pf::PairDev* pairs, const unsigned long long* block_start,
                                                       int n_pairs, pf_score_result* slots) {
    // which pair does this block belong to: largest p with block_start[p] <= blockIdx.x
    int lo = 0, hi = n_pairs;
    const unsigned long long bid = blockIdx.x;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (block_start[mid] <= bid) lo = mid; else hi = mid;
    }
    const pf::PairDev pr = pairs[lo];
    const unsigned long long begin = (bid - block_start[lo]) * kChunk;
    const unsigned long long end = begin + kChunk < pr.n ? begin + kChunk : pr.n;
    Acc acc;
    const int key = pr.cand_dtype * 3 + pr.ref_dtype;
    switch (key) {
        case PF_F32 * 3 + PF_F32: score_chunk<PF_F32, PF_F32>(pr, begin, end, acc); break;
        case PF_F32 * 3 + PF_BF16: score_chunk<PF_F32, PF_BF16>(pr, begin, end, acc); break;
        case PF_F32 * 3 + PF_F64: score_chunk<PF_F32, PF_F64>(pr, begin, end, acc); break;
        case PF_BF16 * 3 + PF_F32: score_chunk<PF_BF16, PF_F32>(pr, begin, end, acc); break;
        case PF_BF16 * 3 + PF_BF16: score_chunk<PF_BF16, PF_BF16>(pr, begin, end, acc); break;
        case PF_BF16 * 3 + PF_F64: score_chunk<PF_BF16, PF_F64>(pr, begin, end, acc); break;
        default: break;
    }
    acc.max_rel = fmax(acc.max_rel, __ddiv_rn(acc.keep_d, acc.keep_b));
    // block reduction: waves by shuffle, then LDS
    __shared__ double s_abs[kBlock / 64], s_rel[kBlock / 64];
    __shared__ unsigned long long s_cnt[kBlock / 64][6];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const double wa = wave_max(acc.max_abs), wr = wave_max(acc.max_rel);
    unsigned long long c[6] = {acc.n_viol, acc.bitdiff, acc.nan_c, acc.nan_r, acc.inf_c, acc.inf_r};
#pragma unroll
    for (int k = 0; k < 6; ++k) c[k] = wave_sum(c[k]);
    if (lane == 0) {
        s_abs[wave] = wa; s_rel[wave] = wr;
#pragma unroll
        for (int k = 0; k < 6; ++k) s_cnt[wave][k] = c[k];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double ma = s_abs[0], mr = s_rel[0];
        unsigned long long t[6];
#pragma unroll
        for (int k = 0; k < 6; ++k) t[k] = s_cnt[0][k];
        for (int w = 1; w < kBlock / 64; ++w) {
            ma = fmax(ma, s_abs[w]); mr = fmax(mr, s_rel[w]);
#pragma unroll
            for (int k = 0; k < 6; ++k) t[k] += s_cnt[w][k];
        }
        // one of kSlots partial results of this pair; the final kernel folds them
        pf_score_result* r = slots + (size_t)lo * kSlots + (bid - block_start[lo]) % kSlots;
        // errors are >= 0 and never NaN, so their bit patterns order like the values
        if (ma > 0.0) raise_max(&r->max_abs, ma);
        if (mr > 0.0) raise_max(&r->max_rel, mr);
        if (t[0]) atomicAdd((unsigned long long*)&r->n_viol, t[0]);
        if (t[1]) atomicAdd((unsigned long long*)&r->reserved_, t[1]);
        if (t[2]) atomicAdd((unsigned long long*)&r->nan_cand, t[2]);
        if (t[3]) atomicAdd((unsigned long long*)&r->nan_ref, t[3]);
        if (t[4]) atomicAdd((unsigned long long*)&r->inf_cand, t[4]);
        if (t[5]) atomicAdd((unsigned long long*)&r->inf_ref, t[5]);
    }
}

__global__ void __launch_bounds__(kBlock) score_final_kernel(const pf::PairDev* pairs, int n_pairs, pf_score_result* res,
                                                             const pf_score_result* slots) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n_pairs) return;
    pf_score_result r = res[p];
    for (int k = 0; k < kSlots; ++k) {
        const pf_score_result& s = slots[(size_t)p * kSlots + k];
        r.max_abs = fmax(r.max_abs, s.max_abs);
        r.max_rel = fmax(r.max_rel, s.max_rel);
        r.n_viol += s.n_viol;
        r.reserved_ += s.reserved_;
        r.nan_cand += s.nan_cand; r.nan_ref += s.nan_ref;
        r.inf_cand += s.inf_cand; r.inf_ref += s.inf_ref;
    }
    r.allclose = r.n_viol == 0 ? 1u : 0u;
    r.bit_identical = (pairs[p].cand_dtype == pairs[p].ref_dtype && r.reserved_ == 0) ? 1u : 0u;
    res[p] = r;
}

__global__ void __launch_bounds__(256) copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, unsigned long long n16) {
    const unsigned long long base = (unsigned long long)blockIdx.x * (256 * 4) + threadIdx.x;
    if (base + 3 * 256 < n16) {
        u32x4 r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(r[u], dst + base + u * 256);
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (base + u * 256 < n16) dst[base + u * 256] = src[base + u * 256];
    }
}

}  // namespace

namespace pf {

unsigned long long score_chunk_elems() { return kChunk; }

hipError_t launch_score_upload(const PairBatch& batch, PairDev* d_pairs, unsigned long long* d_block_start, hipStream_t stream) {
    hipLaunchKernelGGL(score_upload_kernel, dim3(1), dim3(64), 0, stream, batch, d_pairs, d_block_start);
    return hipGetLastError();
}

hipError_t launch_score(const PairDev* d_pairs, const unsigned long long* d_block_start, int n_pairs,
                        unsigned long long total_blocks, pf_score_result* d_results, pf_score_result* d_slots, hipStream_t stream) {
    const int nb = (n_pairs + kBlock - 1) / kBlock;
    const int nbs = (n_pairs * kSlots + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(score_init_kernel, dim3(nbs), dim3(kBlock), 0, stream, d_pairs, n_pairs, d_results, d_slots);
    if (total_blocks)
        hipLaunchKernelGGL(score_kernel, dim3((unsigned)total_blocks), dim3(kBlock), 0, stream, d_pairs, d_block_start, n_pairs,
                           d_slots);
    hipLaunchKernelGGL(score_final_kernel, dim3(nb), dim3(kBlock), 0, stream, d_pairs, n_pairs, d_results, d_slots);
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
    const unsigned long long n16 = bytes / 16;
    const unsigned long long blocks = (n16 + 1023) / 1024;
    if (blocks) hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (u32x4*)dst, (const u32x4*)src, n16);
    return hipGetLastError();
}

}  // namespace pf
