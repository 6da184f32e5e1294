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

#include <mutex>

#include "pf.h"
#include "score_dev.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 256;
constexpr int kPerThread = 64;                       // elements per thread per block-chunk (small pairs)
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
template <> struct Elem<PF_F16> {
    using raw = unsigned int;                         // IEEE binary16 bits in the low half
    static __device__ __forceinline__ float widen32(raw r) { return (float)__builtin_bit_cast(_Float16, (unsigned short)r); }
    static __device__ __forceinline__ double widen(raw r) { return (double)widen32(r); }
    static __device__ __forceinline__ void load8(const void* base, unsigned long long i, raw* out) { Elem<PF_BF16>::load8(base, i, out); }
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

// One element, entirely in fp64, every quantity exact (the definition itself).
template <int CD, int RD>
__device__ __forceinline__ void score_exact(typename Elem<CD>::raw ra, typename Elem<RD>::raw rb, const pf::PairDev& pr, Acc& acc) {
    const double a = Elem<CD>::widen(ra), b = Elem<RD>::widen(rb);
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
    if (a == b) return;
    const double d = fabs(__dsub_rn(a, b));
    const double ab = fabs(b);
    acc.max_abs = fmax(acc.max_abs, d);
    const double allowed = __dadd_rn(pr.atol, __dmul_rn(pr.rtol, ab));
    acc.n_viol += !(d != inf && d <= allowed);
    // a division only where the quotient can exceed the running maximum:
    // d <= max_rel * |b| * (1 - 2^-50) implies RN(d / |b|) <= max_rel
    if (ab == 0.0 || d == inf) acc.max_rel = inf;
    else if (d > acc.max_rel * ab * 0.999999999999999) acc.max_rel = fmax(acc.max_rel, __ddiv_rn(d, ab));
}

template <int CD, int RD>
__device__ __forceinline__ void score_chunk(const pf::PairDev& pr, unsigned long long begin, unsigned long long end, Acc& acc) {
    // vectors of 8 elements, lanes interleaved so that a wave reads contiguous memory
    const unsigned long long nvec = (end - begin) / 8;
    const unsigned int nthr = blockDim.x;          // 256 in the main kernel, 1024 in the one-workgroup-per-pair kernel
    for (unsigned long long v = threadIdx.x; v < nvec; v += nthr) {
        typename Elem<CD>::raw ra[8];
        typename Elem<RD>::raw rb[8];
        Elem<CD>::load8(pr.cand, begin + v * 8, ra);
        Elem<RD>::load8(pr.ref, begin + v * 8, rb);
#pragma unroll
        for (int j = 0; j < 8; ++j) score_one<CD, RD>(ra[j], rb[j], pr, acc);
    }
    for (unsigned long long i = begin + nvec * 8 + threadIdx.x; i < end; i += nthr)
        score_one<CD, RD>(Elem<CD>::load1(pr.cand, i), Elem<RD>::load1(pr.ref, i), pr, acc);
}

__device__ __forceinline__ double wave_max(double v);

// ---- fp32 screening path (both sides f32, bf16 or fp16) ---------------------
// Almost every element can be classified without fp64: with a, b widened to
// fp32, d32 = |a - b| carries a relative error of 2^-24 (and is exact when it
// is subnormal), so comparing it against thresholds that are pulled 2e-6 to
// the safe side decides "certainly inside the tolerance", "certainly outside",
// "certainly not a new maximum of |a-b| or of |a-b|/|b|".  A vector of eight
// elements in which any element is not decided this way (or is NaN/Inf) is
// re-evaluated exactly in fp64, element by element, by score_one; the fast
// counts of that vector are then discarded.  The maxima thresholds are shared
// by the wave and follow the exact maxima found so far, so the exact path
// runs only O(log n) times per wave plus once per genuine near-tie.
struct Screen {
    float rtol_lo, atol_lo, rtol_hi, atol_hi;   // tolerance pulled 2e-6 inwards / outwards
    bool viol_decidable;                         // false: tolerances too small for fp32 screening
};

__device__ __forceinline__ Screen make_screen(const pf::PairDev& pr) {
    Screen sc;
    sc.rtol_lo = (float)(pr.rtol * (1.0 - 2e-6));
    sc.atol_lo = (float)(pr.atol * (1.0 - 2e-6));
    sc.rtol_hi = (float)(pr.rtol * (1.0 + 2e-6));
    sc.atol_hi = (float)(pr.atol * (1.0 + 2e-6));
    const bool r_ok = pr.rtol == 0.0 || pr.rtol >= 1e-30, a_ok = pr.atol == 0.0 || pr.atol >= 1e-30;
    sc.viol_decidable = r_ok && a_ok;
    return sc;
}

// Eight consecutive elements as loaded: packed 32-bit words (4 for bf16 / fp16, 8 for f32).
template <int DT> struct Vec8 {
    static constexpr bool HALF = DT == PF_BF16 || DT == PF_F16;
    static constexpr int NW = HALF ? 4 : 8;
    unsigned int w[NW];
    __device__ __forceinline__ void load(const void* base, unsigned long long i) {
        // the buffers are device memory: say so, or the accesses are compiled as generic (flat) ones
        typedef const __attribute__((address_space(1))) u32x4* gptr;
        const gptr p = (gptr)((const char*)base + i * (HALF ? 2 : 4));
#pragma unroll
        for (int k = 0; k < NW / 4; ++k) {
            const u32x4 r = __builtin_nontemporal_load(p + k);
            w[4 * k] = r.x; w[4 * k + 1] = r.y; w[4 * k + 2] = r.z; w[4 * k + 3] = r.w;
        }
    }
    // element j widened to fp32 (exact)
    __device__ __forceinline__ float f32(int j) const {
        if (DT == PF_BF16) return __uint_as_float((j & 1) ? (w[j >> 1] & 0xffff0000u) : (w[j >> 1] << 16));
        if (DT == PF_F16) return Elem<PF_F16>::widen32((j & 1) ? (w[j >> 1] >> 16) : (w[j >> 1] & 0xffffu));
        return __uint_as_float(w[j]);
    }
    // a raw element widened to fp32 (exact)
    static __device__ __forceinline__ float widen32(unsigned int r) {
        if (DT == PF_BF16) return __uint_as_float(r << 16);
        if (DT == PF_F16) return Elem<PF_F16>::widen32(r);
        return __uint_as_float(r);
    }
    // element j as Elem<DT>::raw
    __device__ __forceinline__ unsigned int raw(int j) const {
        if (HALF) return (j & 1) ? (w[j >> 1] >> 16) : (w[j >> 1] & 0xffffu);
        return w[j];
    }
};

template <int CD, int RD>
__device__ __forceinline__ void score_chunk_fast(const pf::PairDev& pr, unsigned long long begin, unsigned long long end, Acc& acc,
                                                 double seed_abs, double seed_rel) {
    const Screen sc = make_screen(pr);
    const int zero_tol = (pr.rtol == 0.0) & (pr.atol == 0.0);
    const int force_exact = !sc.viol_decidable;
    // the lean screen needs an absolute tolerance fp32 can represent comfortably (then every allowed
    // error bound is >= 1e-30 and needs no guard of its own)
    const bool lean = !force_exact && sc.atol_lo >= 1e-30f;
    // Errors of real elements this lane knows of (the pair's sampled seed and its own maximum): the
    // screening thresholds are their fp32 lower bounds, per lane.  Nothing is exchanged while the
    // kernel runs; every scheme tried cost more than it saved in a kernel of short-lived waves:
    // cross-lane shuffles ~1400 cycles of latency per exchange, a read-before-atomic on global
    // memory ~3000, and atomics of many waves on one address serialise (up to a 4x slower kernel).
    double known_abs = seed_abs, known_rel = seed_rel;
    float thr_abs, thr_rel;
    auto refresh = [&]() {
        const float ka = (float)known_abs, kr = (float)known_rel;     // the rounding is far inside the 2e-6 pulled off below
        thr_abs = ka >= 1e-30f ? ka * 0.999998f : 0.0f;
        thr_rel = kr >= 1e-30f ? kr * 0.999998f : 0.0f;
    };
    refresh();
    unsigned int xor_acc = 0;
    const unsigned long long nvec = (end - begin) / 8;
    const unsigned int nthr = blockDim.x;
    const unsigned long long iters = (nvec + nthr - 1) / nthr;
    // the next vector is already on its way while the current one is screened (two vectors ahead
    // cost registers, hence resident waves, and measured 7% slower)
    Vec8<CD> na;
    Vec8<RD> nb;
    if (threadIdx.x < nvec) {
        na.load(pr.cand, begin + (unsigned long long)threadIdx.x * 8);
        nb.load(pr.ref, begin + (unsigned long long)threadIdx.x * 8);
    }
    for (unsigned long long it = 0; it < iters; ++it) {
        const unsigned long long v = it * nthr + threadIdx.x;
        const bool live = v < nvec;
        const Vec8<CD> va = na;
        const Vec8<RD> vb = nb;
        if (v + nthr < nvec) {
            na.load(pr.cand, begin + (v + nthr) * 8);
            nb.load(pr.ref, begin + (v + nthr) * 8);
        }
        unsigned int fmask = 0;          // bit j: element j needs the exact path
        unsigned int nv = 0;
        // full classification of element j: certainly inside the tolerance, certainly outside (counted
        // here), or flagged for the exact path (undecided, NaN/Inf, possible new maximum).  Branch-free on
        // purpose (bitwise | and &): short-circuit forms turn into exec-mask juggling.
        auto classify = [&](int j) {
            const float a = va.f32(j), b = vb.f32(j);
            const float d = fabsf(a - b), ab = fabsf(b);
            const float lo = __builtin_fmaf(sc.rtol_lo, ab, sc.atol_lo);
            const float hi = __builtin_fmaf(sc.rtol_hi, ab, sc.atol_hi);
            // thresholds below 1e-30 are too close to the fp32 subnormal range to be trusted
            const int ok = (d == 0.0f) | ((d <= lo) & (lo >= 1e-30f));
            const int out = (d > hi) & ((hi >= 1e-30f) | zero_tol);
            const float pr_rel = thr_rel * ab;
            const int f = (!(ok | out)) | (!(d < __builtin_inff())) | (d > thr_abs) | (d > pr_rel) | ((pr_rel < 1e-30f) & (d != 0.0f)) |
                          force_exact;
            nv += out & !f;
            fmask |= (unsigned)f << j;
        };
        if (live) {
            if (CD == RD) {
#pragma unroll
                for (int k = 0; k < Vec8<CD>::NW; ++k) xor_acc |= va.w[k] ^ vb.w[k];
            }
            if (lean) {
                // One bound per element, one comparison: an element passes when |a-b| <= m with
                //   m = clamp(thr_rel |b| - 1e-30, 0, min(rtol_lo |b| + atol_lo, thr_abs)),
                // i.e. inside the tolerance, not a new maximum of either error, and (the lower clamp)
                // never a non-zero error against a reference too small for fp32 to judge.  NaN and
                // infinities fail the comparison.
                const float ta = fminf(thr_abs, 3.0e38f), tr = fminf(thr_rel, 3.0e38f);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float a = va.f32(j), b = vb.f32(j);
                    const float d = fabsf(a - b), ab = fabsf(b);
                    const float lo = __builtin_fmaf(sc.rtol_lo, ab, sc.atol_lo);
                    const float m = __builtin_amdgcn_fmed3f(__builtin_fmaf(tr, ab, -1e-30f), 0.0f, fminf(lo, ta));
                    fmask |= (d <= m) ? 0u : (1u << j);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) classify(j);
            }
        }
        acc.n_viol += nv;                // violations the full classification decided on its own
        if (__any(fmask != 0)) {
            // the flagged elements only; the trip count is the largest number of flagged elements in
            // any lane of the wave
            while (fmask) {
                const int j = __builtin_ctz(fmask);
                fmask &= fmask - 1;
                unsigned int ea = va.raw(0), eb = vb.raw(0);
#pragma unroll
                for (int t = 1; t < 8; ++t) { ea = j == t ? va.raw(t) : ea; eb = j == t ? vb.raw(t) : eb; }
                if (lean) {
                    // certainly outside the tolerance and certainly no new maximum: counted without fp64
                    const float a = Vec8<CD>::widen32(ea), b = Vec8<RD>::widen32(eb);
                    const float d = fabsf(a - b), ab = fabsf(b);
                    const float hi = __builtin_fmaf(sc.rtol_hi, ab, sc.atol_hi), pr_rel = thr_rel * ab;
                    if ((d > hi) & (d < __builtin_inff()) & (d <= thr_abs) & (d <= pr_rel) & (pr_rel >= 1e-30f)) {
                        acc.n_viol += 1;
                        continue;
                    }
                    // certainly inside the tolerance: exactly no new maximum either?  (fp64, no division; the
                    // many elements of quantised data that tie a known maximum end here)
                    if ((d <= __builtin_fmaf(sc.rtol_lo, ab, sc.atol_lo)) & (d < __builtin_inff()) & (ab < __builtin_inff())) {
                        const double d64 = fabs(__dsub_rn((double)a, (double)b)), ab64 = fabs((double)b);
                        if ((d64 <= known_abs) & (d64 <= known_rel * ab64 * 0.999999999999999)) continue;
                    }
                }
                score_exact<CD, RD>(ea, eb, pr, acc);
            }
            // a lane's own maximum raises its thresholds at once
            if ((acc.max_abs > known_abs) | (acc.max_rel > known_rel)) {
                known_abs = fmax(known_abs, acc.max_abs);
                known_rel = fmax(known_rel, acc.max_rel);
                refresh();
            }
        }
    }
    if (CD == RD) acc.bitdiff += xor_acc ? 1u : 0u;
    for (unsigned long long i = begin + nvec * 8 + threadIdx.x; i < end; i += nthr) {
        const typename Elem<CD>::raw ea = Elem<CD>::load1(pr.cand, i);
        const typename Elem<RD>::raw eb = Elem<RD>::load1(pr.ref, i);
        if (CD == RD) acc.bitdiff += ea != eb;
        score_exact<CD, RD>(ea, eb, pr, acc);
    }
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

// Descriptors travel as kernel arguments (copied at launch), so the host array can be released as soon
// as the call returns and no host-to-device copy has to be ordered against the stream.

// Stages a batch of pairs and seeds their maxima, in one launch.  The cheap screen of the main
// kernel passes an element only when it cannot raise a running maximum, so a wave that starts from
// zero sends its first elements through the exact path one record at a time.  Here kSeedParts
// workgroups per pair evaluate one element per lane exactly (16384 elements per pair, in 256 evenly spread runs of 64)
// and each stores its own maxima: the seeds are errors of real elements (the final fold counts
// them too, so an element that merely ties a seed need not be recorded again; on quantised data
// such ties are the common case, and seeds scaled down to strict lower bounds measured 7% slower).
// A sample of that size leaves about one element in 16384 above the seeds.  The first workgroup
// of a pair also writes the descriptor and the block prefix, and all of them clear the pair's
// partial-result slots.  Nothing here is an atomic on global memory or needs an earlier clear.
constexpr int kSeedParts = pf::kScoreSeedParts, kSeedBlock = 1024;
template <int CD, int RD>
__device__ __forceinline__ void seed_sample(const pf::PairDev& pr, unsigned long long k, Acc& acc) {
    // one sample per 64 elements, at most 16384 per pair: small pairs are not worth more
    const unsigned long long most = (unsigned long long)kSeedParts * kSeedBlock;
    const unsigned long long want = pr.n / 64 < most ? pr.n / 64 : most;
    if (k >= want) return;
    // runs of 64 consecutive elements, one run per wave, the runs evenly spread: a wave's load touches
    // one or two cache lines of each buffer instead of 64 (a batch of 48 pairs sampled element by
    // element took 20 us, mostly address translation)
    const unsigned long long runs = (want + 63) / 64;
    const unsigned long long i = (k / 64) * (pr.n / runs) + k % 64;
    if (i < pr.n) score_exact<CD, RD>(Elem<CD>::load1(pr.cand, i), Elem<RD>::load1(pr.ref, i), pr, acc);
}

__global__ void __launch_bounds__(kSeedBlock) score_stage_kernel(pf::PairBatch batch, pf::PairDev* pairs, unsigned long long* block_start,
                                                                 pf_score_result* slots, double* seeds) {
    const int local = blockIdx.x / kSeedParts, part = blockIdx.x % kSeedParts;
    if (local >= batch.count) return;
    const int p = batch.first + local;
    const pf::PairDev pr = batch.pairs[local];
    if (part == 0 && threadIdx.x == 0) {
        pairs[p] = pr;
        block_start[p] = batch.start[local];
        if (batch.last && local == batch.count - 1) block_start[p + 1] = batch.start[batch.count];
    }
    for (int k = part * kSeedBlock + threadIdx.x; k < kSlots; k += kSeedParts * kSeedBlock) {     // every slot, whatever the two constants
        pf_score_result z;
        z.max_abs = 0.0; z.max_rel = 0.0; z.n = 0; z.n_viol = 0;
        z.nan_cand = z.nan_ref = z.inf_cand = z.inf_ref = 0;
        z.allclose = 0; z.bit_identical = 0; z.reserved_ = 0;
        slots[(size_t)p * kSlots + k] = z;
    }
    Acc acc;
    const unsigned long long k = (unsigned long long)part * kSeedBlock + threadIdx.x;
    switch (pr.cand_dtype * 4 + pr.ref_dtype) {
        case PF_F32 * 4 + PF_F32: seed_sample<PF_F32, PF_F32>(pr, k, acc); break;
        case PF_F32 * 4 + PF_BF16: seed_sample<PF_F32, PF_BF16>(pr, k, acc); break;
        case PF_F32 * 4 + PF_F16: seed_sample<PF_F32, PF_F16>(pr, k, acc); break;
        case PF_BF16 * 4 + PF_F32: seed_sample<PF_BF16, PF_F32>(pr, k, acc); break;
        case PF_BF16 * 4 + PF_BF16: seed_sample<PF_BF16, PF_BF16>(pr, k, acc); break;
        case PF_F16 * 4 + PF_F32: seed_sample<PF_F16, PF_F32>(pr, k, acc); break;
        case PF_F16 * 4 + PF_F16: seed_sample<PF_F16, PF_F16>(pr, k, acc); break;
        default: break;          // fp64 references are not screened: no seed needed
    }
    // every lane has a value here, so waves reduce by shuffles (LDS atomics of 64 lanes on one address
    // would be served one lane at a time) and one lane folds the 16 wave results
    __shared__ double s_abs[kSeedBlock / 64], s_rel[kSeedBlock / 64];
    const double wa = wave_max(acc.max_abs), wr = wave_max(acc.max_rel);
    if ((threadIdx.x & 63) == 0) { s_abs[threadIdx.x >> 6] = wa; s_rel[threadIdx.x >> 6] = wr; }
    __syncthreads();
    if (threadIdx.x < 2) {
        const double* w = threadIdx.x == 0 ? s_abs : s_rel;
        double m = w[0];
#pragma unroll
        for (int k = 1; k < kSeedBlock / 64; ++k) m = fmax(m, w[k]);
        seeds[((size_t)p * kSeedParts + part) * 2 + threadIdx.x] = m;
    }
}

// The seed of a pair: the largest of its kSeedParts partial maxima (uniform loads, a few dozen instructions per wave).
__device__ __forceinline__ void load_seed(const double* __restrict__ seeds, int p, double& abs_, double& rel_) {
    abs_ = 0.0; rel_ = 0.0;
#pragma unroll
    for (int k = 0; k < kSeedParts; ++k) {
        abs_ = fmax(abs_, seeds[((size_t)p * kSeedParts + k) * 2]);
        rel_ = fmax(rel_, seeds[((size_t)p * kSeedParts + k) * 2 + 1]);
    }
}

// Block reduction; true on the one thread that holds the block's totals afterwards.  On the screened path
// a lane has something to report only if it went through the exact path, so few lanes do: they fold
// their values into LDS with atomics (one round trip) instead of every wave walking a chain of ~100
// dependent cross-lane shuffles, which used to make up a third of a wave's lifetime.  Waves in which many
// lanes report reduce by shuffles first.
template <int CD, int RD>
__device__ __forceinline__ bool block_fold(Acc& acc, double& ma, double& mr, unsigned long long* t /* [6] */) {
    if (RD == PF_F64) acc.max_rel = fmax(acc.max_rel, __ddiv_rn(acc.keep_d, acc.keep_b));   // only score_one defers a division
    __shared__ unsigned long long s_red[8];      // max_abs bits, max_rel bits, six counts
    const int lane = threadIdx.x & 63;
    if (threadIdx.x < 8) s_red[threadIdx.x] = 0;
    __syncthreads();
    double wa = acc.max_abs, wr = acc.max_rel;
    unsigned long long c[6] = {acc.n_viol, acc.bitdiff, acc.nan_c, acc.nan_r, acc.inf_c, acc.inf_r};
    if (CD == RD) c[1] = (__any(acc.bitdiff != 0) && lane == 0) ? 1u : 0u;      // only "any difference" matters
    const bool mine = (wa > 0.0) | (wr > 0.0) | ((c[0] | c[2] | c[3] | c[4] | c[5]) != 0);
    if (__popcll(__ballot(mine)) > 16) {
        wa = wave_max(wa); wr = wave_max(wr);
#pragma unroll
        for (int k = 0; k < 6; ++k) if (k != 1) c[k] = wave_sum(c[k]);
        if (lane != 0) { wa = 0.0; wr = 0.0; c[0] = c[2] = c[3] = c[4] = c[5] = 0; }
    }
    // errors are >= 0 and never NaN, so their bit patterns order like the values
    if (wa > 0.0) atomicMax(&s_red[0], (unsigned long long)__double_as_longlong(wa));
    if (wr > 0.0) atomicMax(&s_red[1], (unsigned long long)__double_as_longlong(wr));
#pragma unroll
    for (int k = 0; k < 6; ++k) if (c[k]) atomicAdd(&s_red[2 + k], c[k]);
    __syncthreads();
    if (threadIdx.x != 0) return false;
    ma = __longlong_as_double((long long)s_red[0]);
    mr = __longlong_as_double((long long)s_red[1]);
#pragma unroll
    for (int k = 0; k < 6; ++k) t[k] = s_red[2 + k];
    return true;
}

// One instantiation per (candidate dtype, reference dtype): the host orders the
// pairs by dtype combination, so each instantiation owns a contiguous range of
// blocks and is register-allocated for its own path only.
template <int CD, int RD>
__global__ void __launch_bounds__(kBlock) score_kernel(const pf::PairDev* __restrict__ pairs, const unsigned long long* __restrict__ block_start,
                                                       int n_pairs, pf_score_result* slots, const double* __restrict__ seeds,
                                                       unsigned long long block_offset) {
    // which pair does this block belong to: largest p with block_start[p] <= bid
    int lo = 0, hi = n_pairs;
    const unsigned long long bid = block_offset + blockIdx.x;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (block_start[mid] <= bid) lo = mid; else hi = mid;
    }
    const pf::PairDev pr = pairs[lo];
    const unsigned long long begin = (bid - block_start[lo]) * pr.chunk;
    const unsigned long long end = begin + pr.chunk < pr.n ? begin + pr.chunk : pr.n;
    Acc acc;
    pf_score_result* my_slot = slots + (size_t)lo * kSlots + (bid - block_start[lo]) % kSlots;
    if (RD == PF_F64) {
        score_chunk<CD, RD>(pr, begin, end, acc);
    } else {
        double seed_abs, seed_rel;
        load_seed(seeds, lo, seed_abs, seed_rel);
        score_chunk_fast<CD, RD>(pr, begin, end, acc, seed_abs, seed_rel);
    }
    double ma, mr;
    unsigned long long t[6];
    if (block_fold<CD, RD>(acc, ma, mr, t)) {
        // one of kSlots partial results of this pair; the final kernel folds them
        pf_score_result* r = my_slot;
        // nothing at the end of a workgroup waits for memory: no value is read back
        if (ma > 0.0) atomicMax((unsigned long long*)&r->max_abs, (unsigned long long)__double_as_longlong(ma));
        if (mr > 0.0) atomicMax((unsigned long long*)&r->max_rel, (unsigned long long)__double_as_longlong(mr));
        if (t[0]) atomicAdd((unsigned long long*)&r->n_viol, t[0]);
        if (t[1]) __atomic_store_n((unsigned long long*)&r->reserved_, 1ull, __ATOMIC_RELAXED);   // a flag: any non-zero value will do
        if (t[2]) atomicAdd((unsigned long long*)&r->nan_cand, t[2]);
        if (t[3]) atomicAdd((unsigned long long*)&r->nan_ref, t[3]);
        if (t[4]) atomicAdd((unsigned long long*)&r->inf_cand, t[4]);
        if (t[5]) atomicAdd((unsigned long long*)&r->inf_ref, t[5]);
    }
}

// Pairs of at most kSmallPair elements: one workgroup of 1024 lanes scores the whole pair and writes
// its result, in a single launch for up to kPairBatch pairs (descriptors arrive as kernel arguments).
// No slots, no seeds, no second kernel: such a pair costs one kernel (~4 us) instead of three, which
// is what a launch-bound evaluation of small subgraphs is made of.
constexpr int kSmallBlock = 1024;
constexpr unsigned long long kSmallPair = 8192;     // one vector of eight elements per lane
template <int CD, int RD>
__global__ void __launch_bounds__(kSmallBlock) score_small_kernel(pf::PairBatch batch, pf_score_result* res) {
    if ((int)blockIdx.x >= batch.count) return;
    const pf::PairDev pr = batch.pairs[blockIdx.x];
    Acc acc;
    // at most eight elements per lane: evaluating each one exactly is cheaper than screening from a zero threshold
    score_chunk<CD, RD>(pr, 0, pr.n, acc);
    acc.max_rel = fmax(acc.max_rel, __ddiv_rn(acc.keep_d, acc.keep_b));      // the division score_one defers
    double ma, mr;
    unsigned long long t[6];
    if (block_fold<CD, RD>(acc, ma, mr, t)) {
        pf_score_result r;
        r.n = pr.n;
        r.max_abs = ma; r.max_rel = mr; r.n_viol = t[0]; r.reserved_ = t[1];
        r.nan_cand = t[2]; r.nan_ref = t[3]; r.inf_cand = t[4]; r.inf_ref = t[5];
        r.allclose = t[0] == 0 ? 1u : 0u;
        r.bit_identical = (CD == RD && t[1] == 0) ? 1u : 0u;
        res[pr.orig] = r;
    }
}

// The same walk for a call of few mid-size pairs (at most kPairBatch pairs of at most kSlots chunks):
// descriptors and block prefix are kernel arguments, there are no seeds (a lane's thresholds start from
// zero and rise with its own records) and each workgroup stores its totals in a slot of its own.
template <int CD, int RD>
__global__ void __launch_bounds__(kBlock) score_direct_kernel(pf::PairBatch batch, pf_score_result* slots, unsigned long long block_offset) {
    const unsigned long long bid = block_offset + blockIdx.x;
    int lo = 0, hi = batch.count;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (batch.start[mid] <= bid) lo = mid; else hi = mid;
    }
    const pf::PairDev pr = batch.pairs[lo];
    const unsigned long long begin = (bid - batch.start[lo]) * pr.chunk;
    const unsigned long long end = begin + pr.chunk < pr.n ? begin + pr.chunk : pr.n;
    Acc acc;
    double seed_abs = 0.0, seed_rel = 0.0;
    if (RD == PF_F64) {
        score_chunk<CD, RD>(pr, begin, end, acc);
    } else {
        // the workgroup seeds itself: every lane evaluates one element of the chunk exactly (a run of 256
        // consecutive elements in its middle), the largest errors become everybody's starting thresholds
        __shared__ double s_seed[2][kBlock / 64];
        Acc sample;
        const unsigned long long i = begin + (end - begin) / 2 + threadIdx.x;
        if (i < end) score_exact<CD, RD>(Elem<CD>::load1(pr.cand, i), Elem<RD>::load1(pr.ref, i), pr, sample);
        const double wa = wave_max(sample.max_abs), wr = wave_max(sample.max_rel);
        if ((threadIdx.x & 63) == 0) { s_seed[0][threadIdx.x >> 6] = wa; s_seed[1][threadIdx.x >> 6] = wr; }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kBlock / 64; ++w) { seed_abs = fmax(seed_abs, s_seed[0][w]); seed_rel = fmax(seed_rel, s_seed[1][w]); }
        score_chunk_fast<CD, RD>(pr, begin, end, acc, seed_abs, seed_rel);
    }
    double ma, mr;
    unsigned long long t[6];
    if (block_fold<CD, RD>(acc, ma, mr, t)) {
        // the seeds are errors of elements of this chunk (the walk lets elements that tie them pass unrecorded)
        ma = fmax(ma, seed_abs);
        mr = fmax(mr, seed_rel);
        pf_score_result r;
        r.n = end - begin;
        r.max_abs = ma; r.max_rel = mr; r.n_viol = t[0]; r.reserved_ = t[1];
        r.nan_cand = t[2]; r.nan_ref = t[3]; r.inf_cand = t[4]; r.inf_ref = t[5];
        r.allclose = 0; r.bit_identical = 0;
        slots[(size_t)lo * kSlots + (bid - batch.start[lo])] = r;
    }
}

// One wave per pair: lane k folds the slot of chunk k, if the pair has that many chunks.
__global__ void __launch_bounds__(64) score_direct_final_kernel(pf::PairBatch batch, pf_score_result* res, const pf_score_result* slots) {
    const int p = blockIdx.x;
    if (p >= batch.count) return;
    const unsigned long long nb = batch.start[p + 1] - batch.start[p];
    pf_score_result s;
    s.max_abs = 0.0; s.max_rel = 0.0; s.n = 0; s.n_viol = 0; s.nan_cand = s.nan_ref = s.inf_cand = s.inf_ref = 0; s.reserved_ = 0;
    if (threadIdx.x < nb) s = slots[(size_t)p * kSlots + threadIdx.x];
    const double ma = wave_max(s.max_abs), mr = wave_max(s.max_rel);
    const unsigned long long nv = wave_sum(s.n_viol), bd = wave_sum(s.reserved_);
    const unsigned long long nc = wave_sum(s.nan_cand), nr = wave_sum(s.nan_ref);
    const unsigned long long ic = wave_sum(s.inf_cand), ir = wave_sum(s.inf_ref);
    if (threadIdx.x == 0) {
        const pf::PairDev pr = batch.pairs[p];
        pf_score_result r;
        r.n = pr.n;
        r.max_abs = ma; r.max_rel = mr; r.n_viol = nv; r.reserved_ = bd;
        r.nan_cand = nc; r.nan_ref = nr; r.inf_cand = ic; r.inf_ref = ir;
        r.allclose = nv == 0 ? 1u : 0u;
        r.bit_identical = (pr.cand_dtype == pr.ref_dtype && bd == 0) ? 1u : 0u;
        res[pr.orig] = r;
    }
}

// One wave per pair: lane k folds slot k (kSlots == 64), then a wave reduction.
__global__ void __launch_bounds__(64) score_final_kernel(const pf::PairDev* pairs, int n_pairs, pf_score_result* res,
                                                         const pf_score_result* slots, const double* seeds) {
    const int p = blockIdx.x;
    if (p >= n_pairs) return;
    const pf_score_result s = slots[(size_t)p * kSlots + threadIdx.x];
    // the sampled seeds are errors of real elements too (the screen lets elements that tie them pass unrecorded)
    double seed_abs, seed_rel;
    load_seed(seeds, p, seed_abs, seed_rel);
    const double ma = fmax(wave_max(s.max_abs), seed_abs), mr = fmax(wave_max(s.max_rel), seed_rel);
    const unsigned long long nv = wave_sum(s.n_viol), bd = wave_sum(s.reserved_);
    const unsigned long long nc = wave_sum(s.nan_cand), nr = wave_sum(s.nan_ref);
    const unsigned long long ic = wave_sum(s.inf_cand), ir = wave_sum(s.inf_ref);
    if (threadIdx.x == 0) {
        pf_score_result r;
        r.n = pairs[p].n;
        r.max_abs = ma; r.max_rel = mr; r.n_viol = nv; r.reserved_ = bd;
        r.nan_cand = nc; r.nan_ref = nr; r.inf_cand = ic; r.inf_ref = ir;
        r.allclose = nv == 0 ? 1u : 0u;
        r.bit_identical = (pairs[p].cand_dtype == pairs[p].ref_dtype && bd == 0) ? 1u : 0u;
        res[pairs[p].orig] = r;                       // pairs were ordered by dtype combination for the launch
    }
}

// ---- tolerance ladder: violations at all 11 levels in one pass ----------------
// An element passes level k when a == b or |a-b| is finite and <= atol_k + rtol_k |b|
// (fp64, same arithmetic as the single-level scorer).  Both tolerances grow with
// k, so the levels an element fails form a prefix; each level is nevertheless
// tested on its own, which keeps the kernel free of any assumption on rounding.
template <int CD, int RD>
__device__ __forceinline__ void ladder_one(typename Elem<CD>::raw ra, typename Elem<RD>::raw rb, int equal_nan, const double* rt,
                                           const double* at, unsigned int* cnt);

// One workgroup per pair of the batch: writes the descriptor and the block prefix (kernel arguments) and
// clears the pair's slots, in a single launch.
__global__ void __launch_bounds__(kBlock) ladder_stage_kernel(pf::PairBatch batch, pf::PairDev* pairs, unsigned long long* block_start,
                                                              pf_ladder_result* slots) {
    const int local = blockIdx.x;
    if (local >= batch.count) return;
    const int p = batch.first + local;
    if (threadIdx.x == 0) {
        pairs[p] = batch.pairs[local];
        block_start[p] = batch.start[local];
        if (batch.last && local == batch.count - 1) block_start[p + 1] = batch.start[batch.count];
    }
    for (int k = threadIdx.x; k < kSlots; k += kBlock) {
        pf_ladder_result z;
        z.n = 0;
#pragma unroll
        for (int l = 0; l < PF_LADDER_LEVELS; ++l) z.n_viol[l] = 0;
        slots[(size_t)p * kSlots + k] = z;
    }
}

// Pairs of at most kSmallPair elements: one workgroup of 1024 lanes counts the whole pair exactly and writes
// its result; a single launch for up to kPairBatch pairs (see score_small_kernel).
template <int CD, int RD>
__global__ void __launch_bounds__(1024) ladder_small_kernel(pf::PairBatch batch, pf::LadderRow row, pf_ladder_result* res) {
    if ((int)blockIdx.x >= batch.count) return;
    const pf::PairDev pr = batch.pairs[blockIdx.x];
    unsigned int cnt[PF_LADDER_LEVELS];
#pragma unroll
    for (int k = 0; k < PF_LADDER_LEVELS; ++k) cnt[k] = 0;
    for (unsigned long long i = threadIdx.x; i < pr.n; i += blockDim.x)
        ladder_one<CD, RD>(Elem<CD>::load1(pr.cand, i), Elem<RD>::load1(pr.ref, i), pr.equal_nan, row.rtol, row.atol, cnt);
    __shared__ unsigned long long s_cnt[1024 / 64][PF_LADDER_LEVELS];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < PF_LADDER_LEVELS; ++k) {
        const unsigned long long w = wave_sum((unsigned long long)cnt[k]);
        if (lane == 0) s_cnt[wave][k] = w;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        pf_ladder_result r;
        r.n = pr.n;
#pragma unroll
        for (int k = 0; k < PF_LADDER_LEVELS; ++k) {
            unsigned long long t = 0;
            for (int w = 0; w < 1024 / 64; ++w) t += s_cnt[w][k];
            r.n_viol[k] = t;
        }
        res[pr.orig] = r;
    }
}

template <int CD, int RD>
__device__ __forceinline__ void ladder_one(typename Elem<CD>::raw ra, typename Elem<RD>::raw rb, int equal_nan, const double* rt,
                                           const double* at, unsigned int* cnt) {
    const double a = Elem<CD>::widen(ra), b = Elem<RD>::widen(rb);
    const bool na = a != a, nb = b != b;
    if (na | nb) {
        const unsigned int v = !(equal_nan && na && nb);
#pragma unroll
        for (int k = 0; k < PF_LADDER_LEVELS; ++k) cnt[k] += v;
        return;
    }
    if (a == b) return;
    const double d = fabs(__dsub_rn(a, b)), ab = fabs(b);
    const bool fin = d != __builtin_inf();
#pragma unroll
    for (int k = 0; k < PF_LADDER_LEVELS; ++k) cnt[k] += !(fin & (d <= __dadd_rn(at[k], __dmul_rn(rt[k], ab))));
}

// FAST: both tolerances grow with the level (checked on the host), so the bound atol_k + rtol_k |b|,
// rounded like the oracle rounds it, grows with k too (rounding is monotone): an element that passes
// level k passes every later one.  The levels are therefore walked in order, in fp32, against bounds
// pulled 2e-6 inwards (d <= bound: certainly passes; three vector instructions per element and level,
// the table in scalar registers), and a wave stops at the first level all of its elements pass, after
// one level for identical buffers.  An element within 4e-6 of a bound at some level (neither
// "certainly passes" nor "certainly fails"), or with a NaN or an infinity, is recounted exactly in fp64.
template <int CD, int RD, bool FAST>
__global__ void __launch_bounds__(kBlock) ladder_kernel(const pf::PairDev* pairs, const unsigned long long* block_start, int n_pairs,
                                                        pf::LadderTable table, pf_ladder_result* slots, unsigned long long block_offset) {
    int lo = 0, hi = n_pairs;
    const unsigned long long bid = block_offset + blockIdx.x;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (block_start[mid] <= bid) lo = mid; else hi = mid;
    }
    const pf::PairDev pr = pairs[lo];
    const unsigned long long begin = (bid - block_start[lo]) * pr.chunk;
    const unsigned long long end = begin + pr.chunk < pr.n ? begin + pr.chunk : pr.n;
    const double* rt = table.rtol[CD];
    const double* at = table.atol[CD];
    unsigned int cnt[PF_LADDER_LEVELS];
#pragma unroll
    for (int k = 0; k < PF_LADDER_LEVELS; ++k) cnt[k] = 0;
    const unsigned long long nvec = (end - begin) / 8;
    if (FAST && RD != PF_F64) {
        constexpr int L = PF_LADDER_LEVELS;
        float rlo[L], alo[L];
#pragma unroll
        for (int k = 0; k < L; ++k) {
            rlo[k] = (float)(rt[k] * (1.0 - 2e-6));
            alo[k] = (float)(at[k] * (1.0 - 2e-6));
        }
        // the next vector is on its way while the current one is walked
        Vec8<CD> na;
        Vec8<RD> nb;
        if (threadIdx.x < nvec) {
            na.load(pr.cand, begin + (unsigned long long)threadIdx.x * 8);
            nb.load(pr.ref, begin + (unsigned long long)threadIdx.x * 8);
        }
        for (unsigned long long it = 0; it * kBlock < nvec; ++it) {
            const unsigned long long v = it * kBlock + threadIdx.x;
            const bool live = v < nvec;
            const Vec8<CD> va = na;
            const Vec8<RD> vb = nb;
            if (v + kBlock < nvec) {
                na.load(pr.cand, begin + (v + kBlock) * 8);
                nb.load(pr.ref, begin + (v + kBlock) * 8);
            }
            // four elements at a time: their differences, references and scaled differences stay in registers
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float d[4], ab[4], u[4];
                bool redo[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float a = va.f32(half * 4 + j), b = vb.f32(half * 4 + j);
                    d[j] = fabsf(a - b);
                    ab[j] = fabsf(b);
                    // NaN, infinite difference or infinite reference: exact path only (and nothing counted here)
                    redo[j] = live & !((d[j] < __builtin_inff()) & (ab[j] < __builtin_inff()));
                    if (redo[j] | !live) { d[j] = 0.0f; ab[j] = 0.0f; }
                    u[j] = d[j] * (1.0f - 4.1e-6f);    // d > bound >= u: the outward bound (2e-6 the other way) may still hold d
                }
                int levels = 0;                         // levels walked by this wave
#pragma unroll
                for (int k = 0; k < L; ++k) {
                    bool any_fail = false;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float bound = __builtin_fmaf(rlo[k], ab[j], alo[k]);
                        const bool fail = d[j] > bound;
                        cnt[k] += fail;
                        redo[j] |= fail & (u[j] <= bound);
                        any_fail |= fail;
                    }
                    levels = k + 1;
                    if (!__any(any_fail)) break;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (!__any(redo[j])) continue;
                    if (redo[j]) {
                        // take back what the walk counted for this element, count it exactly
#pragma unroll
                        for (int k = 0; k < L; ++k)
                            if (k < levels) cnt[k] -= d[j] > __builtin_fmaf(rlo[k], ab[j], alo[k]);
                        ladder_one<CD, RD>(va.raw(half * 4 + j), vb.raw(half * 4 + j), pr.equal_nan, rt, at, cnt);
                    }
                }
            }
        }
    } else {
        for (unsigned long long v = threadIdx.x; v < nvec; v += kBlock) {
            typename Elem<CD>::raw ra[8];
            typename Elem<RD>::raw rb[8];
            Elem<CD>::load8(pr.cand, begin + v * 8, ra);
            Elem<RD>::load8(pr.ref, begin + v * 8, rb);
#pragma unroll
            for (int j = 0; j < 8; ++j) ladder_one<CD, RD>(ra[j], rb[j], pr.equal_nan, rt, at, cnt);
        }
    }
    for (unsigned long long i = begin + nvec * 8 + threadIdx.x; i < end; i += kBlock)
        ladder_one<CD, RD>(Elem<CD>::load1(pr.cand, i), Elem<RD>::load1(pr.ref, i), pr.equal_nan, rt, at, cnt);
    __shared__ unsigned long long s_cnt[kBlock / 64][PF_LADDER_LEVELS];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < PF_LADDER_LEVELS; ++k) {
        const unsigned long long w = wave_sum((unsigned long long)cnt[k]);
        if (lane == 0) s_cnt[wave][k] = w;
    }
    __syncthreads();
    if (threadIdx.x < PF_LADDER_LEVELS) {
        unsigned long long t = 0;
        for (int w = 0; w < kBlock / 64; ++w) t += s_cnt[w][threadIdx.x];
        pf_ladder_result* r = slots + (size_t)lo * kSlots + (bid - block_start[lo]) % kSlots;
        if (t) atomicAdd((unsigned long long*)&r->n_viol[threadIdx.x], t);
    }
}

__global__ void __launch_bounds__(64) ladder_final_kernel(const pf::PairDev* pairs, int n_pairs, pf_ladder_result* res,
                                                          const pf_ladder_result* slots) {
    const int p = blockIdx.x;
    if (p >= n_pairs) return;
    const pf_ladder_result s = slots[(size_t)p * kSlots + threadIdx.x];
    pf_ladder_result r;
    r.n = pairs[p].n;
#pragma unroll
    for (int k = 0; k < PF_LADDER_LEVELS; ++k) r.n_viol[k] = wave_sum(s.n_viol[k]);
    if (threadIdx.x == 0) res[pairs[p].orig] = r;
}

// One 16-byte vector per lane, non-temporal both ways: the fastest plain streaming
// shape measured on MI355X (more vectors per lane or cached accesses are 5-13% slower).
__global__ void __launch_bounds__(256) copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, unsigned long long n16) {
    const unsigned long long i = (unsigned long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

namespace pf {

// Elements per workgroup, from the elements of the whole call: 16384 for large calls (four times longer
// chunks measured 4-6% slower), fewer while that would leave the call with under 2048 workgroups, down to
// one vector per lane: a workgroup walks its chunk one vector at a time, and a call of a few million
// elements is bound by that latency (2 M elements: 18 us -> 15 us).
unsigned long long score_chunk_elems(unsigned long long n) {
    const unsigned long long step = (unsigned long long)kBlock * 8;
    unsigned long long c = (n / 2048 + step - 1) / step * step;
    if (c < step) c = step;
    return c < kChunk ? c : kChunk;
}

hipError_t launch_score_stage(const PairBatch& batch, PairDev* d_pairs, unsigned long long* d_block_start, pf_score_result* d_slots,
                              double* d_seeds, hipStream_t stream) {
    hipLaunchKernelGGL(score_stage_kernel, dim3(batch.count * kSeedParts), dim3(kSeedBlock), 0, stream, batch, d_pairs, d_block_start,
                       d_slots, d_seeds);
    return hipGetLastError();
}

unsigned long long score_small_pair_elems() { return kSmallPair; }

hipError_t launch_score_direct(const PairBatch& batch, const ScoreRanges& ranges, pf_score_result* d_results, pf_score_result* d_slots,
                               hipStream_t stream) {
#define PF_LAUNCH(CD, RD)                                                                                                  \
    if (ranges.count[CD][RD])                                                                                              \
        hipLaunchKernelGGL((score_direct_kernel<CD, RD>), dim3((unsigned)ranges.count[CD][RD]), dim3(kBlock), 0, stream,     \
                           batch, d_slots, ranges.first[CD][RD]);
    PF_LAUNCH(PF_F32, PF_F32)
    PF_LAUNCH(PF_F32, PF_BF16)
    PF_LAUNCH(PF_F32, PF_F64)
    PF_LAUNCH(PF_BF16, PF_F32)
    PF_LAUNCH(PF_BF16, PF_BF16)
    PF_LAUNCH(PF_BF16, PF_F64)
    PF_LAUNCH(PF_F32, PF_F16)
    PF_LAUNCH(PF_F16, PF_F32)
    PF_LAUNCH(PF_F16, PF_F16)
    PF_LAUNCH(PF_F16, PF_F64)
#undef PF_LAUNCH
    hipLaunchKernelGGL(score_direct_final_kernel, dim3(batch.count), dim3(64), 0, stream, batch, d_results, d_slots);
    return hipGetLastError();
}

hipError_t launch_score_small(const PairBatch& batch, int cd, int rd, pf_score_result* d_results, hipStream_t stream) {
#define PF_SMALL(CD, RD)                                                                                                     \
    if (cd == CD && rd == RD)                                                                                                \
        hipLaunchKernelGGL((score_small_kernel<CD, RD>), dim3(batch.count), dim3(kSmallBlock), 0, stream, batch, d_results);
    PF_SMALL(PF_F32, PF_F32)
    PF_SMALL(PF_F32, PF_BF16)
    PF_SMALL(PF_F32, PF_F64)
    PF_SMALL(PF_BF16, PF_F32)
    PF_SMALL(PF_BF16, PF_BF16)
    PF_SMALL(PF_BF16, PF_F64)
    PF_SMALL(PF_F32, PF_F16)
    PF_SMALL(PF_F16, PF_F32)
    PF_SMALL(PF_F16, PF_F16)
    PF_SMALL(PF_F16, PF_F64)
#undef PF_SMALL
    return hipGetLastError();
}

hipError_t launch_score(const PairDev* d_pairs, const unsigned long long* d_block_start, int n_pairs, const ScoreRanges& ranges,
                        pf_score_result* d_results, pf_score_result* d_slots, const double* d_seeds, hipStream_t stream) {
#define PF_LAUNCH(CD, RD)                                                                                                  \
    if (ranges.count[CD][RD])                                                                                              \
        hipLaunchKernelGGL((score_kernel<CD, RD>), dim3((unsigned)ranges.count[CD][RD]), dim3(kBlock), 0, stream,            \
                           d_pairs, d_block_start, n_pairs, d_slots, d_seeds, ranges.first[CD][RD]);
    PF_LAUNCH(PF_F32, PF_F32)
    PF_LAUNCH(PF_F32, PF_BF16)
    PF_LAUNCH(PF_F32, PF_F64)
    PF_LAUNCH(PF_BF16, PF_F32)
    PF_LAUNCH(PF_BF16, PF_BF16)
    PF_LAUNCH(PF_BF16, PF_F64)
    PF_LAUNCH(PF_F32, PF_F16)
    PF_LAUNCH(PF_F16, PF_F32)
    PF_LAUNCH(PF_F16, PF_F16)
    PF_LAUNCH(PF_F16, PF_F64)
#undef PF_LAUNCH
    hipLaunchKernelGGL(score_final_kernel, dim3(n_pairs), dim3(64), 0, stream, d_pairs, n_pairs, d_results, d_slots, d_seeds);
    return hipGetLastError();
}

hipError_t launch_ladder_stage(const PairBatch& batch, PairDev* d_pairs, unsigned long long* d_block_start, pf_ladder_result* d_slots,
                               hipStream_t stream) {
    hipLaunchKernelGGL(ladder_stage_kernel, dim3(batch.count), dim3(kBlock), 0, stream, batch, d_pairs, d_block_start, d_slots);
    return hipGetLastError();
}

hipError_t launch_ladder_small(const PairBatch& batch, int cd, int rd, const LadderTable& table, pf_ladder_result* d_results,
                               hipStream_t stream) {
    LadderRow row;
    for (int k = 0; k < PF_LADDER_LEVELS; ++k) {
        row.rtol[k] = table.rtol[cd][k];
        row.atol[k] = table.atol[cd][k];
    }
#define PF_SMALL(CD, RD)                                                                                                     \
    if (cd == CD && rd == RD)                                                                                                \
        hipLaunchKernelGGL((ladder_small_kernel<CD, RD>), dim3(batch.count), dim3(1024), 0, stream, batch, row, d_results);
    PF_SMALL(PF_F32, PF_F32)
    PF_SMALL(PF_F32, PF_BF16)
    PF_SMALL(PF_F32, PF_F64)
    PF_SMALL(PF_BF16, PF_F32)
    PF_SMALL(PF_BF16, PF_BF16)
    PF_SMALL(PF_BF16, PF_F64)
    PF_SMALL(PF_F32, PF_F16)
    PF_SMALL(PF_F16, PF_F32)
    PF_SMALL(PF_F16, PF_F16)
    PF_SMALL(PF_F16, PF_F64)
#undef PF_SMALL
    return hipGetLastError();
}

hipError_t launch_ladder(const PairDev* d_pairs, const unsigned long long* d_block_start, int n_pairs, const ScoreRanges& ranges,
                         const LadderTable& table, pf_ladder_result* d_results, pf_ladder_result* d_slots, hipStream_t stream) {
    // the screened kernel needs tolerances that grow with the level and that fp32 represents comfortably
    bool fast[4];
    for (int dt = 0; dt < 4; ++dt) {
        fast[dt] = true;
        for (int k = 0; k < PF_LADDER_LEVELS; ++k) {
            if (!(table.rtol[dt][k] >= 1e-30 && table.atol[dt][k] >= 1e-30 && table.rtol[dt][k] <= 1e30 && table.atol[dt][k] <= 1e30)) fast[dt] = false;
            if (k > 0 && !(table.rtol[dt][k] >= table.rtol[dt][k - 1] && table.atol[dt][k] >= table.atol[dt][k - 1])) fast[dt] = false;
        }
    }
#define PF_LAUNCH(CD, RD)                                                                                                    \
    if (ranges.count[CD][RD]) {                                                                                              \
        if (fast[CD])                                                                                                        \
            hipLaunchKernelGGL((ladder_kernel<CD, RD, true>), dim3((unsigned)ranges.count[CD][RD]), dim3(kBlock), 0, stream,   \
                               d_pairs, d_block_start, n_pairs, table, d_slots, ranges.first[CD][RD]);                       \
        else                                                                                                                 \
            hipLaunchKernelGGL((ladder_kernel<CD, RD, false>), dim3((unsigned)ranges.count[CD][RD]), dim3(kBlock), 0, stream,  \
                               d_pairs, d_block_start, n_pairs, table, d_slots, ranges.first[CD][RD]);                       \
    }
    PF_LAUNCH(PF_F32, PF_F32)
    PF_LAUNCH(PF_F32, PF_BF16)
    PF_LAUNCH(PF_F32, PF_F64)
    PF_LAUNCH(PF_BF16, PF_F32)
    PF_LAUNCH(PF_BF16, PF_BF16)
    PF_LAUNCH(PF_BF16, PF_F64)
    PF_LAUNCH(PF_F32, PF_F16)
    PF_LAUNCH(PF_F16, PF_F32)
    PF_LAUNCH(PF_F16, PF_F16)
    PF_LAUNCH(PF_F16, PF_F64)
#undef PF_LAUNCH
    hipLaunchKernelGGL(ladder_final_kernel, dim3(n_pairs), dim3(64), 0, stream, d_pairs, n_pairs, d_results, d_slots);
    return hipGetLastError();
}

// ---- scratch that lives in the code object ----
// Callers that cannot allocate device memory (code under graph capture, tight serving loops, harnesses
// that forbid hipMalloc) score through pf_score_static, whose workspace is this array.  Every GPU
// holds its own copy at its own address, so the address is looked up once per device, with that
// device current, and only that pointer ever reaches a kernel or a runtime call: the array's name in
// host code is a stand-in, not a device address.
}  // namespace pf

static __device__ __align__(256) unsigned char scratch[PF_STATIC_SCRATCH_BYTES];

namespace pf {

hipError_t static_scratch(void** d_ptr, size_t* bytes) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* per_device[kMaxDevices];          // zero-initialised: not looked up yet
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(mu);
    if (!per_device[dev]) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *d_ptr = per_device[dev];
    *bytes = PF_STATIC_SCRATCH_BYTES;
    return hipSuccess;
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
    const unsigned long long n16 = bytes / 16;
    const unsigned long long blocks = (n16 + 255) / 256;
    if (blocks) hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (u32x4*)dst, (const u32x4*)src, n16);
    return hipGetLastError();
}

}  // namespace pf
