// Error-scoring kernels (ahead-of-time compiled for gfx950) and the plain copy
// kernel used as the practical bandwidth ceiling.
//
// Scoring follows the validity test of the paper's Definition 3.2 / Eq. 1 with
// the atol/rtol pairs of Appendix F.  One pass over every (candidate, reference)
// pair produces, as asked for, either or both of
//   - the single-level result: largest absolute and relative error, NaN/Inf
//     counts, the number of elements outside |a-b| <= atol + rtol*|b|, and
//     whether the two buffers are bit-identical;
//   - the tolerance ladder: that number of elements at each of the 11 tolerance
//     indices t = -10 .. 0 of the candidate's dtype.
// All decisions are those of fp64 arithmetic on exactly widened values and every
// accumulator is order-independent (max, integer sums), so the result does not
// depend on how the elements are spread over lanes.
//
// Launch structure: a staging kernel writes the pair descriptors, clears the pairs' partial-result slots and
// completion counters and samples each pair's seed (16384 elements evaluated exactly: the largest errors found
// become every lane's starting thresholds).  One kernel then walks the data; a workgroup folds its totals into one
// of the pair's 64 slots with fire-and-forget atomics, takes a ticket from the pair's counter, and the workgroup
// that draws the last ticket folds the slots into the result the caller reads (nobody waits for anybody).  Pairs of
// at most 8192 elements are scored whole by one workgroup each, in a single launch.
#include <hip/hip_runtime.h>

#include <mutex>

#include "pf.h"
#include "score_dev.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;
constexpr int L = PF_LADDER_LEVELS;
constexpr unsigned long long kStep = (unsigned long long)kBlock * 8;     // elements one pass of a workgroup covers

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

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ unsigned int wave_sum32(unsigned int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- the single-level result ----------------------------------------------------
// Per-lane accumulators.  max_abs / max_rel hold the largest errors this lane has evaluated exactly.
struct Acc {
    double max_abs = 0.0, max_rel = 0.0;
    double keep_d = 0.0, keep_b = 1.0;       // score_one: element with the largest estimated quotient (0/1: none yet)
    float keep_q = 0.0f;
    unsigned int n_viol = 0, bitdiff = 0;          // per lane: a chunk has fewer than 2^31 elements
    unsigned int nan_c = 0, nan_r = 0, inf_c = 0, inf_r = 0;
};

__device__ __forceinline__ bool est_range_ok(float x) {   // 1e-18 <= x <= 1e18, false for 0/inf/nan
    return x >= 1e-18f && x <= 1e18f;
}

// One element against an fp64 reference.  The largest relative error needs a correctly rounded fp64
// division, far too slow to run on every element: each lane tracks the running maximum of a cheap fp32
// estimate q ~ d/|b| (relative error < 1e-6) and keeps the (d, |b|) of that element; only elements whose
// estimate lies within 2e-6 of the running maximum, or whose operands leave the range where the estimate
// is trustworthy, are divided on the spot.  An element that is neither kept nor divided is smaller than
// the kept one by more than both estimates can be wrong, so the exact maximum is
// max(exact divisions, kept_d / kept_b), evaluated once per lane at the end.
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
    // A division only where the quotient can exceed the largest one m this lane has found: the fused multiply-add
    // rounds m |b| - d once, so its sign is that of the exact value; m |b| >= d means d / |b| <= m, and
    // rounding the quotient cannot lift it past m, which is representable.  Elements that tie the
    // maximum (the common case on quantised data) are settled here without dividing.
    if (ab == 0.0 || d == inf) acc.max_rel = inf;
    else if (__builtin_fma(acc.max_rel, ab, -d) < 0.0) acc.max_rel = fmax(acc.max_rel, __ddiv_rn(d, ab));
}

// ---- fp32 screening (both sides f32, bf16 or fp16) ---------------------------
// Almost every element can be classified without fp64: with a, b widened to fp32, d32 = |a - b| carries a
// relative error of 2^-24 (and is exact when it is subnormal), so comparing it against thresholds that are
// pulled 2e-6 to the safe side decides "certainly inside the tolerance", "certainly outside", "certainly
// not a new maximum of |a-b| or of |a-b|/|b|".  Elements not decided this way (or NaN/Inf) are evaluated
// exactly in fp64 by score_exact.
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
    // element j as Elem<DT>::raw
    __device__ __forceinline__ unsigned int raw(int j) const {
        if (HALF) return (j & 1) ? (w[j >> 1] >> 16) : (w[j >> 1] & 0xffffu);
        return w[j];
    }
};

// a raw element widened to fp32 (exact)
template <int DT> struct Elem32 {
    static __device__ __forceinline__ float widen(unsigned int r) {
        if (DT == PF_BF16) return __uint_as_float(r << 16);
        if (DT == PF_F16) return Elem<PF_F16>::widen32(r);
        return __uint_as_float(r);
    }
};

// ---- the tolerance ladder --------------------------------------------------------
// An element passes level k when a == b or |a-b| is finite and <= atol_k + rtol_k |b| (fp64, the
// arithmetic of the single-level test).  This is the definition, level by level.
template <int CD, int RD>
__device__ __forceinline__ void ladder_one(typename Elem<CD>::raw ra, typename Elem<RD>::raw rb, int equal_nan, const double* rt,
                                           const double* at, unsigned int* cnt) {
    const double a = Elem<CD>::widen(ra), b = Elem<RD>::widen(rb);
    const bool na = a != a, nb = b != b;
    if (na | nb) {
        const unsigned int v = !(equal_nan && na && nb);
#pragma unroll
        for (int k = 0; k < L; ++k) cnt[k] += v;
        return;
    }
    if (a == b) return;
    const double d = fabs(__dsub_rn(a, b)), ab = fabs(b);
    const bool fin = d != __builtin_inf();
#pragma unroll
    for (int k = 0; k < L; ++k) cnt[k] += !(fin & (d <= __dadd_rn(at[k], __dmul_rn(rt[k], ab))));
}

// The levels of four elements at once, in fp32.  Both tolerances grow with the level (checked on the host), so
// the bound atol_k + rtol_k |b|, rounded like the definition rounds it, grows with k too (rounding is monotone):
// the levels an element fails form a prefix.  The levels are therefore walked upwards against bounds pulled
// 2e-6 inwards (d <= bound: certainly passes) and a wave stops at the first level all of its elements pass.
// Data that differ by a rounding error of the stored dtype fail the lowest few levels all alike: after level 0
// the walk tests the pivot level kPivot, and when every lane finds there exactly the failures of level 0 the
// levels between need no test (a failure set between two equal ones equals them).  An element within 4e-6 of a
// bound at some level (neither "certainly passes" nor "certainly fails"), or with a NaN or an infinity, is
// flagged in `redo`; the caller takes back what the walk counted for it and counts it by the definition.
constexpr int kPivot = 3;
struct LadderBounds {
    float rlo[L], alo[L];
};
__device__ __forceinline__ int ladder_walk4(const float* d, const float* ab, const LadderBounds& lb, unsigned int* cnt, bool* redo) {
    float u[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        u[j] = d[j] * (1.0f - 4.1e-6f);               // d > bound >= u: the outward bound (2e-6 the other way) may still hold d
        redo[j] = !(d[j] + ab[j] < __builtin_inff());  // NaN, infinite difference or infinite reference (or a sum beyond the fp32 range)
    }
    auto level = [&](int k) -> unsigned int {
        unsigned int f = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float bound = __builtin_fmaf(lb.rlo[k], ab[j], lb.alo[k]);
            const bool fail = d[j] > bound;
            f += fail;
            redo[j] |= fail & (u[j] <= bound);
        }
        cnt[k] += f;
        return f;
    };
    const unsigned int f0 = level(0);
    if (!__any(f0 != 0)) return 0;
    unsigned int f = level(kPivot);
    if (!__any(f != f0)) {
#pragma unroll
        for (int k = 1; k < kPivot; ++k) cnt[k] += f0;
    } else {
#pragma unroll
        for (int k = 1; k < kPivot; ++k) level(k);
    }
    int kmax = kPivot;
#pragma unroll
    for (int k = kPivot + 1; k < L; ++k) {
        if (!__any(f != 0)) break;
        f = level(k);
        kmax = k;
    }
    return kmax;
}
// what the walk counted for one element, up to the last level it reached
__device__ __forceinline__ void ladder_take_back(float d, float ab, const LadderBounds& lb, int kmax, unsigned int* cnt) {
#pragma unroll
    for (int k = 0; k < L; ++k)
        if (k <= kmax) cnt[k] -= d > __builtin_fmaf(lb.rlo[k], ab, lb.alo[k]);
}

// ---- one workgroup, one chunk ------------------------------------------------------
// MODE bit 0: the single-level result, bit 1: the ladder.
constexpr int kScore = 1, kLadder = 2;

template <int CD, int RD, int MODE>
__device__ __forceinline__ void walk_exact(const pf::PairDev& pr, const pf::LadderRow& row, unsigned long long begin,
                                           unsigned long long end, Acc& acc, unsigned int* cnt) {
    // fp64 references: every element by the definition (vectors of 8, lanes interleaved so that a wave reads contiguous memory)
    const unsigned long long nvec = (end - begin) / 8;
    const unsigned int nthr = blockDim.x;
    for (unsigned long long v = threadIdx.x; v < nvec; v += nthr) {
        typename Elem<CD>::raw ra[8];
        typename Elem<RD>::raw rb[8];
        Elem<CD>::load8(pr.cand, begin + v * 8, ra);
        Elem<RD>::load8(pr.ref, begin + v * 8, rb);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (MODE & kScore) score_one<CD, RD>(ra[j], rb[j], pr, acc);
            if (MODE & kLadder) ladder_one<CD, RD>(ra[j], rb[j], pr.equal_nan, row.rtol, row.atol, cnt);
        }
    }
    for (unsigned long long i = begin + nvec * 8 + threadIdx.x; i < end; i += nthr) {
        const typename Elem<CD>::raw ea = Elem<CD>::load1(pr.cand, i);
        const typename Elem<RD>::raw eb = Elem<RD>::load1(pr.ref, i);
        if (MODE & kScore) score_one<CD, RD>(ea, eb, pr, acc);
        if (MODE & kLadder) ladder_one<CD, RD>(ea, eb, pr.equal_nan, row.rtol, row.atol, cnt);
    }
}

template <int CD, int RD, int MODE>
__device__ __forceinline__ void walk_screened(const pf::PairDev& pr, const pf::LadderRow& row, bool ladder_fast, unsigned long long wg,
                                              Acc& acc, unsigned int* cnt, double seed_abs, double seed_rel) {
    const Screen sc = make_screen(pr);
    const int zero_tol = (pr.rtol == 0.0) & (pr.atol == 0.0);
    const int force_exact = !sc.viol_decidable;
    // the lean screen needs an absolute tolerance fp32 can represent comfortably (then every allowed
    // error bound is >= 1e-30 and needs no guard of its own)
    const bool lean = !force_exact && sc.atol_lo >= 1e-30f;
    LadderBounds lb;
    if (MODE & kLadder) {
#pragma unroll
        for (int k = 0; k < L; ++k) {
            lb.rlo[k] = (float)(row.rtol[k] * (1.0 - 2e-6));
            lb.alo[k] = (float)(row.atol[k] * (1.0 - 2e-6));
        }
    }
    unsigned int xor_acc = 0;
    // This workgroup's share of the pair: chunks wg, wg + wgs, wg + 2 wgs, ... of pr.chunk elements each, every chunk
    // walked in passes of one vector (eight elements) per lane.  At any moment the workgroups of a pair read
    // neighbouring chunks; over its life a workgroup sees several chunks, so the errors its lanes have met keep
    // screening for them.  (c, p): chunk and pass of the vector in hand.
    const unsigned long long whole = pr.n / 8 * 8;                             // elements in whole vectors of the pair
    const unsigned long long n_chunks = (pr.n + pr.chunk - 1) / pr.chunk;
    const unsigned int ppc = (unsigned int)(pr.chunk / kStep);                 // passes per chunk
    const unsigned long long my_chunks = wg < n_chunks ? (n_chunks - wg + pr.wgs - 1) / pr.wgs : 0;
    const unsigned long long iters = my_chunks * ppc;
    // off: first element of the vector in hand (additions only: this runs once per eight elements)
    unsigned long long off = wg * pr.chunk + (unsigned long long)threadIdx.x * 8;
    const unsigned long long jump = (pr.wgs - 1) * pr.chunk + kStep;           // from the last pass of a chunk to the next chunk of this workgroup
    unsigned int p = 0;
    auto advance = [&]() {
        if (++p == ppc) { p = 0; off += jump; }
        else off += kStep;
    };
    // the next vector is already on its way while the current one is screened; lanes past the end hold zeros,
    // which pass every test and count nothing
    Vec8<CD> na;
    Vec8<RD> nb;
#pragma unroll
    for (int k = 0; k < Vec8<CD>::NW; ++k) na.w[k] = 0;
#pragma unroll
    for (int k = 0; k < Vec8<RD>::NW; ++k) nb.w[k] = 0;
    if (iters && off < whole) {
        na.load(pr.cand, off);
        nb.load(pr.ref, off);
    }
    // Screening thresholds, per lane: fp32 lower bounds of the largest errors known.  They start from the pair's
    // seed (errors of sampled elements, exact) and follow the errors this lane evaluates exactly or meets in fp32.
    double known_abs = seed_abs, known_rel = seed_rel;
    float thr_abs = 0.0f, thr_rel = 0.0f;
    struct { float d = 0.0f, q = 0.0f; unsigned int da = 0, db = 0, qa = 0, qb = 0; } keep;   // largest |a-b| and quotient seen in fp32, and whose they are
    auto refresh = [&]() {
        // roundings far inside the 2e-6 pulled off below; the kept candidates are fp32 values of real elements, good to 1e-6
        const float ka = fmaxf((float)known_abs, keep.d * (1.0f - 4e-6f));
        const float kr = fmaxf((float)known_rel, keep.q * (1.0f - 4e-6f));
        thr_abs = ka >= 1e-30f ? ka * 0.999998f : 0.0f;
        thr_rel = kr >= 1e-30f ? kr * 0.999998f : 0.0f;
    };
    refresh();
    for (unsigned long long it = 0; it < iters; ++it) {
        const bool live = off < whole;
        const Vec8<CD> va = na;
        const Vec8<RD> vb = nb;
        advance();
        if (it + 1 < iters && off < whole) {
            na.load(pr.cand, off);
            nb.load(pr.ref, off);
        } else {
#pragma unroll
            for (int k = 0; k < Vec8<CD>::NW; ++k) na.w[k] = 0;
#pragma unroll
            for (int k = 0; k < Vec8<RD>::NW; ++k) nb.w[k] = 0;
        }
        if (MODE & kScore) {
            if (CD == RD) {
#pragma unroll
                for (int k = 0; k < Vec8<CD>::NW; ++k) xor_acc |= va.w[k] ^ vb.w[k];
            }
            unsigned int fmask = 0;          // bit j: element j needs a closer look
            unsigned int nv = 0;
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
                // full classification: certainly inside the tolerance, certainly outside (counted here), or
                // flagged (undecided, NaN/Inf, possible new maximum).  Branch-free on purpose (bitwise | and &).
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float a = va.f32(j), b = vb.f32(j);
                    const float d = fabsf(a - b), ab = fabsf(b);
                    const float lo = __builtin_fmaf(sc.rtol_lo, ab, sc.atol_lo);
                    const float hi = __builtin_fmaf(sc.rtol_hi, ab, sc.atol_hi);
                    // thresholds below 1e-30 are too close to the fp32 subnormal range to be trusted
                    const int ok = (d == 0.0f) | ((d <= lo) & (lo >= 1e-30f));
                    const int out = (d > hi) & ((hi >= 1e-30f) | zero_tol);
                    const float pr_rel = thr_rel * ab;
                    const int f = (!(ok | out)) | (!(d < __builtin_inff())) | (d > thr_abs) | (d > pr_rel) | ((pr_rel < 1e-30f) & (d != 0.0f)) |
                                  (force_exact & live);
                    nv += out & !f;
                    fmask |= (unsigned)f << j;
                }
            }
            acc.n_viol += nv;                // violations the full classification decided on its own
            if (__any(fmask != 0)) {
                // the flagged elements only; the trip count is the largest number of flagged elements in any lane of the wave
                bool kept = false;
                while (fmask) {
                    const int j = __builtin_ctz(fmask);
                    fmask &= fmask - 1;
                    unsigned int ea = va.raw(0), eb = vb.raw(0);
#pragma unroll
                    for (int t = 1; t < 8; ++t) { ea = j == t ? va.raw(t) : ea; eb = j == t ? vb.raw(t) : eb; }
                    if (lean) {
                        const float a = Elem32<CD>::widen(ea), b = Elem32<RD>::widen(eb);
                        const float d = fabsf(a - b), ab = fabsf(b);
                        const float hi = __builtin_fmaf(sc.rtol_hi, ab, sc.atol_hi), pr_rel = thr_rel * ab;
                        const bool fin = (d < __builtin_inff()) & (ab < __builtin_inff());
                        // certainly outside the tolerance and certainly no new maximum: counted without fp64
                        if ((d > hi) & fin & (d <= thr_abs) & (d <= pr_rel) & (pr_rel >= 1e-30f)) {
                            acc.n_viol += 1;
                            continue;
                        }
                        // Certainly inside the tolerance and finite: the element only matters as a possible new maximum.
                        if ((d <= __builtin_fmaf(sc.rtol_lo, ab, sc.atol_lo)) & fin) {
                            // exactly no new maximum?  The errors of this lane's own exact evaluations are the yardstick (fp64,
                            // no division: see score_exact); the many elements of quantised data that tie a maximum end here.
                            const double d64 = fabs(__dsub_rn((double)a, (double)b)), ab64 = fabs((double)b);
                            if ((d64 <= known_abs) & (__builtin_fma(known_rel, ab64, -d64) >= 0.0)) continue;
                            // Otherwise the candidates for both maxima are tracked in fp32, like score_one does: an element
                            // certainly larger than the kept one replaces it, one certainly smaller is dropped, and only one
                            // within 2e-6 of it is evaluated exactly.  The kept elements are evaluated once, at the end.
                            bool amb = false;
                            if (d > keep.d * 1.000002f) { keep.d = d; keep.da = ea; keep.db = eb; }
                            else amb |= d >= keep.d * 0.999998f;
                            if ((int)est_range_ok(d) & (int)est_range_ok(ab)) {
                                const float q = d * __builtin_amdgcn_rcpf(ab);
                                if (q > keep.q * 1.000002f) { keep.q = q; keep.qa = ea; keep.qb = eb; }
                                else amb |= q >= keep.q * 0.999998f;
                            } else amb = true;
                            if (!amb) { kept = true; continue; }
                        }
                    }
                    score_exact<CD, RD>(ea, eb, pr, acc);
                }
                // a lane's own maximum raises its thresholds at once
                if (kept | (acc.max_abs > known_abs) | (acc.max_rel > known_rel)) {
                    known_abs = fmax(known_abs, acc.max_abs);
                    known_rel = fmax(known_rel, acc.max_rel);
                    refresh();
                }
            }
        }
        if (MODE & kLadder) {
            if (ladder_fast) {
                // four elements at a time: their differences, references and scaled differences stay in registers
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    float d[4], ab[4];
                    bool redo[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float a = va.f32(half * 4 + j), b = vb.f32(half * 4 + j);
                        d[j] = fabsf(a - b);
                        ab[j] = fabsf(b);
                    }
                    const int kmax = ladder_walk4(d, ab, lb, cnt, redo);
                    if (__any(redo[0] | redo[1] | redo[2] | redo[3])) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (redo[j]) {
                                ladder_take_back(d[j], ab[j], lb, kmax, cnt);
                                ladder_one<CD, RD>(va.raw(half * 4 + j), vb.raw(half * 4 + j), pr.equal_nan, row.rtol, row.atol, cnt);
                            }
                        }
                    }
                }
            } else if (live) {
#pragma unroll
                for (int j = 0; j < 8; ++j) ladder_one<CD, RD>(va.raw(j), vb.raw(j), pr.equal_nan, row.rtol, row.atol, cnt);
            }
        }
    }
    if (MODE & kScore) {
        // the kept candidates, exactly (they lie inside the tolerance and are finite: only the maxima are concerned)
        if (keep.d > 0.0f) {
            const double a = Elem<CD>::widen(keep.da), b = Elem<RD>::widen(keep.db);
            acc.max_abs = fmax(acc.max_abs, fabs(__dsub_rn(a, b)));
        }
        if (keep.q > 0.0f) {
            const double a = Elem<CD>::widen(keep.qa), b = Elem<RD>::widen(keep.qb);
            acc.max_rel = fmax(acc.max_rel, __ddiv_rn(fabs(__dsub_rn(a, b)), fabs(b)));
        }
        if (CD == RD) acc.bitdiff += xor_acc ? 1u : 0u;
    }
    // the elements after the last whole vector of the pair, by its first workgroup
    for (unsigned long long i = whole + threadIdx.x; wg == 0 && i < pr.n; i += kBlock) {
        const typename Elem<CD>::raw ea = Elem<CD>::load1(pr.cand, i);
        const typename Elem<RD>::raw eb = Elem<RD>::load1(pr.ref, i);
        if (MODE & kScore) {
            if (CD == RD) acc.bitdiff += ea != eb;
            score_exact<CD, RD>(ea, eb, pr, acc);
        }
        if (MODE & kLadder) ladder_one<CD, RD>(ea, eb, pr.equal_nan, row.rtol, row.atol, cnt);
    }
}

// Block reduction of the single-level accumulators; true on the one thread that holds the block's totals
// afterwards.  On the screened path a lane has something to report only if it evaluated elements exactly, so few
// lanes do: they fold their values into LDS with atomics (one round trip) instead of every wave walking a chain
// of ~100 dependent cross-lane shuffles.  Waves in which many lanes report reduce by shuffles first.
template <int CD, int RD>
__device__ __forceinline__ bool block_fold(Acc& acc, double& ma, double& mr, unsigned long long* t /* [6] */) {
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

// Block totals of the ladder counts: level k's total ends up on thread k (k < 11).
template <int NW>
__device__ __forceinline__ void ladder_block_totals(const unsigned int* cnt, unsigned long long (*s_cnt)[L], unsigned long long* tot) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < L; ++k) {
        const unsigned int w = wave_sum32(cnt[k]);
        if (lane == 0) s_cnt[wave][k] = w;
    }
    __syncthreads();
    if (threadIdx.x < L) {
        unsigned long long t = 0;
        for (int w = 0; w < NW; ++w) t += s_cnt[w][threadIdx.x];
        *tot = t;
    }
}

// Descriptors in device memory are the same for every lane: each word is moved to a scalar register, so that a
// descriptor costs no vector registers for the life of the workgroup.
__device__ __forceinline__ unsigned long long uniform_u64(const unsigned long long* p) {
    const unsigned long long v = *p;
    const unsigned int lo = __builtin_amdgcn_readfirstlane((unsigned int)v), hi = __builtin_amdgcn_readfirstlane((unsigned int)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ double uniform_f64(const double* p) { return __longlong_as_double((long long)uniform_u64((const unsigned long long*)p)); }
__device__ __forceinline__ pf::PairDev uniform_pair(const pf::PairDev* p) {
    static_assert(sizeof(pf::PairDev) % 4 == 0, "descriptor is a whole number of words");
    constexpr int NWORDS = (int)(sizeof(pf::PairDev) / 4);
    unsigned int w[NWORDS];
    const unsigned int* src = (const unsigned int*)p;
#pragma unroll
    for (int k = 0; k < NWORDS; ++k) w[k] = __builtin_amdgcn_readfirstlane(src[k]);
    pf::PairDev d;
    __builtin_memcpy(&d, w, sizeof d);
    return d;
}

// Stages a batch of pairs, in one launch: kSeedParts workgroups per pair.  The first of them writes the descriptor
// and the workgroup prefix and clears the pair's ticket; all of them clear the pair's slots and evaluate one
// element per lane exactly (16384 elements per pair, in 256 evenly spread runs of 64, so that a wave's load touches
// one or two cache lines), each storing its own two maxima: the seeds are errors of real elements (the final fold
// counts them too, so an element that merely ties a seed need not be recorded again; on quantised data such
// ties are the common case).  Nothing here is an atomic on global memory or needs an earlier clear.
constexpr int kSeedParts = pf::kScoreSeedParts, kSeedBlock = 1024, kSlots = pf::kScoreSlots;
static_assert(kSlots == 64, "the last workgroup folds the slots with one wave, one slot per lane");
template <int CD, int RD>
__device__ __forceinline__ void seed_sample(const pf::PairDev& pr, unsigned long long k, Acc& acc) {
    // one sample per 64 elements, at most 16384 per pair: small pairs are not worth more
    const unsigned long long most = (unsigned long long)kSeedParts * kSeedBlock;
    const unsigned long long want = pr.n / 64 < most ? pr.n / 64 : most;
    if (k >= want) return;
    const unsigned long long runs = (want + 63) / 64;
    const unsigned long long i = (k / 64) * (pr.n / runs) + k % 64;
    if (i < pr.n) score_exact<CD, RD>(Elem<CD>::load1(pr.cand, i), Elem<RD>::load1(pr.ref, i), pr, acc);
}

__global__ void __launch_bounds__(kSeedBlock) stage_kernel(pf::PairBatch batch, pf::ScoreSpace sp) {
    const int local = blockIdx.x / kSeedParts, part = blockIdx.x % kSeedParts;
    if (local >= batch.count) return;
    const int p = batch.first + local;
    const pf::PairDev pr = batch.pairs[local];
    if (part == 0 && threadIdx.x == 0) {
        sp.pairs[p] = pr;
        sp.start[p] = batch.start[local];
        if (batch.last && local == batch.count - 1) sp.start[p + 1] = batch.start[batch.count];
    }
    const int k0 = part * kSeedBlock + threadIdx.x;
    if (k0 < kSlots + 1) sp.tickets[(size_t)p * (kSlots + 1) + k0] = 0;
    // which pair each workgroup of the walking kernel belongs to (one load there instead of a search over the prefix)
    for (unsigned long long w = (unsigned long long)k0; w < pr.wgs; w += (unsigned long long)kSeedParts * kSeedBlock)
        sp.wg_pair[batch.start[local] + w] = p;
    if (sp.sslots)
        for (int k = k0; k < kSlots; k += kSeedParts * kSeedBlock) {
            pf_score_result z;
            z.max_abs = 0.0; z.max_rel = 0.0; z.n = 0; z.n_viol = 0;
            z.nan_cand = z.nan_ref = z.inf_cand = z.inf_ref = 0;
            z.allclose = 0; z.bit_identical = 0; z.reserved_ = 0;
            sp.sslots[(size_t)p * kSlots + k] = z;
        }
    if (sp.lslots)
        for (int k = k0; k < kSlots; k += kSeedParts * kSeedBlock) {
            pf_ladder_result z;
            z.n = 0;
#pragma unroll
            for (int l = 0; l < L; ++l) z.n_viol[l] = 0;
            sp.lslots[(size_t)p * kSlots + k] = z;
        }
    if (!sp.sslots) return;             // seeds serve the single-level result only
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
    // every lane has a value here, so waves reduce by shuffles and one lane folds the 16 wave results
    __shared__ double s_abs[kSeedBlock / 64], s_rel[kSeedBlock / 64];
    const double wa = wave_max(acc.max_abs), wr = wave_max(acc.max_rel);
    if ((threadIdx.x & 63) == 0) { s_abs[threadIdx.x >> 6] = wa; s_rel[threadIdx.x >> 6] = wr; }
    __syncthreads();
    if (threadIdx.x < 2) {
        const double* w = threadIdx.x == 0 ? s_abs : s_rel;
        double m = w[0];
#pragma unroll
        for (int q = 1; q < kSeedBlock / 64; ++q) m = fmax(m, w[q]);
        sp.seeds[((size_t)p * kSeedParts + part) * 2 + threadIdx.x] = m;
    }
}

// One instantiation per (candidate dtype, reference dtype, results wanted): the host orders the pairs by dtype
// combination, so each instantiation owns a contiguous range of workgroups and is register-allocated for its
// own path only.  A workgroup walks its chunks, folds its totals into a slot of its pair and takes a ticket; the
// last one of the pair to do so folds the slots.
template <int CD, int RD, int MODE>
__global__ void __launch_bounds__(kBlock) pair_kernel(pf::ScoreSpace sp, pf::LadderRow row, int ladder_fast, pf_score_result* sres,
                                                      pf_ladder_result* lres, unsigned long long block_offset) {
    const unsigned long long bid = block_offset + blockIdx.x;
    const int lo = __builtin_amdgcn_readfirstlane(sp.wg_pair[bid]);       // written by the staging launch
    const pf::PairDev pr = uniform_pair(sp.pairs + lo);
    const unsigned long long wg = bid - uniform_u64(sp.start + lo);          // this workgroup among the pr.wgs of its pair
    Acc acc;
    unsigned int cnt[L];
#pragma unroll
    for (int k = 0; k < L; ++k) cnt[k] = 0;
    double seed_abs = 0.0, seed_rel = 0.0;
    if (RD == PF_F64) {
        for (unsigned long long begin = wg * pr.chunk; begin < pr.n; begin += pr.wgs * pr.chunk)
            walk_exact<CD, RD, MODE>(pr, row, begin, begin + pr.chunk < pr.n ? begin + pr.chunk : pr.n, acc, cnt);
        if (MODE & kScore) acc.max_rel = fmax(acc.max_rel, __ddiv_rn(acc.keep_d, acc.keep_b));      // the division score_one defers
    } else {
        if (MODE & kScore) {
            // the seed of the pair: the largest of its kSeedParts partial maxima (uniform loads, a few dozen instructions per wave)
#pragma unroll
            for (int k = 0; k < kSeedParts; ++k) {
                seed_abs = fmax(seed_abs, uniform_f64(sp.seeds + ((size_t)lo * kSeedParts + k) * 2));
                seed_rel = fmax(seed_rel, uniform_f64(sp.seeds + ((size_t)lo * kSeedParts + k) * 2 + 1));
            }
        }
        walk_screened<CD, RD, MODE>(pr, row, ladder_fast != 0, wg, acc, cnt, seed_abs, seed_rel);
    }
    const size_t slot = (size_t)lo * kSlots + (size_t)(wg % kSlots);
    if (MODE & kScore) {
        double ma, mr;
        unsigned long long t[6];
        if (block_fold<CD, RD>(acc, ma, mr, t)) {
            // nothing here waits for memory: no value is read back
            pf_score_result* r = sp.sslots + slot;
            if (ma > 0.0) atomicMax((unsigned long long*)&r->max_abs, (unsigned long long)__double_as_longlong(ma));
            if (mr > 0.0) atomicMax((unsigned long long*)&r->max_rel, (unsigned long long)__double_as_longlong(mr));
            if (t[0]) atomicAdd((unsigned long long*)&r->n_viol, t[0]);
            if (t[1]) atomicAdd((unsigned long long*)&r->reserved_, 1ull);
            if (t[2]) atomicAdd((unsigned long long*)&r->nan_cand, t[2]);
            if (t[3]) atomicAdd((unsigned long long*)&r->nan_ref, t[3]);
            if (t[4]) atomicAdd((unsigned long long*)&r->inf_cand, t[4]);
            if (t[5]) atomicAdd((unsigned long long*)&r->inf_ref, t[5]);
        }
    }
    if (MODE & kLadder) {
        __shared__ unsigned long long s_cnt[kBlock / 64][L];
        unsigned long long tot = 0;
        ladder_block_totals<kBlock / 64>(cnt, s_cnt, &tot);
        if (threadIdx.x < L && tot) atomicAdd((unsigned long long*)&sp.lslots[slot].n_viol[threadIdx.x], tot);
    }
    // The ticket.  Slots and tickets are only ever touched by device-scope atomics, which are carried out at
    // the level of the memory system that all workgroups share; the wave that issued this workgroup's slot updates
    // (wave 0 issued all of them) waits until every one has been acknowledged before it draws the ticket, and
    // the workgroup that draws the pair's last ticket reads the slots with device-scope atomic loads afterwards.
    // (A device-scope release / acquire pair would say the same, but on this chip each one writes back and
    // invalidates a whole L2: with 3072 workgroups that quadrupled the kernel's duration.)
    __shared__ unsigned int s_last;
    if (threadIdx.x < 64) {
        __builtin_amdgcn_s_waitcnt(0);            // vmcnt(0) expcnt(0) lgkmcnt(0): every access of this wave has completed
        if (threadIdx.x == 0) {
            // Two levels, so that thousands of workgroups finishing together do not queue up on one address:
            // a ticket of the slot first (about wgs / 64 workgroups share one), and whoever completes a slot
            // draws one of the pair's 64 (or wgs, if fewer) tickets.
            const unsigned int s = (unsigned int)(wg % kSlots);
            const unsigned int users = (unsigned int)(pr.wgs / kSlots) + (s < (unsigned int)(pr.wgs % kSlots) ? 1u : 0u);
            const unsigned int used = pr.wgs < (unsigned long long)kSlots ? (unsigned int)pr.wgs : (unsigned int)kSlots;
            unsigned int last = 0;
            if (__hip_atomic_fetch_add(sp.tickets + (size_t)lo * (kSlots + 1) + 1 + s, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == users)
                last = __hip_atomic_fetch_add(sp.tickets + (size_t)lo * (kSlots + 1), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == used;
            s_last = last;
        }
    }
    __syncthreads();
    if (!s_last || threadIdx.x >= 64) return;
    const int k = threadIdx.x;                     // one wave: lane k folds slot k (kSlots == 64)
    if (MODE & kScore) {
        const unsigned long long* q = (const unsigned long long*)(sp.sslots + (size_t)lo * kSlots + k);
        auto ld = [&](int word) { return __hip_atomic_load(q + word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
        static_assert(sizeof(pf_score_result) == 80, "slot layout");
        // words: 0 max_abs, 1 max_rel, 2 n, 3 n_viol, 4 nan_cand, 5 nan_ref, 6 inf_cand, 7 inf_ref, 8 flags, 9 reserved_
        const double ma = fmax(wave_max(__longlong_as_double((long long)ld(0))), seed_abs);
        const double mr = fmax(wave_max(__longlong_as_double((long long)ld(1))), seed_rel);
        const unsigned long long nv = wave_sum(ld(3)), nc = wave_sum(ld(4)), nr = wave_sum(ld(5)), ic = wave_sum(ld(6)), ir = wave_sum(ld(7));
        const unsigned long long bd = wave_sum(ld(9));
        if (k == 0) {
            pf_score_result r;
            r.n = pr.n;
            r.max_abs = ma; r.max_rel = mr; r.n_viol = nv; r.reserved_ = bd;
            r.nan_cand = nc; r.nan_ref = nr; r.inf_cand = ic; r.inf_ref = ir;
            r.allclose = nv == 0 ? 1u : 0u;
            r.bit_identical = (CD == RD && bd == 0) ? 1u : 0u;
            sres[pr.orig] = r;                    // pairs were ordered by dtype combination for the launch
        }
    }
    if (MODE & kLadder) {
        const unsigned long long* q = (const unsigned long long*)(sp.lslots + (size_t)lo * kSlots + k);
        pf_ladder_result r;
        r.n = pr.n;
#pragma unroll
        for (int l = 0; l < L; ++l) r.n_viol[l] = wave_sum(__hip_atomic_load(q + 1 + l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        if (k == 0) lres[pr.orig] = r;
    }
}

// Pairs of at most kSmallPair elements: one workgroup of 1024 lanes scores the whole pair by the definition
// (at most eight elements per lane: cheaper than screening from a zero threshold) and writes its results, in a
// single launch for up to kPairBatch pairs (descriptors arrive as kernel arguments).  Such a pair costs one
// kernel, which is what a launch-bound evaluation of small subgraphs is made of.
constexpr int kSmallBlock = 1024;
constexpr unsigned long long kSmallPair = 8192;     // one vector of eight elements per lane
template <int CD, int RD, int MODE>
__global__ void __launch_bounds__(kSmallBlock) small_kernel(pf::PairBatch batch, pf::LadderRow row, pf_score_result* sres, pf_ladder_result* lres) {
    if ((int)blockIdx.x >= batch.count) return;
    const pf::PairDev pr = batch.pairs[blockIdx.x];
    Acc acc;
    unsigned int cnt[L];
#pragma unroll
    for (int k = 0; k < L; ++k) cnt[k] = 0;
    walk_exact<CD, RD, MODE>(pr, row, 0, pr.n, acc, cnt);
    if (MODE & kScore) {
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
            sres[pr.orig] = r;
        }
    }
    if (MODE & kLadder) {
        __shared__ unsigned long long s_cnt[kSmallBlock / 64][L];
        unsigned long long tot = 0;
        ladder_block_totals<kSmallBlock / 64>(cnt, s_cnt, &tot);
        if (threadIdx.x < L) lres[pr.orig].n_viol[threadIdx.x] = tot;
        if (threadIdx.x == 0) lres[pr.orig].n = pr.n;
    }
}

// One 16-byte vector per lane, non-temporal both ways: the fastest plain streaming
// shape measured on MI355X (more vectors per lane or cached accesses are 5-13% slower).
__global__ void __launch_bounds__(256) copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, unsigned long long n16) {
    const unsigned long long i = (unsigned long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

template <int MODE>
void launch_pairs_mode(const pf::ScoreSpace& sp, const pf::ScoreRanges& ranges, const pf::LadderTable& table, const bool* fast,
                       pf_score_result* sres, pf_ladder_result* lres, hipStream_t stream) {
#define PF_LAUNCH(CD, RD)                                                                                                      \
    if (ranges.count[CD][RD]) {                                                                                                \
        pf::LadderRow row;                                                                                                     \
        for (int k = 0; k < L; ++k) { row.rtol[k] = table.rtol[CD][k]; row.atol[k] = table.atol[CD][k]; }                      \
        hipLaunchKernelGGL((pair_kernel<CD, RD, MODE>), dim3((unsigned)ranges.count[CD][RD]), dim3(kBlock), 0, stream, sp,      \
                           row, (int)fast[CD], sres, lres, ranges.first[CD][RD]);                                              \
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
}

template <int MODE>
void launch_small_mode(const pf::PairBatch& batch, int cd, int rd, const pf::LadderRow& row, pf_score_result* sres, pf_ladder_result* lres,
                       hipStream_t stream) {
#define PF_SMALL(CD, RD)                                                                                                        \
    if (cd == CD && rd == RD)                                                                                                   \
        hipLaunchKernelGGL((small_kernel<CD, RD, MODE>), dim3(batch.count), dim3(kSmallBlock), 0, stream, batch, row, sres, lres);
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
}

}  // namespace

namespace pf {

// Elements per chunk and workgroups per call.  A call is walked by at most about score_target_wgs() workgroups
// (and at least one per pair); beyond that a workgroup walks several chunks, round robin.  Measured on one pair
// of 90 M bf16 elements: the single-level kernel (5 workgroups resident per compute unit) is fastest with one
// round of resident workgroups, 1280, and chunks of 8192 or 4096 elements; the ladder kernels, with fewer resident
// waves and more arithmetic per element, with 3072 workgroups and chunks of 16384.  A call of many pairs of
// different sizes and dtypes needs more, shorter-lived workgroups to even out (780 pairs, 5 GB: 1800 us with
// 1280 workgroups, 1275 us with 10240, no better beyond), so the target grows with the number of pairs.
// Smaller calls get smaller chunks, so that they still spread over the chip, down to one vector per lane (a call
// of a few million elements is bound by the latency of walking a chunk one vector at a time).
unsigned long long score_target_wgs(bool ladder, int n_pairs) {
    const unsigned long long k = n_pairs < 1 ? 1 : (unsigned long long)n_pairs;
    const unsigned long long t = ladder ? 3072 * (k < 4 ? k : 4) : 1280 * (k < 8 ? k : 8);
    return t < kScoreMaxTargetWGs ? t : kScoreMaxTargetWGs;
}
unsigned long long score_chunk_elems(unsigned long long n, bool ladder) {
    unsigned long long c = (n / 2048 + kStep - 1) / kStep * kStep;
    if (c < kStep) c = kStep;
    const unsigned long long most = (ladder ? 8 : 4) * (unsigned long long)kStep;
    return c > most ? most : c;
}

unsigned long long score_small_pair_elems() { return kSmallPair; }

hipError_t launch_stage(const PairBatch& batch, const ScoreSpace& sp, hipStream_t stream) {
    hipLaunchKernelGGL(stage_kernel, dim3(batch.count * kSeedParts), dim3(kSeedBlock), 0, stream, batch, sp);
    return hipGetLastError();
}

// the screened ladder walk needs tolerances that grow with the level and that fp32 represents comfortably
static void ladder_fast_flags(const LadderTable& table, bool* fast) {
    for (int dt = 0; dt < 4; ++dt) {
        fast[dt] = true;
        for (int k = 0; k < L; ++k) {
            if (!(table.rtol[dt][k] >= 1e-30 && table.atol[dt][k] >= 1e-30 && table.rtol[dt][k] <= 1e30 && table.atol[dt][k] <= 1e30)) fast[dt] = false;
            if (k > 0 && !(table.rtol[dt][k] >= table.rtol[dt][k - 1] && table.atol[dt][k] >= table.atol[dt][k - 1])) fast[dt] = false;
        }
    }
}

hipError_t launch_pairs(const ScoreSpace& sp, const ScoreRanges& ranges, const LadderTable& table, pf_score_result* d_sres,
                        pf_ladder_result* d_lres, hipStream_t stream) {
    bool fast[4];
    ladder_fast_flags(table, fast);
    if (d_sres && d_lres) launch_pairs_mode<kScore | kLadder>(sp, ranges, table, fast, d_sres, d_lres, stream);
    else if (d_sres) launch_pairs_mode<kScore>(sp, ranges, table, fast, d_sres, d_lres, stream);
    else launch_pairs_mode<kLadder>(sp, ranges, table, fast, d_sres, d_lres, stream);
    return hipGetLastError();
}

hipError_t launch_small(const PairBatch& batch, int cd, int rd, const LadderTable& table, pf_score_result* d_sres, pf_ladder_result* d_lres,
                        hipStream_t stream) {
    LadderRow row;
    for (int k = 0; k < L; ++k) {
        row.rtol[k] = table.rtol[cd][k];
        row.atol[k] = table.atol[cd][k];
    }
    if (d_sres && d_lres) launch_small_mode<kScore | kLadder>(batch, cd, rd, row, d_sres, d_lres, stream);
    else if (d_sres) launch_small_mode<kScore>(batch, cd, rd, row, d_sres, d_lres, stream);
    else launch_small_mode<kLadder>(batch, cd, rd, row, d_sres, d_lres, stream);
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
