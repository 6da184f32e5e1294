// Device-side helpers prepended to every generated kernel (as source text).
//
// Everything is written for gfx950 wave64: 16-byte global accesses, bf16
// conversion through the hardware pack instruction, cross-lane reductions by
// xor shuffles inside a wave and one LDS exchange across waves.
#pragma once

namespace pf {

static const char* kDevicePrelude = R"PF(
typedef unsigned short u16;
typedef unsigned int u32;
typedef _Float16 f16;                      // IEEE binary16 tensors (bf16 tensors are addressed as u16)
typedef u32 u32x2 __attribute__((ext_vector_type(2)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// Vector types for accesses that are only element-aligned (rows whose byte length is not a
// multiple of 16): gfx950 under HSA serves unaligned global accesses, and the compiler emits
// the same wide instructions for them.
typedef u32 u32_a2 __attribute__((aligned(2)));
typedef u32x2 u32x2_a2 __attribute__((aligned(2)));
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef f32x2 f32x2_a4 __attribute__((aligned(4)));
typedef f32x4 f32x4_a4 __attribute__((aligned(4)));
template <bool UA> struct VT { typedef u32 b1; typedef u32x2 b2; typedef u32x4 b4; typedef f32x2 f2; typedef f32x4 f4; };
template <> struct VT<true> { typedef u32_a2 b1; typedef u32x2_a2 b2; typedef u32x4_a2 b4; typedef f32x2_a4 f2; typedef f32x4_a4 f4; };
#define PF_DEV __device__ __forceinline__

PF_DEV float pf_bits2f(u32 u) { return __builtin_bit_cast(float, u); }
PF_DEV u32 pf_f2bits(float f) { return __builtin_bit_cast(u32, f); }
PF_DEV u32 pf_pack_bf16(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(u32, __builtin_convertvector(v, bf16x2));   // round to nearest even
}
PF_DEV u16 pf_f2bf(float f) { return __builtin_bit_cast(u16, (__bf16)f); }

// ---- loads of N contiguous elements into fp32 registers (p aligned to the access) ----
template <int N, bool NT, bool UA> struct LdBf16;
template <bool NT, bool UA> struct LdBf16<1, NT, UA> {
    static PF_DEV void run(const u16* p, float* o) { o[0] = pf_bits2f((u32)(NT ? __builtin_nontemporal_load(p) : *p) << 16); }
};
template <bool NT, bool UA> struct LdBf16<2, NT, UA> {
    static PF_DEV void run(const u16* p, float* o) {
        typedef typename VT<UA>::b1 V; u32 r = NT ? __builtin_nontemporal_load((const V*)p) : *(const V*)p;
        o[0] = pf_bits2f(r << 16); o[1] = pf_bits2f(r & 0xffff0000u);
    }
};
template <bool NT, bool UA> struct LdBf16<4, NT, UA> {
    static PF_DEV void run(const u16* p, float* o) {
        typedef typename VT<UA>::b2 V; u32x2 r = NT ? __builtin_nontemporal_load((const V*)p) : *(const V*)p;
        o[0] = pf_bits2f(r.x << 16); o[1] = pf_bits2f(r.x & 0xffff0000u);
        o[2] = pf_bits2f(r.y << 16); o[3] = pf_bits2f(r.y & 0xffff0000u);
    }
};
template <bool NT, bool UA> struct LdBf16<8, NT, UA> {
    static PF_DEV void run(const u16* p, float* o) {
        typedef typename VT<UA>::b4 V; u32x4 r = NT ? __builtin_nontemporal_load((const V*)p) : *(const V*)p;
        o[0] = pf_bits2f(r.x << 16); o[1] = pf_bits2f(r.x & 0xffff0000u);
        o[2] = pf_bits2f(r.y << 16); o[3] = pf_bits2f(r.y & 0xffff0000u);
        o[4] = pf_bits2f(r.z << 16); o[5] = pf_bits2f(r.z & 0xffff0000u);
        o[6] = pf_bits2f(r.w << 16); o[7] = pf_bits2f(r.w & 0xffff0000u);
    }
};
template <int N, bool NT, bool UA> struct LdF32;
template <bool NT, bool UA> struct LdF32<1, NT, UA> {
    static PF_DEV void run(const float* p, float* o) { o[0] = NT ? __builtin_nontemporal_load(p) : *p; }
};
template <bool NT, bool UA> struct LdF32<2, NT, UA> {
    static PF_DEV void run(const float* p, float* o) {
        typedef typename VT<UA>::f2 V; f32x2 r = NT ? __builtin_nontemporal_load((const V*)p) : *(const V*)p;
        o[0] = r.x; o[1] = r.y;
    }
};
template <bool NT, bool UA> struct LdF32<4, NT, UA> {
    static PF_DEV void run(const float* p, float* o) {
        typedef typename VT<UA>::f4 V; f32x4 r = NT ? __builtin_nontemporal_load((const V*)p) : *(const V*)p;
        o[0] = r.x; o[1] = r.y; o[2] = r.z; o[3] = r.w;
    }
};
template <bool NT, bool UA> struct LdF32<8, NT, UA> {
    static PF_DEV void run(const float* p, float* o) {
        LdF32<4, NT, UA>::run(p, o); LdF32<4, NT, UA>::run(p + 4, o + 4);
    }
};
// fp16: the same accesses as bf16, then an exact hardware widening of each half
PF_DEV float pf_h2f(u32 bits) { return (float)__builtin_bit_cast(f16, (u16)bits); }
template <int N, bool NT, bool UA> struct LdF16;
template <bool NT, bool UA> struct LdF16<1, NT, UA> {
    static PF_DEV void run(const f16* p, float* o) { o[0] = (float)(NT ? __builtin_nontemporal_load(p) : *p); }
};
template <bool NT, bool UA> struct LdF16<2, NT, UA> {
    static PF_DEV void run(const f16* p, float* o) {
        typedef typename VT<UA>::b1 V; u32 r = NT ? __builtin_nontemporal_load((const V*)p) : *(const V*)p;
        o[0] = pf_h2f(r & 0xffffu); o[1] = pf_h2f(r >> 16);
    }
};
template <bool NT, bool UA> struct LdF16<4, NT, UA> {
    static PF_DEV void run(const f16* p, float* o) {
        typedef typename VT<UA>::b2 V; u32x2 r = NT ? __builtin_nontemporal_load((const V*)p) : *(const V*)p;
        o[0] = pf_h2f(r.x & 0xffffu); o[1] = pf_h2f(r.x >> 16); o[2] = pf_h2f(r.y & 0xffffu); o[3] = pf_h2f(r.y >> 16);
    }
};
template <bool NT, bool UA> struct LdF16<8, NT, UA> {
    static PF_DEV void run(const f16* p, float* o) {
        typedef typename VT<UA>::b4 V; u32x4 r = NT ? __builtin_nontemporal_load((const V*)p) : *(const V*)p;
        o[0] = pf_h2f(r.x & 0xffffu); o[1] = pf_h2f(r.x >> 16); o[2] = pf_h2f(r.y & 0xffffu); o[3] = pf_h2f(r.y >> 16);
        o[4] = pf_h2f(r.z & 0xffffu); o[5] = pf_h2f(r.z >> 16); o[6] = pf_h2f(r.w & 0xffffu); o[7] = pf_h2f(r.w >> 16);
    }
};
template <int N, bool NT, bool UA = false> PF_DEV void pf_ld(const f16* p, float* o) { LdF16<N, NT, UA>::run(p, o); }
PF_DEV float pf_ld1(const f16* p) { return (float)*p; }
template <int N, bool NT, bool UA = false> PF_DEV void pf_ld(const u16* p, float* o) { LdBf16<N, NT, UA>::run(p, o); }
template <int N, bool NT, bool UA = false> PF_DEV void pf_ld(const float* p, float* o) { LdF32<N, NT, UA>::run(p, o); }
PF_DEV float pf_ld1(const u16* p) { return pf_bits2f((u32)*p << 16); }
PF_DEV float pf_ld1(const float* p) { return *p; }

// ---- stores of N contiguous fp32 registers, rounded once to the stored dtype ----
template <int N, bool NT, bool UA> struct StBf16;
template <bool NT, bool UA> struct StBf16<1, NT, UA> {
    static PF_DEV void run(u16* p, const float* v) { u16 r = pf_f2bf(v[0]); if (NT) __builtin_nontemporal_store(r, p); else *p = r; }
};
template <bool NT, bool UA> struct StBf16<2, NT, UA> {
    static PF_DEV void run(u16* p, const float* v) {
        u32 r = pf_pack_bf16(v[0], v[1]);
        typedef typename VT<UA>::b1 V; if (NT) __builtin_nontemporal_store(r, (V*)p); else *(V*)p = r;
    }
};
template <bool NT, bool UA> struct StBf16<4, NT, UA> {
    static PF_DEV void run(u16* p, const float* v) {
        u32x2 r = {pf_pack_bf16(v[0], v[1]), pf_pack_bf16(v[2], v[3])};
        typedef typename VT<UA>::b2 V; if (NT) __builtin_nontemporal_store(r, (V*)p); else *(V*)p = r;
    }
};
template <bool NT, bool UA> struct StBf16<8, NT, UA> {
    static PF_DEV void run(u16* p, const float* v) {
        u32x4 r = {pf_pack_bf16(v[0], v[1]), pf_pack_bf16(v[2], v[3]), pf_pack_bf16(v[4], v[5]), pf_pack_bf16(v[6], v[7])};
        typedef typename VT<UA>::b4 V; if (NT) __builtin_nontemporal_store(r, (V*)p); else *(V*)p = r;
    }
};
template <int N, bool NT, bool UA> struct StF32;
template <bool NT, bool UA> struct StF32<1, NT, UA> {
    static PF_DEV void run(float* p, const float* v) { if (NT) __builtin_nontemporal_store(v[0], p); else *p = v[0]; }
};
template <bool NT, bool UA> struct StF32<2, NT, UA> {
    static PF_DEV void run(float* p, const float* v) {
        f32x2 r = {v[0], v[1]};
        typedef typename VT<UA>::f2 V; if (NT) __builtin_nontemporal_store(r, (V*)p); else *(V*)p = r;
    }
};
template <bool NT, bool UA> struct StF32<4, NT, UA> {
    static PF_DEV void run(float* p, const float* v) {
        f32x4 r = {v[0], v[1], v[2], v[3]};
        typedef typename VT<UA>::f4 V; if (NT) __builtin_nontemporal_store(r, (V*)p); else *(V*)p = r;
    }
};
template <bool NT, bool UA> struct StF32<8, NT, UA> {
    static PF_DEV void run(float* p, const float* v) { StF32<4, NT, UA>::run(p, v); StF32<4, NT, UA>::run(p + 4, v + 4); }
};
// fp16 stores: one round-to-nearest-even conversion per element (the default rounding mode), packed in pairs
PF_DEV u32 pf_pack_f16(float lo, float hi) { return (u32)__builtin_bit_cast(u16, (f16)lo) | ((u32)__builtin_bit_cast(u16, (f16)hi) << 16); }
template <int N, bool NT, bool UA> struct StF16;
template <bool NT, bool UA> struct StF16<1, NT, UA> {
    static PF_DEV void run(f16* p, const float* v) { f16 r = (f16)v[0]; if (NT) __builtin_nontemporal_store(r, p); else *p = r; }
};
template <bool NT, bool UA> struct StF16<2, NT, UA> {
    static PF_DEV void run(f16* p, const float* v) {
        u32 r = pf_pack_f16(v[0], v[1]);
        typedef typename VT<UA>::b1 V; if (NT) __builtin_nontemporal_store(r, (V*)p); else *(V*)p = r;
    }
};
template <bool NT, bool UA> struct StF16<4, NT, UA> {
    static PF_DEV void run(f16* p, const float* v) {
        u32x2 r = {pf_pack_f16(v[0], v[1]), pf_pack_f16(v[2], v[3])};
        typedef typename VT<UA>::b2 V; if (NT) __builtin_nontemporal_store(r, (V*)p); else *(V*)p = r;
    }
};
template <bool NT, bool UA> struct StF16<8, NT, UA> {
    static PF_DEV void run(f16* p, const float* v) {
        u32x4 r = {pf_pack_f16(v[0], v[1]), pf_pack_f16(v[2], v[3]), pf_pack_f16(v[4], v[5]), pf_pack_f16(v[6], v[7])};
        typedef typename VT<UA>::b4 V; if (NT) __builtin_nontemporal_store(r, (V*)p); else *(V*)p = r;
    }
};
template <int N, bool NT, bool UA = false> PF_DEV void pf_st(f16* p, const float* v) { StF16<N, NT, UA>::run(p, v); }
PF_DEV void pf_st1(f16* p, float v) { *p = (f16)v; }
template <int N, bool NT, bool UA = false> PF_DEV void pf_st(u16* p, const float* v) { StBf16<N, NT, UA>::run(p, v); }
template <int N, bool NT, bool UA = false> PF_DEV void pf_st(float* p, const float* v) { StF32<N, NT, UA>::run(p, v); }
PF_DEV void pf_st1(u16* p, float v) { *p = pf_f2bf(v); }
PF_DEV void pf_st1(float* p, float v) { *p = v; }

// ---- scalar math ----
PF_DEV float pf_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
#if PF_PRECISE
// fp32 graphs: every operator stays within about two ulp of the exact result, built from the hardware's
// one-ulp estimates (v_rcp_f32, v_exp_f32) instead of the correctly rounded library routines, which cost
// two to three times the instructions and would make these kernels bound by the vector ALU.
//
// a / b = a * (1/b): one ulp from the reciprocal, half an ulp from the product.  The reciprocal estimate
// flushes subnormal results and inputs, so divisors outside [2^-126, 2^126) take the correctly rounded
// division, as do quotients that come out non-finite (the division defines what 0/0, x/0, inf/inf are).
// (One test per element: collecting the tests of a lane's elements into a single branch per operator measured
// 2-5 us slower on the subgraphs with several divisions.)
PF_DEV float pf_div(float a, float b) {
    const float q = a * pf_rcp(b);
    const bool plain = (((pf_f2bits(b) & 0x7f800000u) - 0x00800000u) < 0x7e000000u) & (__builtin_fabsf(q) < __builtin_inff());
    if (__builtin_expect(!plain, 0)) return a / b;
    return q;
}
// e^x = 2^(x log2 e): the product x log2 e is carried as two floats (its rounding error alone would cost
// |x| * 1e-7 of relative accuracy) and the low part enters as a first-order correction.
PF_DEV float pf_exp(float x) {
    const float L = 1.4426950216293335f, Llo = 1.9259629911e-8f;      // log2 e = L + Llo
    const float y = x * L;
    const float ylo = __builtin_fmaf(x, Llo, __builtin_fmaf(x, L, -y));
    const float p = __builtin_amdgcn_exp2f(y);
    const float r = __builtin_fmaf(p, ylo * 0.6931471806f, p);
    return (r == r) ? r : p;       // x infinite or the result out of range: the correction is inf - inf, p is the answer
}
// tanh: an odd polynomial where 1 - 2 / (1 + e^2x) would cancel (|x| < 0.625, 0.8 ulp), the exponential form beyond
PF_DEV float pf_tanh(float x) {
    const float ax = __builtin_fabsf(x), u = x * x;
    float q = __builtin_fmaf(u, -0.005691985599696636f, 0.020626291632652283f);
    q = __builtin_fmaf(q, u, -0.05373531952500343f);
    q = __builtin_fmaf(q, u, 0.13331381976604462f);
    q = __builtin_fmaf(q, u, -0.3333328068256378f);
    const float small = __builtin_fmaf(x * u, q, x);
    const float t = __builtin_amdgcn_exp2f(ax * -2.8853900817779268f);      // e^(-2|x|) <= 0.29: its rounding hardly shows
    const float big = __builtin_copysignf((1.0f - t) * pf_rcp(1.0f + t), x);
    return ax < 0.625f ? small : big;                                       // NaN compares false and leaves through `big`
}
PF_DEV float pf_sigmoid(float x) { return pf_rcp(1.0f + pf_exp(-x)); }
PF_DEV float pf_gelu_tanh(float x) {
    // 0.5 x (1 + tanh u) = x / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3)
    const float u = 0.7978845608028654f * __builtin_fmaf(0.044715f * x, x * x, x);
    return x * pf_rcp(1.0f + pf_exp(-2.0f * u));
}
#else
PF_DEV float pf_div(float a, float b) { return a * pf_rcp(b); }
PF_DEV float pf_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }
PF_DEV float pf_tanh(float x) { return 1.0f - 2.0f * pf_rcp(1.0f + __builtin_amdgcn_exp2f(x * 2.8853900817779268f)); }
PF_DEV float pf_sigmoid(float x) { return pf_rcp(1.0f + __builtin_amdgcn_exp2f(x * -1.4426950408889634f)); }
PF_DEV float pf_gelu_tanh(float x) {
    // x / (1 + exp(-2u)), with -2 * log2(e) * sqrt(2/pi) folded into the polynomial
    float t = x * x;
    float p = __builtin_fmaf(t, -0.10294324f, -2.3022082f);
    return x * pf_rcp(1.0f + __builtin_amdgcn_exp2f(x * p));
}
#endif
PF_DEV float pf_rsqrt(float x) { return __builtin_amdgcn_rsqf(x); }
PF_DEV float pf_gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.7071067811865476f)); }
PF_DEV float pf_max_nan(float a, float b) {       // max that propagates NaN
    float m = fmaxf(a, b);
    return (a != a) ? a : ((b != b) ? b : m);
}

PF_DEV float pf_min_nan(float a, float b) {       // min that propagates NaN
    float m = fminf(a, b);
    return (a != a) ? a : ((b != b) ? b : m);
}

// ---- reductions across the T lanes that share a row ----
// T <= 64: the lanes are consecutive lanes of one wave.  T > 64: whole waves;
// wave results meet in LDS (one slot set per call site, so one barrier each).
template <int T> PF_DEV float pf_wave_sum(float v) {
#pragma unroll
    for (int o = (T < 64 ? T : 64) / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <int T> PF_DEV double pf_wave_sum(double v) {
#pragma unroll
    for (int o = (T < 64 ? T : 64) / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <int T> PF_DEV float pf_wave_max(float v) {
#pragma unroll
    for (int o = (T < 64 ? T : 64) / 2; o > 0; o >>= 1) v = pf_max_nan(v, __shfl_xor(v, o, 64));
    return v;
}
template <int T, typename A> PF_DEV A pf_team_sum(A v, A* lds /* [BLOCK/64] */) {
    v = pf_wave_sum<T>(v);
    if (T > 64) {
        const int wave = threadIdx.x >> 6;
        if ((threadIdx.x & 63) == 0) lds[wave] = v;
        __syncthreads();
        const int first = (wave / (T / 64)) * (T / 64);
        A s = lds[first];
#pragma unroll
        for (int w = 1; w < T / 64; ++w) s += lds[first + w];
        v = s;
    }
    return v;
}
template <int T> PF_DEV float pf_team_max(float v, float* lds) {
    v = pf_wave_max<T>(v);
    if (T > 64) {
        const int wave = threadIdx.x >> 6;
        if ((threadIdx.x & 63) == 0) lds[wave] = v;
        __syncthreads();
        const int first = (wave / (T / 64)) * (T / 64);
        float s = lds[first];
#pragma unroll
        for (int w = 1; w < T / 64; ++w) s = pf_max_nan(s, lds[first + w]);
        v = s;
    }
    return v;
}
)PF";

}  // namespace pf
