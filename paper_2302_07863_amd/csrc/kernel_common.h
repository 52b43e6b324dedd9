// Device helpers shared by the kernel translation units of the BiLD library (gfx950, wave64): bf16 conversion,
// wavefront reductions on the DPP path, online softmax statistics, activation functions.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>

#include <type_traits>

#include "bild_internal.h"

namespace bild {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t f2bf(float f) {  // fp32 -> bf16 bits, nearest even
    uint32_t u = __float_as_uint(f);
    return (u + (((u >> 16) & 1u) + 0x7FFFu)) >> 16;
}
__device__ __forceinline__ float bf2f(uint32_t h) { return __uint_as_float(h << 16); }

// Two fp32 values as (high, low) bf16 pairs, a in the low half-words: high = bf16(v) to nearest even,
// low = bf16(v - high), by the packed conversion instruction of gfx950.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    const f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t& hi, uint32_t& lo) {
    const f32x2 v = {a, b};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    const f32x2 r = v - __builtin_convertvector(h, f32x2);
    hi = __builtin_bit_cast(uint32_t, h);
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2));
}

// Wavefront reductions on the data-parallel-primitive path (no LDS crossbar):
// two quad permutes, two row mirrors, then row broadcasts carry the row totals
// upward so that lane 63 holds the result, which is read back as a uniform value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float fill, float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, fill), __builtin_bit_cast(int, v),
                                                                  CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f<0xB1, 0xF>(0.f, v);   // quad_perm [1,0,3,2]
    v += dpp_f<0x4E, 0xF>(0.f, v);   // quad_perm [2,3,0,1]
    v += dpp_f<0x141, 0xF>(0.f, v);  // row_half_mirror
    v += dpp_f<0x140, 0xF>(0.f, v);  // row_mirror: every lane of a 16-lane row holds the row total
    v += dpp_f<0x142, 0xA>(0.f, v);  // row_bcast15 into rows 1 and 3
    v += dpp_f<0x143, 0xC>(0.f, v);  // row_bcast31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f<0xB1, 0xF>(-INFINITY, v));
    v = fmaxf(v, dpp_f<0x4E, 0xF>(-INFINITY, v));
    v = fmaxf(v, dpp_f<0x141, 0xF>(-INFINITY, v));
    v = fmaxf(v, dpp_f<0x140, 0xF>(-INFINITY, v));
    v = fmaxf(v, dpp_f<0x142, 0xA>(-INFINITY, v));
    v = fmaxf(v, dpp_f<0x143, 0xC>(-INFINITY, v));
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// The values of the lanes l and l ^ 16 (or l ^ 32) side by side in every lane, through gfx950's lane-swap instructions
// instead of a trip through the LDS crossbar: swapping a register with a copy of itself leaves the even 16-lane rows'
// values (the lower half's) in the first result and the odd rows' (the upper half's) in the second, in all lanes.
__device__ __forceinline__ void pair_xor16(uint32_t x, uint32_t& even, uint32_t& odd) {
    const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    even = r[0];
    odd = r[1];
}
__device__ __forceinline__ void pair_xor32(uint32_t x, uint32_t& lower, uint32_t& upper) {
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    lower = r[0];
    upper = r[1];
}
// max / sum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (every lane gets the result; the sums are formed in one fixed order)
__device__ __forceinline__ float quad_rows_max(float v) {
    uint32_t a, b;
    pair_xor16(__float_as_uint(v), a, b);
    v = fmaxf(__uint_as_float(a), __uint_as_float(b));
    pair_xor32(__float_as_uint(v), a, b);
    return fmaxf(__uint_as_float(a), __uint_as_float(b));
}
__device__ __forceinline__ float quad_rows_sum(float v) {
    uint32_t a, b;
    pair_xor16(__float_as_uint(v), a, b);
    v = __uint_as_float(a) + __uint_as_float(b);
    pair_xor32(__float_as_uint(v), a, b);
    return __uint_as_float(a) + __uint_as_float(b);
}

// exp through the hardware's base-2 exponential (one multiply and one transcendental instruction instead of the library
// routine's range reduction).  Used where the argument is a difference of logits or scores, at most zero: relative error of
// a few 1e-7 for the arguments near zero that carry the softmax mass, below 1e-5 relative where the result is negligible
// anyway, exp(-inf) = 0.  These exponentials sit on the critical path of every latency-bound stage that has them.
__device__ __forceinline__ float fexp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }

// ---- online softmax statistics ------------------------------------------------------
struct Stat {
    float m, s;
    int idx;
};
__device__ __forceinline__ Stat stat_neutral() { return Stat{-INFINITY, 0.f, 0x7FFFFFFF}; }
__device__ __forceinline__ void stat_push(Stat& a, float z, int n) {
    if (z > a.m) {  // strict: equal maxima keep the lower id (ids arrive in increasing order)
        a.s = a.s * fexp(a.m - z) + 1.f;
        a.m = z;
        a.idx = n;
    } else {
        a.s += fexp(z - a.m);
    }
}
__device__ __forceinline__ Stat stat_merge(const Stat& a, const Stat& b) {
    Stat r;
    r.m = fmaxf(a.m, b.m);
    const float sa = (a.m == -INFINITY) ? 0.f : a.s * fexp(a.m - r.m);
    const float sb = (b.m == -INFINITY) ? 0.f : b.s * fexp(b.m - r.m);
    r.s = sa + sb;
    r.idx = (a.m > b.m || (a.m == b.m && a.idx < b.idx)) ? a.idx : b.idx;
    return r;
}
// merge of the statistics of the lanes l, l ^ 16, l ^ 32, l ^ 48 (every lane gets the result)
__device__ __forceinline__ Stat stat_quad_rows(const Stat& v) {
    Stat x, y;
    uint32_t a, b;
    pair_xor16(__float_as_uint(v.m), a, b); x.m = __uint_as_float(a); y.m = __uint_as_float(b);
    pair_xor16(__float_as_uint(v.s), a, b); x.s = __uint_as_float(a); y.s = __uint_as_float(b);
    pair_xor16((uint32_t)v.idx, a, b); x.idx = (int)a; y.idx = (int)b;
    const Stat h = stat_merge(x, y);
    pair_xor32(__float_as_uint(h.m), a, b); x.m = __uint_as_float(a); y.m = __uint_as_float(b);
    pair_xor32(__float_as_uint(h.s), a, b); x.s = __uint_as_float(a); y.s = __uint_as_float(b);
    pair_xor32((uint32_t)h.idx, a, b); x.idx = (int)a; y.idx = (int)b;
    return stat_merge(x, y);
}
__device__ __forceinline__ Stat stat_shfl_xor(const Stat& a, int o) {
    Stat b;
    b.m = __shfl_xor(a.m, o, 64);
    b.s = __shfl_xor(a.s, o, 64);
    b.idx = __shfl_xor(a.idx, o, 64);
    return b;
}

__device__ __forceinline__ float gelu_tanh_f(float u) {
    // tanh(y) = 1 - 2 / (1 + e^(2y)) (saturates correctly at both ends; near zero the result is added to 1)
    const float y = 0.7978845608028654f * (u + 0.044715f * u * u * u);
    const float th = 1.f - 2.f * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(y * 2.8853900817779268f));
    return 0.5f * u * (1.f + th);
}
__device__ __forceinline__ float silu_f(float u) { return u * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(u * -1.4426950408889634f)); }


// ---- activation traffic: plain vector loads and stores (the kernel boundary makes them visible) ----
__device__ __forceinline__ float4 ld_act4(const float* p) { return *(const float4*)p; }
__device__ __forceinline__ float ld_act(const float* p) { return *p; }
__device__ __forceinline__ void st_u64(void* p, uint32_t lo, uint32_t hi) { *(uint2*)p = make_uint2(lo, hi); }
__device__ __forceinline__ void st_act4(float* p, const float4 v) { *(float4*)p = v; }
__device__ __forceinline__ void st_act(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_u16(uint16_t* p, uint16_t v) { *p = v; }


}  // namespace bild
