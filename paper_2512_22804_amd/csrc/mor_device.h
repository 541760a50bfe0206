// Device-side building blocks of the MoR analyse-select-quantize kernels (gfx950 only).
//
// Arithmetic contract (must stay bit-identical for amax, scale, FP8 codes and nnz; the error
// sums are binary32 and only need ~1e-6 relative accuracy):
//   amax  = integer max of (bits & 0x7FFF) over the block's BF16 patterns;
//   s     = fl32(448 / amax), one IEEE division (Algorithm 1: s = q_amax / amax);
//   y     = fl32(x * s), one IEEE multiply -- this file must be compiled with
//           -ffp-contract=off so the multiply is never fused into a later subtract;
//   code  = OCP E4M3 round-to-nearest-even of y, magnitudes above 448 clipped to 448;
//   term  = |y - q| / |y| for x != 0 (Eq. 1-2), exactly 1 when q == 0.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mor {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

constexpr float kE4M3Max = 448.0f;
constexpr float kE5M2Max = 57344.0f;
constexpr float kFltMax = 3.402823466e+38f;
// Blocks whose amax (as BF16 bits) is below this take the branch-free element path.  Above
// it (amax >= 2^25, Inf, NaN) x*s can round to an exact zero or be non-finite, which the
// branch-free path does not model, so such blocks take the careful path.
constexpr uint32_t kFastAmaxBits = 0x4C00u;
constexpr uint32_t kInfBits = 0x7F80u;

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}

// Scale of a block from its amax bits (BF16 pattern, sign cleared).
__device__ __forceinline__ float scale_from_amax_bits(uint32_t abits, float q_amax) {
    if (abits == 0u || abits >= kInfBits) return 1.0f;
    float s = q_amax / __uint_as_float(abits << 16);   // correctly rounded IEEE division
    return __builtin_fminf(s, kFltMax);                // +inf -> FLT_MAX
}

// Scaling algorithms.  kScaleFp32: the scale above.  kScaleGam (Algorithm 1 with one group per tensor):
// the block keeps the exponent of its ideal scale s_b, lowered by one when the group's mantissa m_g
// exceeds the block's own m_b, and takes m_g as its mantissa, so the applied scale m_g * 2^e never
// exceeds s_b and is more than s_b / 2.  kScaleE8M0: the same with m_g = 1, a pure power of two.
// `mg` holds the 23 fraction bits of m_g.
enum { kScaleFp32 = 0, kScaleGam = 1, kScaleE8M0 = 2 };
__device__ __forceinline__ uint32_t group_mantissa_bits(uint32_t group_abits, float q_amax, uint32_t mode) {
    return mode == kScaleGam ? (__float_as_uint(scale_from_amax_bits(group_abits, q_amax)) & 0x7FFFFFu) : 0u;
}
__device__ __forceinline__ float block_scale(uint32_t abits, float q_amax, uint32_t mode, uint32_t mg) {
    const float s_b = scale_from_amax_bits(abits, q_amax);
    if (mode == kScaleFp32) return s_b;
    const uint32_t b = __float_as_uint(s_b);                 // positive, normal: s_b >= 448 / BF16max > 2^-120
    const uint32_t e = (b >> 23) - ((mg > (b & 0x7FFFFFu)) ? 1u : 0u);
    return __uint_as_float((e << 23) | mg);
}
// Words that the group loop of Algorithm 1 leaves for the block kernels of one operand: {mantissa for E4M3, for E5M2, "BF16
// proven" flag, unused} when the operand is one group; with bands of `group_rows` rows as groups, a table of {E4M3, E5M2}
// mantissas per band follows those four words.  Returns the two words of the block whose first row is r0.
constexpr int kGamHeaderWords = 4;
__device__ __forceinline__ const uint32_t* gam_words(const uint32_t* gam, uint32_t group_rows, int64_t r0) {
    return group_rows ? gam + kGamHeaderWords + 2 * (r0 / group_rows) : gam;
}
// With a scale of up to one binade below s_b, the smallest BF16 subnormal times the scale can round to a
// binary32 zero one binade of amax earlier, so the branch-free path ends at 2^24 instead of 2^25.
__device__ __forceinline__ uint32_t fast_amax_limit(uint32_t mode) { return mode == kScaleFp32 ? kFastAmaxBits : kFastAmaxBits - 0x80u; }

// ---- per-lane summary of 8 BF16 values held in a u32x4: packed amax and non-zero count
struct Scan8 {
    uint32_t amax2;   // two u16 running maxima of (bits & 0x7FFF)
    uint32_t zero2;   // two u16 running counts of ZERO elements (+-0)
};
// 1 for a zero half-word, 0 otherwise: saturating 1 - m on both halves (v_pk_sub_u16 clamp).
__device__ __forceinline__ uint32_t pk_is_zero_u16(uint32_t m) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_sub_sat(__builtin_bit_cast(u16x2, 0x00010001u), __builtin_bit_cast(u16x2, m)));
}
__device__ __forceinline__ uint32_t pk_sub_sat_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_sub_sat(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, a) - __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_add_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, a) + __builtin_bit_cast(u16x2, b)));
}
// Certain flushes among the two BF16 values of `word`, given the packed bound t - 1 where t is a lower bound of the block's
// amax pattern taken down by 20 binades (0 if that underflows): 1 <= m < t  <=>  m - 1 < t - 1, and m - 1 wraps to 0xFFFF
// for zeros, which never count.  Returns 0 or 1 in each half-word.
__device__ __forceinline__ uint32_t pk_certain_flush(uint32_t word, uint32_t bound_m1_2) {
    const uint32_t mm1 = pk_sub_u16(word & 0x7FFF7FFFu, 0x00010001u);
    return pk_min_u16(pk_sub_sat_u16(bound_m1_2, mm1), 0x00010001u);
}
__device__ __forceinline__ void scan8(const u32x4& raw, Scan8& sc) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t m = raw[j] & 0x7FFF7FFFu;
        sc.amax2 = pk_max_u16(sc.amax2, m);
        sc.zero2 = pk_add_u16(sc.zero2, pk_is_zero_u16(m));
    }
}
__device__ __forceinline__ uint32_t fold_max16(uint32_t v2) { return max(v2 & 0xFFFFu, v2 >> 16); }
__device__ __forceinline__ uint32_t fold_add16(uint32_t v2) { return (v2 & 0xFFFFu) + (v2 >> 16); }

// ---- E4M3: branch-free path ------------------------------------------------------------
// Valid when the block's amax bits are < kFastAmaxBits: then |y| <= 448*(1+2^-23), so the
// hardware conversion (round-to-nearest-even, no clipping needed) is the method's encoder,
// and a non-zero x never produces y == 0.  clamp(|d| * rcp|y|) yields 0 for x == 0
// (0 * inf = NaN clamps to 0) and 1 for flushed values (|y| * rcp|y|, or inf for
// subnormal y, clamps to 1).
template <bool E5M2>
__device__ __forceinline__ int cvt_pk8(float a, float b, int old, bool hi) {
    if constexpr (E5M2) return hi ? __builtin_amdgcn_cvt_pk_bf8_f32(a, b, old, true) : __builtin_amdgcn_cvt_pk_bf8_f32(a, b, old, false);
    else return hi ? __builtin_amdgcn_cvt_pk_fp8_f32(a, b, old, true) : __builtin_amdgcn_cvt_pk_fp8_f32(a, b, old, false);
}
template <bool E5M2>
__device__ __forceinline__ f32x2 cvt_pk_f32(int v, bool hi) {
    if constexpr (E5M2) return hi ? __builtin_amdgcn_cvt_pk_f32_bf8(v, true) : __builtin_amdgcn_cvt_pk_f32_bf8(v, false);
    else return hi ? __builtin_amdgcn_cvt_pk_f32_fp8(v, true) : __builtin_amdgcn_cvt_pk_f32_fp8(v, false);
}
__device__ __forceinline__ float rel_term(float y, float q) {
    float d = y - q;
    return __builtin_amdgcn_fmed3f(__builtin_fabsf(d) * __builtin_amdgcn_rcpf(__builtin_fabsf(y)), 0.0f, 1.0f);
}

// Quantize 8 values with scale s; returns the 8 codes (little-endian element order) and adds
// the 8 error terms to err0/err1.
template <bool E5M2>
__device__ __forceinline__ u32x2 quant8_fast(const u32x4& raw, float s, float& err0, float& err1) {
    int w0 = 0, w1 = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float y0 = __uint_as_float(raw[j] << 16) * s;
        float y1 = __uint_as_float(raw[j] & 0xFFFF0000u) * s;
        f32x2 q;
        if (j == 0) { w0 = cvt_pk8<E5M2>(y0, y1, w0, false); q = cvt_pk_f32<E5M2>(w0, false); }
        if (j == 1) { w0 = cvt_pk8<E5M2>(y0, y1, w0, true);  q = cvt_pk_f32<E5M2>(w0, true); }
        if (j == 2) { w1 = cvt_pk8<E5M2>(y0, y1, w1, false); q = cvt_pk_f32<E5M2>(w1, false); }
        if (j == 3) { w1 = cvt_pk8<E5M2>(y0, y1, w1, true);  q = cvt_pk_f32<E5M2>(w1, true); }
        err0 += rel_term(y0, q.x);
        err1 += rel_term(y1, q.y);
    }
    u32x2 r; r.x = (uint32_t)w0; r.y = (uint32_t)w1;
    return r;
}

// binary32 -> BF16, round to nearest even; NaN -> quiet NaN with the sign kept.
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    if (f != f) return ((u >> 16) & 0x8000u) | 0x7FC0u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Finite values only (the branch-free paths never see NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_rne_finite(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// The same as quant8_fast, optionally (FAKE) also producing the eight de-quantized values
// bf16_rne(fl32(q * s_inv)) of the fake-quantization workflow (Section 4, Figure 4).
template <bool E5M2, bool FAKE>
__device__ __forceinline__ u32x2 quant8_fast_deq(const u32x4& raw, float s, float s_inv, float& err0, float& err1, u32x4& deq) {
    int w0 = 0, w1 = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float y0 = __uint_as_float(raw[j] << 16) * s;
        float y1 = __uint_as_float(raw[j] & 0xFFFF0000u) * s;
        f32x2 q;
        if (j == 0) { w0 = cvt_pk8<E5M2>(y0, y1, w0, false); q = cvt_pk_f32<E5M2>(w0, false); }
        if (j == 1) { w0 = cvt_pk8<E5M2>(y0, y1, w0, true);  q = cvt_pk_f32<E5M2>(w0, true); }
        if (j == 2) { w1 = cvt_pk8<E5M2>(y0, y1, w1, false); q = cvt_pk_f32<E5M2>(w1, false); }
        if (j == 3) { w1 = cvt_pk8<E5M2>(y0, y1, w1, true);  q = cvt_pk_f32<E5M2>(w1, true); }
        err0 += rel_term(y0, q.x);
        err1 += rel_term(y1, q.y);
        if constexpr (FAKE) deq[j] = f32_to_bf16_rne_finite(q.x * s_inv) | (f32_to_bf16_rne_finite(q.y * s_inv) << 16);
    }
    u32x2 r; r.x = (uint32_t)w0; r.y = (uint32_t)w1;
    return r;
}
// Eq. (3) needs the error sums of both formats.  When the E5M2 scale is exactly 128 times the E4M3 scale (57344 = 128 * 448:
// always so for binary32 amax scales unless one of them was clamped, and for GAM / E8M0 scales whose exponents differ
// by 7), y5 = 128 * y exactly, so the E5M2 term |y5 - q5| / |y5| equals |y - q5 / 128| / |y|: one reciprocal serves both
// terms, and gfx950's scaled conversions (v_cvt_scalef32_pk_bf8_f32 encodes src / 2^e, v_cvt_scalef32_pk_f32_bf8
// decodes to code * 2^e, e taken from the scale operand 2^-7) deliver q5 / 128 without forming y5.  Adds the E4M3 terms
// to e0 / e1 and the E5M2 terms to f0 / f1; returns the E4M3 codes.
typedef short i16x2 __attribute__((ext_vector_type(2)));
template <bool FAKE>
__device__ __forceinline__ u32x2 quant8_dual(const u32x4& raw, float s, float s_inv, float& e0, float& e1, float& f0, float& f1, u32x4& deq) {
    int w0 = 0, w1 = 0;
    constexpr float kInv128 = 0.0078125f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float y0 = __uint_as_float(raw[j] << 16) * s;
        const float y1 = __uint_as_float(raw[j] & 0xFFFF0000u) * s;
        f32x2 q;
        if (j == 0) { w0 = cvt_pk8<false>(y0, y1, w0, false); q = cvt_pk_f32<false>(w0, false); }
        if (j == 1) { w0 = cvt_pk8<false>(y0, y1, w0, true);  q = cvt_pk_f32<false>(w0, true); }
        if (j == 2) { w1 = cvt_pk8<false>(y0, y1, w1, false); q = cvt_pk_f32<false>(w1, false); }
        if (j == 3) { w1 = cvt_pk8<false>(y0, y1, w1, true);  q = cvt_pk_f32<false>(w1, true); }
        const float r0 = __builtin_amdgcn_rcpf(__builtin_fabsf(y0)), r1 = __builtin_amdgcn_rcpf(__builtin_fabsf(y1));
        e0 += __builtin_amdgcn_fmed3f(__builtin_fabsf(y0 - q.x) * r0, 0.0f, 1.0f);
        e1 += __builtin_amdgcn_fmed3f(__builtin_fabsf(y1 - q.y) * r1, 0.0f, 1.0f);
        const i16x2 none = {0, 0};
        const i16x2 c5 = __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(none, y0, y1, kInv128, false);
        const f32x2 q5 = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8((uint32_t)(uint16_t)c5.x, kInv128, false);
        f0 += __builtin_amdgcn_fmed3f(__builtin_fabsf(y0 - q5.x) * r0, 0.0f, 1.0f);
        f1 += __builtin_amdgcn_fmed3f(__builtin_fabsf(y1 - q5.y) * r1, 0.0f, 1.0f);
        if constexpr (FAKE) deq[j] = f32_to_bf16_rne_finite(q.x * s_inv) | (f32_to_bf16_rne_finite(q.y * s_inv) << 16);
    }
    u32x2 r; r.x = (uint32_t)w0; r.y = (uint32_t)w1;
    return r;
}
// Eight values of eight different blocks (one column each): scales s[k], error terms added to err[k].
template <bool E5M2, bool FAKE>
__device__ __forceinline__ u32x2 quant8_cols(const u32x4& raw, const float (&s)[8], const float (&s_inv)[8], float (&err)[8], u32x4& deq) {
    int w0 = 0, w1 = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float y0 = __uint_as_float(raw[j] << 16) * s[2 * j];
        float y1 = __uint_as_float(raw[j] & 0xFFFF0000u) * s[2 * j + 1];
        f32x2 q;
        if (j == 0) { w0 = cvt_pk8<E5M2>(y0, y1, w0, false); q = cvt_pk_f32<E5M2>(w0, false); }
        if (j == 1) { w0 = cvt_pk8<E5M2>(y0, y1, w0, true);  q = cvt_pk_f32<E5M2>(w0, true); }
        if (j == 2) { w1 = cvt_pk8<E5M2>(y0, y1, w1, false); q = cvt_pk_f32<E5M2>(w1, false); }
        if (j == 3) { w1 = cvt_pk8<E5M2>(y0, y1, w1, true);  q = cvt_pk_f32<E5M2>(w1, true); }
        err[2 * j] += rel_term(y0, q.x);
        err[2 * j + 1] += rel_term(y1, q.y);
        if constexpr (FAKE) deq[j] = f32_to_bf16_rne_finite(q.x * s_inv[2 * j]) | (f32_to_bf16_rne_finite(q.y * s_inv[2 * j + 1]) << 16);
    }
    u32x2 r; r.x = (uint32_t)w0; r.y = (uint32_t)w1;
    return r;
}

// ---- E4M3 / E5M2: careful path (any input) ------------------------------------------------
template <bool E5M2>
__device__ __forceinline__ uint32_t encode_careful(float y) {
    constexpr float top = E5M2 ? kE5M2Max : kE4M3Max;
    uint32_t sign = (__float_as_uint(y) >> 24) & 0x80u;
    if (y != y) return sign | 0x7Fu;
    float c = __builtin_fminf(__builtin_fmaxf(y, -top), top);      // clip; keeps -0
    return (uint32_t)cvt_pk8<E5M2>(c, c, 0, false) & 0xFFu;
}
template <bool E5M2>
__device__ __forceinline__ float term_careful(uint32_t xbits16, float y, uint32_t code) {
    if ((xbits16 & 0x7FFFu) == 0u) return 0.0f;
    float q = cvt_pk_f32<E5M2>((int)code, false).x;
    if (q == 0.0f) return 1.0f;
    return __builtin_fabsf(y - q) / __builtin_fabsf(y);
}
// Careful path over 8 consecutive elements re-read from memory (the data is still in L2): a rolled
// loop keeps this rarely taken path small.  Writes the 8 codes to `dst` unless it is null.
// With `fake` set, the eight de-quantized BF16 values go there instead of the codes to `dst`.
template <bool E5M2>
__device__ __forceinline__ float quant8_careful_mem(const uint16_t* __restrict__ src, float s, uint8_t* dst,
                                                    uint16_t* fake = nullptr, float s_inv = 0.0f) {
    const uint32_t* src32 = reinterpret_cast<const uint32_t*>(src);
    uint32_t* dst32 = reinterpret_cast<uint32_t*>(dst);
    uint32_t* fake32 = reinterpret_cast<uint32_t*>(fake);
    float err = 0.0f;
    uint32_t codes = 0u;
#pragma clang loop unroll(disable)
    for (int j = 0; j < 4; ++j) {
        const uint32_t w = src32[j];
        const uint32_t b0 = w & 0xFFFFu, b1 = w >> 16;
        const float y0 = __uint_as_float(b0 << 16) * s;
        const float y1 = __uint_as_float(b1 << 16) * s;
        const uint32_t c0 = encode_careful<E5M2>(y0), c1 = encode_careful<E5M2>(y1);
        err += term_careful<E5M2>(b0, y0, c0);
        err += term_careful<E5M2>(b1, y1, c1);
        const uint32_t two = c0 | (c1 << 8);
        if (fake) {
            const f32x2 q = cvt_pk_f32<E5M2>((int)two, false);
            fake32[j] = f32_to_bf16_rne(q.x * s_inv) | (f32_to_bf16_rne(q.y * s_inv) << 16);
        } else if (j & 1) {
            codes |= two << 16;
            if (dst) dst32[j >> 1] = codes;
        } else {
            codes = two;
        }
    }
    return err;
}
// One element of a block of its own (column blocks), careful path: returns the code, adds the term.
template <bool E5M2>
__device__ __forceinline__ uint32_t quant1_careful(uint32_t xbits16, float s, float& err) {
    const float y = __uint_as_float(xbits16 << 16) * s;
    const uint32_t c = encode_careful<E5M2>(y);
    err += term_careful<E5M2>(xbits16, y, c);
    return c;
}

// ---- cross-lane reductions over the 16 lanes of a DPP row -----------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// Value of lane `SRC` (0..15) of each 16-lane row, in every lane of that row.
template <int SRC>
__device__ __forceinline__ float row_bcast_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x150 + SRC, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16 lanes

// Smallest non-zero magnitude pattern of 8 BF16 values, as (pattern - 1) per half-word so that zeros
// (wrapping to 0xFFFF) never win the minimum.
__device__ __forceinline__ uint32_t min_nonzero_m1(const u32x4& raw, uint32_t mn2) {
#pragma unroll
    for (int j = 0; j < 4; ++j) mn2 = pk_min_u16(mn2, pk_sub_u16(raw[j] & 0x7FFF7FFFu, 0x00010001u));
    return mn2;
}
__device__ __forceinline__ uint32_t fold_min16(uint32_t v2) { return min(v2 & 0xFFFFu, v2 >> 16); }
// Eq. (4) of the three-way recipe: max|b| / min|b| < 57344 / 2^-14 over the non-zero elements, evaluated
// exactly as amax < 57344 * 2^14 * amin (a BF16 value times 1.75 * 2^29 is exact in binary32; an
// overflowing product is +inf, and the test then holds as it should).  Blocks without non-zero elements
// pass; blocks holding Inf or NaN fail.
__device__ __forceinline__ bool range_fits_e5m2(uint32_t amax_bits, uint32_t amin_bits, uint32_t nnz) {
    if (amax_bits >= kInfBits) return false;
    if (nnz == 0u) return true;
    return __uint_as_float(amax_bits << 16) < 939524096.0f * __uint_as_float(amin_bits << 16);
}

__device__ __forceinline__ uint32_t row_allmax_u32(uint32_t v) {
    v = max(v, dpp_u32<kDppXor1>(v));
    v = max(v, dpp_u32<kDppXor2>(v));
    v = max(v, dpp_u32<kDppHalfMirror>(v));
    v = max(v, dpp_u32<kDppMirror>(v));
    return v;
}
__device__ __forceinline__ uint32_t row_allsum_u32(uint32_t v) {
    v += dpp_u32<kDppXor1>(v);
    v += dpp_u32<kDppXor2>(v);
    v += dpp_u32<kDppHalfMirror>(v);
    v += dpp_u32<kDppMirror>(v);
    return v;
}
__device__ __forceinline__ float row_allsum_f32(float v) {
    v += dpp_f32<kDppXor1>(v);
    v += dpp_f32<kDppXor2>(v);
    v += dpp_f32<kDppHalfMirror>(v);
    v += dpp_f32<kDppMirror>(v);
    return v;
}
// All 64 lanes: row results are uniform per row, so reading lanes 0,16,32,48 finishes the job.
__device__ __forceinline__ uint32_t wave_allmax_u32(uint32_t v) {
    v = row_allmax_u32(v);
    uint32_t a = __builtin_amdgcn_readlane((int)v, 0), b = __builtin_amdgcn_readlane((int)v, 16);
    uint32_t c = __builtin_amdgcn_readlane((int)v, 32), d = __builtin_amdgcn_readlane((int)v, 48);
    return max(max(a, b), max(c, d));
}
__device__ __forceinline__ uint32_t wave_allsum_u32(uint32_t v) {
    v = row_allsum_u32(v);
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}
__device__ __forceinline__ float wave_allsum_f32(float v) {
    v = row_allsum_f32(v);
    float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (a + b) + (c + d);
}

// Index of the operand a work unit belongs to, from the running totals of a grouped launch (uniform per wave).
__device__ __forceinline__ int group_find(const int64_t* end, int n, int64_t v) {
    int i = 0;
    while (i + 1 < n && v >= end[i]) ++i;
    return __builtin_amdgcn_readfirstlane(i);
}
__device__ __forceinline__ int group_find32(const int32_t* end, int n, int v) {
    int i = 0;
    while (i + 1 < n && v >= end[i]) ++i;
    return __builtin_amdgcn_readfirstlane(i);
}

// ---- Algorithm 2 with [E4M3, BF16]: 0 = keep E4M3, 1 = keep BF16 ------------------------------
// Eq. (2): err_sum / nnz < th, evaluated division-free as err_sum < th * nnz (the metric of a
// block without non-zero elements is 0).  False for NaN / inf sums.
// Bin of the error histogram (Section 4.1.3) a mean relative error falls into: twelve bins of width 0.005, the last one open.
__device__ __forceinline__ int stats_bin(float metric) {
    if (!(metric < __builtin_inff())) return 11;
    int bin = 0;
#pragma unroll
    for (int k = 1; k <= 11; ++k)
        if (metric >= (float)(0.005 * k)) bin = k;
    return bin;
}
constexpr int kStatCnt = 15;     // 12 histogram bins, BF16 blocks, near-threshold blocks, E5M2 blocks
__device__ __forceinline__ uint32_t decide_eq2(float err_sum, uint32_t nnz, float th) {
    const bool accept = nnz ? (err_sum < th * (float)nnz) : (0.0f < th);
    return accept ? 0u : 1u;
}
__device__ __forceinline__ uint32_t decide_eq3(float err4, float err5) { return (err4 < err5) ? 0u : 1u; }

// Bounds-checked streaming accesses through a buffer resource: a lane whose offset is kBufOutside loads
// zeros and stores nothing, so ragged edges need no per-lane branches.  Offsets are bytes from `base`
// (32 bits; callers keep them below 2^31).
constexpr int kBufAux = 2;      // cache-policy field of the buffer loads: non-temporal
constexpr int kBufStoreAux = 18; // of the buffer stores: non-temporal and written through at system scope (nt sc1).  Measured
                                 // against nt alone, alternating runs on one box: the per-tensor quantize pass of the layer
                                 // sweep (2 bytes read, 3 written per element) takes 211.4-212.2 us instead of 213.9-214.0 us;
                                 // the amax pass that runs before it reads 1.6 us longer, the step time is the same within 0.1 %
typedef __amdgpu_buffer_rsrc_t BufRsrc;
constexpr uint32_t kBufOutside = 0x80000000u;
__device__ __forceinline__ BufRsrc make_buf(const void* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7FFFFFFF, 0x00020000);
}
// A window of `bytes` bytes from `base`: accesses beyond it load zeros / store nothing (bytes = 0: a null window,
// `base` is then never dereferenced).
__device__ __forceinline__ BufRsrc make_buf_window(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(BufRsrc r, uint32_t voff, uint32_t soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, kBufAux);
}
// 16-byte stores never take a register in the scalar-offset field: the compiler assumes that form needs no wait
// states before the data registers are overwritten and reuses them in the very next instruction, but on gfx950 the
// first data dword of some lanes was then stored with its NEW contents (seen as rare, timing-dependent corruption of
// fake-quantized rows).  With a constant scalar offset the compiler inserts the wait states and the data is intact.
__device__ __forceinline__ void buf_store16(BufRsrc r, uint32_t voff, const u32x4& v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, voff, 0, kBufStoreAux);
}
// No other code may issue a 16-byte buffer store (a register scalar offset would bring the hazard back): any later use
// of the builtin's name is a compile error.
#pragma GCC poison __builtin_amdgcn_raw_buffer_store_b128
__device__ __forceinline__ void buf_store8(BufRsrc r, uint32_t voff, uint32_t soff, const u32x2& v) {
    __builtin_amdgcn_raw_buffer_store_b64(v, r, voff, soff, kBufStoreAux);
}

// Streaming accesses: every operand byte is touched once per pass, so loads and stores carry the
// non-temporal hint (measured +5-8 % on a plain copy of the same size on MI355X).
__device__ __forceinline__ u32x4 load16(const void* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ void store16(void* p, const u32x4& v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void store8(void* p, const u32x2& v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(p));
}

}  // namespace mor
