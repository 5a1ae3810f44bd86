// Device helpers of the online 2:4 sparsification, shared by the sweeps that perform it: magnitude
// Top-2 of an aligned group of four (Alg. 1 "X~ <- TopK(X)"), the norm-compensation factor of the
// method section ("Norm-Compensated Sparsification", s = sqrt(|X|^2 / (|X~|^2 + eps))) and the E4M3
// conversion of the FP8 composition.
#pragma once
#include "rtl_internal.h"

namespace rtl {

__device__ __forceinline__ float bits_to_f32(uint32_t u) { return __uint_as_float(u); }

// fp32 -> bf16 round-to-nearest-even, NaN kept (quiet bit set).
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x40u;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? nan : r;
}

struct GroupOut {
    uint32_t packed;  // two kept bf16: lower position in the low half
    uint32_t nibble;  // pos0 | pos1 << 2
    float num, den;   // sum of squares of the four / of the two kept
};

// Two fp32 values -> two E4M3 codes (low byte = first): round to nearest even, saturating at
// +-448 (so do +-inf), NaN -> 0x7F. The hardware conversion is exact for |t| <= 448 but turns
// larger magnitudes into NaN codes, hence the clamp.
__device__ __forceinline__ uint32_t e4m3_pair(float t0, float t1) {
    const float c0 = __builtin_amdgcn_fmed3f(t0, -448.f, 448.f);
    const float c1 = __builtin_amdgcn_fmed3f(t1, -448.f, 448.f);
    uint32_t p = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c0, c1, 0, false) & 0xFFFFu;
    if (__builtin_isunordered(t0, t1)) {   // rare: at least one NaN
        if (t0 != t0) p = (p & 0xFF00u) | 0x7Fu;
        if (t1 != t1) p = (p & 0x00FFu) | 0x7F00u;
    }
    return p;
}

// The compensation factor exactly as defined: every square rounded on its own, the sums in the
// stated order, IEEE divide and square root. Squares of bf16 values are exact in fp32 unless they
// fall below 2^-126, so the fused multiply-adds of the fast path give the same sums for ordinary
// magnitudes; for tiny ones (|x| < 2^-63) only this unfused form matches a plain evaluation.
__device__ __forceinline__ float exact_group_scale(float f0, float f1, float f2, float f3, float ka,
                                                   float kb, float eps) {
#pragma clang fp contract(off)
    const float q0 = f0 * f0, q1 = f1 * f1, q2 = f2 * f2, q3 = f3 * f3;
    const float num = ((q0 + q1) + q2) + q3;
    const float qa = ka * ka, qb = kb * kb;
    const float den = (qa + qb) + eps;
    return sqrtf(num / den);
}

// d0 = x0 | x1 << 16, d1 = x2 | x3 << 16 (bf16 bit patterns). With FP8 the kept pair leaves as two
// E4M3 codes of (s * x) * inv (inv = 1 / x_scale) in the low 16 bits of `packed`.
template <int COMP, bool FP8 = false>
__device__ __forceinline__ GroupOut select_group(uint32_t d0, uint32_t d1, float eps, float inv = 1.0f) {
    // Magnitude keys made unique by appending (3 - position): the larger composite key wins,
    // so equal magnitudes resolve to the lower position.
    const uint32_t c0 = ((d0 & 0x7FFFu) << 2) | 3u;
    const uint32_t c1 = ((d0 >> 14) & 0x1FFFCu) | 2u;
    const uint32_t c2 = ((d1 & 0x7FFFu) << 2) | 1u;
    const uint32_t c3 = ((d1 >> 14) & 0x1FFFCu);
    const uint32_t hi01 = max(c0, c1), lo01 = min(c0, c1);
    const uint32_t hi23 = max(c2, c3), lo23 = min(c2, c3);
    const uint32_t m1 = max(hi01, hi23);
    const uint32_t m2 = max(min(hi01, hi23), hi01 > hi23 ? lo01 : lo23);
    const uint32_t p1 = ~m1 & 3u, p2 = ~m2 & 3u;
    const uint32_t pos0 = min(p1, p2), pos1 = max(p1, p2);
    // The kept pair (lower position in the low half) with one byte permute over the 8 bytes of the group:
    // selector bytes 2 pos0, 2 pos0 + 1, 2 pos1, 2 pos1 + 1 (bytes 0..3 address d0, 4..7 address d1).
    const uint32_t sel = __umul24(pos0 | (pos1 << 16), 0x0202u) + 0x01000100u;
    const uint32_t pair = __builtin_amdgcn_perm(d1, d0, sel);
    GroupOut o;
    o.nibble = pos0 | (pos1 << 2);
    o.num = 0.f;
    o.den = 0.f;
    if constexpr (COMP != RTL_COMP_NONE) {
        const float f0 = bits_to_f32(d0 << 16), f1 = bits_to_f32(d0 & 0xFFFF0000u);
        const float f2 = bits_to_f32(d1 << 16), f3 = bits_to_f32(d1 & 0xFFFF0000u);
        const float ka = bits_to_f32(pair << 16), kb = bits_to_f32(pair & 0xFFFF0000u);
        // squares of bf16 values are exact in fp32; the additions are in the stated order
        // (fused multiply-adds round exactly like a multiply and an add here, see exact_group_scale)
        o.num = __builtin_fmaf(f3, f3, __builtin_fmaf(f2, f2, __builtin_fmaf(f1, f1, f0 * f0)));
        o.den = __builtin_fmaf(kb, kb, ka * ka);
        if constexpr (COMP == RTL_COMP_GROUP) {
            // The stored values are bf16_rne(s * k) with s = sqrtf(num / den) in IEEE fp32. The
            // correctly rounded divide and square root cost ~25 instructions, enough to make this
            // sweep ALU bound, so s is first taken from the 1-ulp hardware reciprocal and square
            // root: relative to the real value the fast product is off by at most 4.5 and the exact
            // one by at most 2.5 half-units, so they differ by at most 7 fp32 units. The exact
            // sequence only runs when a fast product lies within 8 units of a bf16 rounding
            // boundary, i.e. whenever the two could round differently. The result is bit-identical.
            const float d = o.den + eps;
            float s = __builtin_amdgcn_sqrtf(o.num * __builtin_amdgcn_rcpf(d));
            float p0 = s * ka, p1 = s * kb;
            const uint32_t l0 = (__float_as_uint(p0) + 8u) & 0xFFFFu;   // window [0x8000-8, 0x8000+8)
            const uint32_t l1 = (__float_as_uint(p1) + 8u) & 0xFFFFu;
            const bool near = (l0 - 0x8000u < 16u) | (l1 - 0x8000u < 16u);
            // tiny (but non-zero) or huge / non-finite scopes are left to the exact sequence too
            const uint32_t nb = __float_as_uint(o.num);
            const bool odd_range = (nb - 0x0D800000u >= 0x63800000u) & (nb != 0u);
            if constexpr (FP8) {
                // Same idea one rounding later: t = p * inv is what gets rounded, to 3 mantissa
                // bits. The fast and the exact p differ by at most 7 units, which the common
                // multiplication by inv and its own rounding turn into at most 15 units of t, i.e.
                // less than 2^-19 |t|. The conversion is monotone, so if t (1 - 2^-17) and
                // t (1 + 2^-17), which bracket the exact t even after their own roundings, give the
                // same code, the exact t gives it too, wherever the format's boundaries sit
                // (normal range, subnormal range, saturation: beyond 448 the raw conversion returns
                // the NaN code on both sides, or differs across the limit and the exact sequence runs).
                float t0 = p0 * inv, t1 = p1 * inv;
                constexpr float kBelow = 1.0f - 0x1p-17f, kAbove = 1.0f + 0x1p-17f;
                const uint32_t c_below = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(t0 * kBelow, t1 * kBelow, 0, false);
                const uint32_t c_above = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(t0 * kAbove, t1 * kAbove, 0, false);
                if ((c_below != c_above) | odd_range) {
                    s = exact_group_scale(f0, f1, f2, f3, ka, kb, eps);
                    t0 = (s * ka) * inv;
                    t1 = (s * kb) * inv;
                    o.packed = e4m3_pair(t0, t1);
                } else if (fmaxf(fabsf(t0), fabsf(t1)) <= 448.0f) {
                    o.packed = c_below & 0xFFFFu;      // inside the format's range the raw conversion is the code
                } else {
                    o.packed = e4m3_pair(t0, t1);      // saturating values: the raw conversion returns NaN codes
                }
                return o;
            }
            if (near | odd_range) {
                s = exact_group_scale(f0, f1, f2, f3, ka, kb, eps);
                p0 = s * ka;
                p1 = s * kb;
            }
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            const f32x2 pp = {p0, p1};
            const bf16x2 pb = __builtin_convertvector(pp, bf16x2);   // RNE, one instruction on gfx950
            o.packed = __builtin_bit_cast(uint32_t, pb);
            return o;
        }
    }
    if constexpr (FP8) {
        o.packed = e4m3_pair(bits_to_f32(pair << 16) * inv, bits_to_f32(pair & 0xFFFF0000u) * inv);
        return o;
    }
    o.packed = pair;
    return o;
}

}  // namespace rtl
