// Online 2:4 sparsification of an activation matrix: magnitude Top-2 of every aligned group of
// four along K (Alg. 1 "X~ <- TopK(X)"), the norm-compensation factor of the method section
// ("Norm-Compensated Sparsification", s = sqrt(|X|^2 / (|X~|^2 + eps))), and compression into
// kept values + 2-bit positions (App. A operand format). One sweep over X; HBM-bandwidth bound:
// 2 bytes read + 1.125 bytes written per input element.
//
// Mapping: one wavefront per row (two for long rows, each taking a run of whole steps); a lane
// takes 8 consecutive bf16 (one 16-byte load = two groups) per step and the wave walks the row in
// steps of 512 elements, so every load, the
// 8-byte value stores and the 4-byte metadata stores (four lanes' bytes gathered with DPP
// quad permutes) are contiguous across the wave in the canonical (row-major) output. The
// k-major output the GEMM streams (64-byte value blocks and 8-byte metadata records per row and
// 64-k block, rows contiguous) is written as 64-byte pieces, two neighbouring rows per line.
#include "rtl_internal.h"

namespace rtl {
namespace {

constexpr int kWavesPerBlock = 8;
constexpr int kUnroll = 3;   // 6 and 24 steps per row at K = 3072 / 12288 divide evenly

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
    const uint64_t x64 = (uint64_t)d0 | ((uint64_t)d1 << 32);
    uint32_t v0 = (uint32_t)(x64 >> (16u * pos0)) & 0xFFFFu;
    uint32_t v1 = (uint32_t)(x64 >> (16u * pos1)) & 0xFFFFu;
    GroupOut o;
    o.nibble = pos0 | (pos1 << 2);
    o.num = 0.f;
    o.den = 0.f;
    if constexpr (COMP != RTL_COMP_NONE) {
        const float f0 = bits_to_f32(d0 << 16), f1 = bits_to_f32(d0 & 0xFFFF0000u);
        const float f2 = bits_to_f32(d1 << 16), f3 = bits_to_f32(d1 & 0xFFFF0000u);
        const float ka = bits_to_f32(v0 << 16), kb = bits_to_f32(v1 << 16);
        // squares of bf16 values are exact in fp32; the additions are in the stated order
        o.num = ((f0 * f0 + f1 * f1) + f2 * f2) + f3 * f3;
        o.den = ka * ka + kb * kb;
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
                }
                o.packed = e4m3_pair(t0, t1);
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
        o.packed = e4m3_pair(bits_to_f32(v0 << 16) * inv, bits_to_f32(v1 << 16) * inv);
        return o;
    }
    o.packed = v0 | (v1 << 16);
    return o;
}

template <int CTRL>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, true);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// `vals`: bf16 [M,K/2], or one-byte E4M3 codes [M,K/2] when FP8 (then x_scale[0] is the divisor).
template <int COMP, bool FP8>
__global__ __launch_bounds__(kWavesPerBlock * 64) void sparsify_pack_kernel(
    const uint16_t* __restrict__ X, int64_t M, int K, int64_t ldx, float eps,
    void* __restrict__ vals, uint8_t* __restrict__ meta, uint8_t* __restrict__ vals_km,
    uint8_t* __restrict__ meta_km, int64_t Mpad, float* __restrict__ scale,
    float* __restrict__ rowsums, const float* __restrict__ x_scale, int parts, LoraReduce lora) {
    const int lane = threadIdx.x & 63;
    // `parts` waves share a row (NONE / GROUP only: nothing is summed along the row), each taking a
    // run of whole 512-element steps; short rows then still give every SIMD enough waves in flight.
    const int64_t gw = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t row = gw / parts;
    if (row >= M) return;  // whole wave leaves together
    // Side job for the LoRA branch (Alg. 1 "Y_r <- X (L_A L_B)^T" evaluated as (X L_B^T) L_A^T): the
    // first wave of a row folds the row's split-contraction partials of T = X L_B^T in range order and
    // stores T as two bf16 planes, hi = bf16(T), lo = bf16(T - hi) (the matrix unit takes bf16 operands;
    // the pair keeps 16 significant bits). 64 values per row: one per lane.
    if (lora.T && gw % parts == 0) {
        // (the loads of up to eight ranges are in flight together; the additions keep the range order)
        float acc = 0.f;
        for (int sp0 = 0; sp0 < lora.splits; sp0 += 8) {
            float p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                p[u] = sp0 + u < lora.splits ? lora.partials[((int64_t)(sp0 + u) * M + row) * 64 + lane] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (sp0 + u < lora.splits) acc += p[u];
        }
        const uint32_t hi = f32_to_bf16_rne(acc);
        lora.T[row * 64 + lane] = (uint16_t)hi;
        lora.T[(M + row) * 64 + lane] = (uint16_t)f32_to_bf16_rne(acc - __uint_as_float(hi << 16));
    }
    const int span = ((K + parts - 1) / parts + 511) / 512 * 512;
    const int kbeg = (int)(gw % parts) * span;
    const int kend = min(K, kbeg + span);
    const uint16_t* xr = X + row * ldx;
    // canonical value row (only dereferenced when vals != null): bf16 form / FP8 form
    uint16_t* vr = static_cast<uint16_t*>(vals) + row * (int64_t)(K / 2);
    uint8_t* vr8 = static_cast<uint8_t*>(vals) + row * (int64_t)(K / 2);
    uint8_t* vkr = vals_km + row * 64;                     // only dereferenced when vals_km != null
    uint8_t* mr = meta + row * (int64_t)(K / 8);          // only dereferenced when meta != null
    constexpr int KM_REC = FP8 ? 16 : 8;                   // k-major record: 128 or 64 dense k
    uint8_t* kmr = meta_km + row * KM_REC;                 // only dereferenced when meta_km != null
    float inv = 1.0f;
    if constexpr (FP8) inv = 1.0f / x_scale[0];
    float num = 0.f, den = 0.f;
    // rows of metadata are K/8 bytes: whole 32-bit words only when K is a multiple of 32
    const bool word_meta = (K & 31) == 0;
    for (int k0 = kbeg; k0 < kend; k0 += 512 * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int k = k0 + u * 512 + lane * 8;
            v[u] = make_uint4(0, 0, 0, 0);
            if (k < kend) v[u] = *reinterpret_cast<const uint4*>(xr + k);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int k = k0 + u * 512 + lane * 8;
            const GroupOut g0 = select_group<COMP, FP8>(v[u].x, v[u].y, eps, inv);
            const GroupOut g1 = select_group<COMP, FP8>(v[u].z, v[u].w, eps, inv);
            if constexpr (COMP == RTL_COMP_ROW || COMP == RTL_COMP_TENSOR) {
                num += g0.num + g1.num;   // zero-filled lanes past K contribute nothing
                den += g0.den + g1.den;
            }
            const uint32_t b = g0.nibble | (g1.nibble << 4);
            // gather the metadata bytes of the four lanes of a quad into its first lane
            const uint32_t w = b | (quad_bcast<0x55>(b) << 8) | (quad_bcast<0xAA>(b) << 16) |
                               (quad_bcast<0xFF>(b) << 24);
            if (k < kend) {
                if constexpr (FP8) {
                    const uint32_t codes = g0.packed | (g1.packed << 16);
                    if (vals) *reinterpret_cast<uint32_t*>(vr8 + k / 2) = codes;
                    // k-major twin: 64 codes (64 bytes) per row and 128-k block
                    if (vals_km)
                        *reinterpret_cast<uint32_t*>(vkr + (int64_t)(k >> 7) * Mpad * 64 + ((k & 127) >> 1)) = codes;
                } else {
                    const uint2 pair = make_uint2(g0.packed, g1.packed);
                    if (vals) *reinterpret_cast<uint2*>(vr + k / 2) = pair;
                    // k-major twin: 32 values (64 bytes) per row and 64-k block
                    if (vals_km)
                        *reinterpret_cast<uint2*>(vkr + (int64_t)(k >> 6) * Mpad * 64 + (k & 63)) = pair;
                }
                if (meta) {
                    if (word_meta) {
                        if ((lane & 3) == 0) *reinterpret_cast<uint32_t*>(mr + k / 8) = w;
                    } else {
                        mr[k / 8] = (uint8_t)b;
                    }
                }
                // k-major twin: the quad's word is one 32-k slice of the row's record of its block
                // (8 bytes per 64 k, or 16 bytes per 128 k with FP8 values)
                if (meta_km && (lane & 3) == 0) {
                    if constexpr (FP8)
                        *reinterpret_cast<uint32_t*>(kmr + (int64_t)(k >> 7) * Mpad * 16 + ((k >> 5) & 3) * 4) = w;
                    else
                        *reinterpret_cast<uint32_t*>(kmr + (int64_t)(k >> 6) * Mpad * 8 + ((k >> 5) & 1) * 4) = w;
                }
            }
        }
    }
    if constexpr (COMP == RTL_COMP_ROW || COMP == RTL_COMP_TENSOR) {
        num = wave_sum(num);
        den = wave_sum(den);
        if (lane == 0) {
            if constexpr (COMP == RTL_COMP_ROW) {
                scale[row] = sqrtf(num / (den + eps));
            } else {
                rowsums[2 * row] = num;
                rowsums[2 * row + 1] = den;
            }
        }
    }
}

// TENSOR scope: fold the per-row sums in a fixed order (fp64) and emit the single factor.
// `fused` (nullable) receives the factor times mul[0] (the FP8 activation scale).
__global__ __launch_bounds__(256) void tensor_scale_kernel(const float* __restrict__ rowsums,
                                                           int64_t M, float eps,
                                                           float* __restrict__ scale,
                                                           const float* __restrict__ mul,
                                                           float* __restrict__ fused) {
    __shared__ double sn[256], sd[256];
    double n = 0.0, d = 0.0;
    for (int64_t r = threadIdx.x; r < M; r += 256) {
        n += (double)rowsums[2 * r];
        d += (double)rowsums[2 * r + 1];
    }
    sn[threadIdx.x] = n;
    sd[threadIdx.x] = d;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            sn[threadIdx.x] += sn[threadIdx.x + s];
            sd[threadIdx.x] += sd[threadIdx.x + s];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float sc = (float)sqrt(sn[0] / (sd[0] + (double)eps));
        scale[0] = sc;
        if (fused) fused[0] = mul[0] * sc;
    }
}

// Direct cast bf16 -> E4M3 (weights "directly quantized to FP8"): 8 elements per thread.
__global__ __launch_bounds__(256) void quantize_fp8_kernel(const uint16_t* __restrict__ W, int64_t rows,
                                                           int64_t cols8, int64_t ld,
                                                           uint8_t* __restrict__ Wq, int64_t ldq) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * cols8) return;
    const int64_t r = t / cols8, c = (t % cols8) * 8;
    const uint4 v = *reinterpret_cast<const uint4*>(W + r * ld + c);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t lo = e4m3_pair(bits_to_f32(w[2 * h] << 16), bits_to_f32(w[2 * h] & 0xFFFF0000u));
        const uint32_t hi = e4m3_pair(bits_to_f32(w[2 * h + 1] << 16), bits_to_f32(w[2 * h + 1] & 0xFFFF0000u));
        o[h] = lo | (hi << 16);
    }
    *reinterpret_cast<uint2*>(Wq + r * ldq + c) = make_uint2(o[0], o[1]);
}

// One thread per (row, 64-k block) and 16-byte piece: rows run fastest so that the k-major writes of
// a warp are contiguous. Piece 0..3 = the block's 64 bytes of values; piece 0 also moves the
// 8-byte metadata record.
__global__ __launch_bounds__(256) void operand_to_kmajor_kernel(const uint16_t* __restrict__ vals,
                                                                const uint8_t* __restrict__ meta,
                                                                int64_t M, int64_t KB, int64_t Mpad,
                                                                uint8_t* __restrict__ vals_km,
                                                                uint8_t* __restrict__ meta_km) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= M * KB * 4) return;
    const int piece = (int)(t & 3);
    const int64_t row = (t >> 2) % M, kb = (t >> 2) / M;
    const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint8_t*>(vals) +
                                                    (row * KB + kb) * 64 + piece * 16);
    *reinterpret_cast<uint4*>(vals_km + (kb * Mpad + row) * 64 + piece * 16) = v;
    if (piece == 0) {
        const uint2 m = *reinterpret_cast<const uint2*>(meta + row * KB * 8 + kb * 8);
        *reinterpret_cast<uint2*>(meta_km + (kb * Mpad + row) * 8) = m;
    }
}

}  // namespace

// Querying one kernel makes the runtime load this translation unit's code object.
hipError_t prepare_pack_kernels() {
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(operand_to_kmajor_kernel));
}

hipError_t launch_operand_to_kmajor(const uint16_t* vals, const uint8_t* meta, int64_t M, int64_t K,
                                    uint8_t* vals_km, uint8_t* meta_km, hipStream_t stream) {
    const int64_t KB = K / 64, n = M * KB * 4;
    hipLaunchKernelGGL(operand_to_kmajor_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       vals, meta, M, KB, kmajor_rows(M), vals_km, meta_km);
    return hipGetLastError();
}

template <bool FP8>
static hipError_t launch_pack_any(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                  float eps, void* vals, uint8_t* meta, uint8_t* vals_km, uint8_t* meta_km,
                                  float* scale, float* rowsums, const float* x_scale, float* fused_scale,
                                  LoraReduce lora, hipStream_t stream) {
    const int64_t Mpad = kmajor_rows(M);
    // Waves per row: two once each still has a full unrolled trip of work (measured: 34 -> 31 us at
    // [4096,12288], 141 -> 131 us at [16896,12288], no change at K = 3072; four or more waves per row
    // lose on the short rows). ROW / TENSOR sum along the row inside one wave.
    int parts = 1;
    if ((comp == RTL_COMP_NONE || comp == RTL_COMP_GROUP) && K >= 2 * 512 * kUnroll) parts = 2;
    const dim3 grid((unsigned)((M * parts + kWavesPerBlock - 1) / kWavesPerBlock));
    const dim3 block(kWavesPerBlock * 64);
    switch (comp) {
        case RTL_COMP_NONE:
            hipLaunchKernelGGL((sparsify_pack_kernel<RTL_COMP_NONE, FP8>), grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, vals_km, meta_km, Mpad, scale, rowsums, x_scale, parts, lora);
            break;
        case RTL_COMP_GROUP:
            hipLaunchKernelGGL((sparsify_pack_kernel<RTL_COMP_GROUP, FP8>), grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, vals_km, meta_km, Mpad, scale, rowsums, x_scale, parts, lora);
            break;
        case RTL_COMP_ROW:
            hipLaunchKernelGGL((sparsify_pack_kernel<RTL_COMP_ROW, FP8>), grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, vals_km, meta_km, Mpad, scale, rowsums, x_scale, parts, lora);
            break;
        case RTL_COMP_TENSOR:
            hipLaunchKernelGGL((sparsify_pack_kernel<RTL_COMP_TENSOR, FP8>), grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, vals_km, meta_km, Mpad, scale, rowsums, x_scale, parts, lora);
            hipLaunchKernelGGL(tensor_scale_kernel, dim3(1), dim3(256), 0, stream, rowsums, M, eps,
                               scale, x_scale, fused_scale);
            break;
    }
    return hipGetLastError();
}

hipError_t launch_sparsify_pack(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                float eps, uint16_t* vals, uint8_t* meta, uint8_t* vals_km,
                                uint8_t* meta_km, float* scale, float* rowsums, hipStream_t stream,
                                LoraReduce lora) {
    return launch_pack_any<false>(X, M, K, ldx, comp, eps, vals, meta, vals_km, meta_km, scale, rowsums,
                                  nullptr, nullptr, lora, stream);
}

hipError_t launch_sparsify_pack_fp8(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                    float eps, const float* x_scale, uint8_t* vals8, uint8_t* meta,
                                    uint8_t* vals_km, uint8_t* meta_km, float* scale, float* rowsums,
                                    float* fused_scale, hipStream_t stream) {
    return launch_pack_any<true>(X, M, K, ldx, comp, eps, vals8, meta, vals_km, meta_km, scale, rowsums,
                                 x_scale, fused_scale, LoraReduce{}, stream);
}

hipError_t launch_quantize_fp8(const uint16_t* W, int64_t rows, int64_t cols, int64_t ld, uint8_t* Wq,
                               int64_t ldq, hipStream_t stream) {
    const int64_t n = rows * (cols / 8);
    hipLaunchKernelGGL(quantize_fp8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, W,
                       rows, cols / 8, ld, Wq, ldq);
    return hipGetLastError();
}

}  // namespace rtl
