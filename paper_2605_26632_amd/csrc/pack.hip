// Online 2:4 sparsification of an activation matrix: magnitude Top-2 of every aligned group of
// four along K (Alg. 1 "X~ <- TopK(X)"), the norm-compensation factor of the method section
// ("Norm-Compensated Sparsification", s = sqrt(|X|^2 / (|X~|^2 + eps))), and compression into
// kept values + 2-bit positions (App. A operand format). One sweep over X; HBM-bandwidth bound:
// 2 bytes read + 1.125 bytes written per input element.
//
// Mapping: one wavefront per row; a lane takes 8 consecutive bf16 (one 16-byte load = two
// groups) per step and the wave walks the row in steps of 512 elements, so every load, the
// 8-byte value stores and the 4-byte metadata stores (four lanes' bytes gathered with DPP
// quad permutes) are contiguous across the wave.
#include "rtl_internal.h"

namespace rtl {
namespace {

constexpr int kWavesPerBlock = 4;
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

// d0 = x0 | x1 << 16, d1 = x2 | x3 << 16 (bf16 bit patterns).
template <int COMP>
__device__ __forceinline__ GroupOut select_group(uint32_t d0, uint32_t d1, float eps) {
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
            if (near | odd_range) {
                s = sqrtf(o.num / d);
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

template <int COMP>
__global__ __launch_bounds__(kWavesPerBlock * 64) void sparsify_pack_kernel(
    const uint16_t* __restrict__ X, int64_t M, int K, int64_t ldx, float eps,
    uint16_t* __restrict__ vals, uint8_t* __restrict__ meta, uint8_t* __restrict__ meta_km,
    int64_t Mpad, float* __restrict__ scale, float* __restrict__ rowsums) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (row >= M) return;  // whole wave leaves together
    const uint16_t* xr = X + row * ldx;
    uint16_t* vr = vals + row * (int64_t)(K / 2);
    uint8_t* mr = meta + row * (int64_t)(K / 8);          // only dereferenced when meta != null
    uint8_t* kmr = meta_km + row * 8;                      // only dereferenced when meta_km != null
    float num = 0.f, den = 0.f;
    // rows of metadata are K/8 bytes: whole 32-bit words only when K is a multiple of 32
    const bool word_meta = (K & 31) == 0;
    for (int k0 = 0; k0 < K; k0 += 512 * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int k = k0 + u * 512 + lane * 8;
            v[u] = make_uint4(0, 0, 0, 0);
            if (k < K) v[u] = *reinterpret_cast<const uint4*>(xr + k);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int k = k0 + u * 512 + lane * 8;
            const GroupOut g0 = select_group<COMP>(v[u].x, v[u].y, eps);
            const GroupOut g1 = select_group<COMP>(v[u].z, v[u].w, eps);
            if constexpr (COMP == RTL_COMP_ROW || COMP == RTL_COMP_TENSOR) {
                num += g0.num + g1.num;   // zero-filled lanes past K contribute nothing
                den += g0.den + g1.den;
            }
            const uint32_t b = g0.nibble | (g1.nibble << 4);
            // gather the metadata bytes of the four lanes of a quad into its first lane
            const uint32_t w = b | (quad_bcast<0x55>(b) << 8) | (quad_bcast<0xAA>(b) << 16) |
                               (quad_bcast<0xFF>(b) << 24);
            if (k < K) {
                *reinterpret_cast<uint2*>(vr + k / 2) = make_uint2(g0.packed, g1.packed);
                if (meta) {
                    if (word_meta) {
                        if ((lane & 3) == 0) *reinterpret_cast<uint32_t*>(mr + k / 8) = w;
                    } else {
                        mr[k / 8] = (uint8_t)b;
                    }
                }
                // k-major twin: the quad's word is half of the row's 8-byte record of block k / 64
                if (meta_km && (lane & 3) == 0)
                    *reinterpret_cast<uint32_t*>(kmr + (int64_t)(k >> 6) * Mpad * 8 + ((k >> 5) & 1) * 4) = w;
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
__global__ __launch_bounds__(256) void tensor_scale_kernel(const float* __restrict__ rowsums,
                                                           int64_t M, float eps,
                                                           float* __restrict__ scale) {
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
    if (threadIdx.x == 0) scale[0] = (float)sqrt(sn[0] / (sd[0] + (double)eps));
}

// One thread per (row, 64-k block): rows run fastest so the k-major writes are contiguous.
__global__ __launch_bounds__(256) void meta_to_kmajor_kernel(const uint8_t* __restrict__ meta,
                                                             int64_t M, int64_t KB, int64_t Mpad,
                                                             uint8_t* __restrict__ km) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= M * KB) return;
    const int64_t row = t % M, kb = t / M;
    const uint2 v = *reinterpret_cast<const uint2*>(meta + row * KB * 8 + kb * 8);
    *reinterpret_cast<uint2*>(km + (kb * Mpad + row) * 8) = v;
}

}  // namespace

hipError_t launch_meta_to_kmajor(const uint8_t* meta, int64_t M, int64_t K, uint8_t* meta_km,
                                 hipStream_t stream) {
    const int64_t KB = K / 64, n = M * KB;
    hipLaunchKernelGGL(meta_to_kmajor_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       meta, M, KB, kmajor_rows(M), meta_km);
    return hipGetLastError();
}

hipError_t launch_sparsify_pack(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                float eps, uint16_t* vals, uint8_t* meta, uint8_t* meta_km,
                                float* scale, float* rowsums, hipStream_t stream) {
    const int64_t Mpad = kmajor_rows(M);
    const dim3 grid((unsigned)((M + kWavesPerBlock - 1) / kWavesPerBlock));
    const dim3 block(kWavesPerBlock * 64);
    switch (comp) {
        case RTL_COMP_NONE:
            hipLaunchKernelGGL(sparsify_pack_kernel<RTL_COMP_NONE>, grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, meta_km, Mpad, scale, rowsums);
            break;
        case RTL_COMP_GROUP:
            hipLaunchKernelGGL(sparsify_pack_kernel<RTL_COMP_GROUP>, grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, meta_km, Mpad, scale, rowsums);
            break;
        case RTL_COMP_ROW:
            hipLaunchKernelGGL(sparsify_pack_kernel<RTL_COMP_ROW>, grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, meta_km, Mpad, scale, rowsums);
            break;
        case RTL_COMP_TENSOR:
            hipLaunchKernelGGL(sparsify_pack_kernel<RTL_COMP_TENSOR>, grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, meta_km, Mpad, scale, rowsums);
            hipLaunchKernelGGL(tensor_scale_kernel, dim3(1), dim3(256), 0, stream, rowsums, M, eps,
                               scale);
            break;
    }
    return hipGetLastError();
}

}  // namespace rtl
