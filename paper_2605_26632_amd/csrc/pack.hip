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
// When only the k-major output is wanted and nothing is summed along a row (the rtl_sparse_linear
// path with NONE / GROUP scope), sparsify_pack_block_kernel runs instead: its mapping follows the
// output layout (32 rows x 64-k blocks per wave) and every access is a whole line. (The FP8 sweep keeps
// the row mapping: with its heavier per-group arithmetic the block mapping measured the same.)
#include "rtl_internal.h"
#include "select.h"

namespace rtl {
namespace {

constexpr int kWavesPerBlock = 8;
constexpr int kUnroll = 3;   // 6 and 24 steps per row at K = 3072 / 12288 divide evenly

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
    float* __restrict__ rowsums, const float* __restrict__ x_scale, int parts) {
    const int lane = threadIdx.x & 63;
    // `parts` waves share a row (NONE / GROUP only: nothing is summed along the row), each taking a
    // run of whole 512-element steps; short rows then still give every SIMD enough waves in flight.
    const int64_t gw = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t row = gw / parts;
    if (row >= M) return;  // whole wave leaves together
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

// The same sweep for the case that matters most: only the k-major outputs are wanted (what
// rtl_sparse_linear feeds its tile loop) and nothing is summed along a row (NONE / GROUP). Then the
// mapping can follow the OUTPUT layout instead of the input rows: a wave takes 32 rows and a run of
// 64-k blocks; per block, lane (r, c) = (lane / 8, lane % 8) loads chunk c (16 bytes, two groups) of
// the rows r, r + 8, r + 16, r + 24 of its 32. Every load instruction then reads 8 whole 128-byte
// lines, every value store writes 512 contiguous bytes (the 64-byte blocks of 8 neighbouring rows are
// adjacent in the k-major layout) and the metadata of a row (8 bytes per block) leaves as one store.
// The row mapping above writes the same buffer as 64-byte pieces of single rows, half a line at a
// time, which costs HBM efficiency once the activation is large.
constexpr int kBlockWaves = 4;      // waves per workgroup: the same 32 rows, consecutive runs of blocks
constexpr int kBlockUnroll = 2;     // 64-k blocks in flight per wave
template <int COMP>
__global__ __launch_bounds__(kBlockWaves * 64) void sparsify_pack_block_kernel(
    const uint16_t* __restrict__ X, int64_t M, int KB, int64_t ldx, float eps, uint8_t* __restrict__ vals_km,
    uint8_t* __restrict__ meta_km, int64_t Mpad, int per, unsigned row_blocks) {
    const int lane = threadIdx.x & 63, r8 = lane >> 3, c = lane & 7;
    const int wave = threadIdx.x >> 6;
    // workgroup id = run group * row_blocks + row block: neighbours take neighbouring rows of one K range
    const int64_t m0 = (int64_t)(blockIdx.x % row_blocks) * 32;
    const int b0 = ((int)(blockIdx.x / row_blocks) * kBlockWaves + wave) * per;   // first block of this wave's run
    const int b1 = min(KB, b0 + per);
    const uint16_t* xr[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) xr[t] = X + min(m0 + 8 * t + r8, M - 1) * ldx + c * 8;   // rows past M: clamped, results land in padding rows
    // lane's row r8 of the tile (t adds 8 rows = 512 bytes of values, 64 bytes of metadata)
    uint8_t* vdst = vals_km + (m0 + r8) * 64 + c * 8;
    uint8_t* mdst = meta_km + (m0 + r8) * 8;
    for (int b = b0; b < b1; b += kBlockUnroll) {
        uint4 v[kBlockUnroll][4];
#pragma unroll
        for (int u = 0; u < kBlockUnroll; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                v[u][t] = make_uint4(0, 0, 0, 0);
                if (b + u < b1) v[u][t] = *reinterpret_cast<const uint4*>(xr[t] + (int64_t)(b + u) * 64);
            }
#pragma unroll
        for (int u = 0; u < kBlockUnroll; ++u) {
            if (b + u >= b1) break;
            uint8_t* vb = vdst + (int64_t)(b + u) * Mpad * 64;
            uint8_t* mb = mdst + (int64_t)(b + u) * Mpad * 8;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const GroupOut g0 = select_group<COMP, false>(v[u][t].x, v[u][t].y, eps);
                const GroupOut g1 = select_group<COMP, false>(v[u][t].z, v[u][t].w, eps);
                *reinterpret_cast<uint2*>(vb + t * 512) = make_uint2(g0.packed, g1.packed);
                // the row's eight metadata bytes: quads gather theirs into a word, the first quad of the
                // row fetches the second quad's word from four lanes up
                const uint32_t nb = g0.nibble | (g1.nibble << 4);
                const uint32_t w = nb | (quad_bcast<0x55>(nb) << 8) | (quad_bcast<0xAA>(nb) << 16) |
                                   (quad_bcast<0xFF>(nb) << 24);
                const uint32_t w_hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)w, 0x104, 0xF, 0xF, true);   // row_shl:4
                if (c == 0) *reinterpret_cast<uint2*>(mb + t * 64) = make_uint2(w, w_hi);
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
    const float2* rs = reinterpret_cast<const float2*>(rowsums);
    int64_t r = threadIdx.x;
    for (; r + 3 * 256 < M; r += 4 * 256) {     // four loads in flight; the additions keep the row order of a thread
        const float2 v0 = rs[r], v1 = rs[r + 256], v2 = rs[r + 512], v3 = rs[r + 768];
        n += (double)v0.x; d += (double)v0.y;
        n += (double)v1.x; d += (double)v1.y;
        n += (double)v2.x; d += (double)v2.y;
        n += (double)v3.x; d += (double)v3.y;
    }
    for (; r < M; r += 256) {
        const float2 v = rs[r];
        n += (double)v.x;
        d += (double)v.y;
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
                                  hipStream_t stream) {
    const int64_t Mpad = kmajor_rows(M);
    if constexpr (!FP8) {
        // only the k-major outputs, nothing summed along a row: the block mapping (see its kernel)
        if (!vals && !meta && vals_km && meta_km && K % 64 == 0 &&
            (comp == RTL_COMP_NONE || comp == RTL_COMP_GROUP)) {
            // Blocks per wave: two once the rows are long (measured flat between one and three: at
            // [4096,12288] 190.9 / 190.7 / 190.2 us per rtl_sparse_linear call, at [16896,12288] 817 / 812 /
            // 814; six and more lose), one for short rows, where more waves matter more.
            const int KB = (int)(K / 64);
            const int per = KB >= 96 ? kBlockUnroll : 1;
            const int runs = (KB + per - 1) / per;                     // waves per 32 rows
            const int64_t row_blocks = (M + 31) / 32, groups = (runs + kBlockWaves - 1) / kBlockWaves;
            if (row_blocks * groups < ((int64_t)1 << 31)) {            // (else: far beyond memory; the row mapping serves)
                const dim3 grid((unsigned)(row_blocks * groups));
                if (comp == RTL_COMP_GROUP)
                    hipLaunchKernelGGL((sparsify_pack_block_kernel<RTL_COMP_GROUP>), grid, dim3(kBlockWaves * 64), 0,
                                       stream, X, M, KB, ldx, eps, vals_km, meta_km, Mpad, per, (unsigned)row_blocks);
                else
                    hipLaunchKernelGGL((sparsify_pack_block_kernel<RTL_COMP_NONE>), grid, dim3(kBlockWaves * 64), 0,
                                       stream, X, M, KB, ldx, eps, vals_km, meta_km, Mpad, per, (unsigned)row_blocks);
                return hipGetLastError();
            }
        }
    }
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
                               (int)K, ldx, eps, vals, meta, vals_km, meta_km, Mpad, scale, rowsums, x_scale, parts);
            break;
        case RTL_COMP_GROUP:
            hipLaunchKernelGGL((sparsify_pack_kernel<RTL_COMP_GROUP, FP8>), grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, vals_km, meta_km, Mpad, scale, rowsums, x_scale, parts);
            break;
        case RTL_COMP_ROW:
            hipLaunchKernelGGL((sparsify_pack_kernel<RTL_COMP_ROW, FP8>), grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, vals_km, meta_km, Mpad, scale, rowsums, x_scale, parts);
            break;
        case RTL_COMP_TENSOR:
            hipLaunchKernelGGL((sparsify_pack_kernel<RTL_COMP_TENSOR, FP8>), grid, block, 0, stream, X, M,
                               (int)K, ldx, eps, vals, meta, vals_km, meta_km, Mpad, scale, rowsums, x_scale, parts);
            hipLaunchKernelGGL(tensor_scale_kernel, dim3(1), dim3(256), 0, stream, rowsums, M, eps,
                               scale, x_scale, fused_scale);
            break;
    }
    return hipGetLastError();
}

hipError_t launch_sparsify_pack(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                float eps, uint16_t* vals, uint8_t* meta, uint8_t* vals_km,
                                uint8_t* meta_km, float* scale, float* rowsums, hipStream_t stream) {
    return launch_pack_any<false>(X, M, K, ldx, comp, eps, vals, meta, vals_km, meta_km, scale, rowsums,
                                  nullptr, nullptr, stream);
}

hipError_t launch_sparsify_pack_fp8(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                    float eps, const float* x_scale, uint8_t* vals8, uint8_t* meta,
                                    uint8_t* vals_km, uint8_t* meta_km, float* scale, float* rowsums,
                                    float* fused_scale, hipStream_t stream) {
    return launch_pack_any<true>(X, M, K, ldx, comp, eps, vals8, meta, vals_km, meta_km, scale, rowsums,
                                 x_scale, fused_scale, stream);
}

hipError_t launch_tensor_scale(const float* rowsums, int64_t M, float eps, float* scale, hipStream_t stream,
                               const float* mul, float* fused) {
    hipLaunchKernelGGL(tensor_scale_kernel, dim3(1), dim3(256), 0, stream, rowsums, M, eps, scale, mul, fused);
    return hipGetLastError();
}

hipError_t launch_quantize_fp8(const uint16_t* W, int64_t rows, int64_t cols, int64_t ld, uint8_t* Wq,
                               int64_t ldq, hipStream_t stream) {
    const int64_t n = rows * (cols / 8);
    hipLaunchKernelGGL(quantize_fp8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, W,
                       rows, cols / 8, ld, Wq, ldq);
    return hipGetLastError();
}

}  // namespace rtl
