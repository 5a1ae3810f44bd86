// One pass over X for the LoRA branch of Alg. 1: the sweep that sparsifies and compresses the
// activation ("X~ <- TopK(X)", "S(X) <- s X~", App. A operand format) also forms the rank-64
// down-projection T = X L_B^T of the residual "Y_r <- X (L_A L_B)^T", evaluated as (X L_B^T) L_A^T.
// X is 100 MB at the headline shape and a second sweep over it costs as much as two thirds of the
// first, so both consumers are fed from the same tile in LDS.
//
// Mapping: a workgroup of four waves owns 128 rows and a run of 64-k blocks (the contraction is split
// over workgroups so that every compute unit has rows to stream; the fp32 partial planes are summed in
// range order by lora_reduce_kernel). A stage is one 64-k block: 128 rows x 128 bytes of X and the 64
// rows x 128 bytes of L_B, brought into a ring of LDS buffers with direct-to-LDS loads (whole lines,
// no register staging). Wave w takes rows 32 w .. 32 w + 31: lane (i, kb) reads the 64 bytes
// [64 kb, 64 kb + 64) of row i as four 16-byte chunks. Each chunk is at once
//   * the first operand of two v_mfma_f32_32x32x16_bf16 (one per 32 ranks), with the matching chunk of
//     L_B as the second (the labelling of k inside a stage is free as long as both operands agree), and
//   * two groups of four for the Top-2 selection, whose kept values and positions leave in the k-major
//     layout the tile loop streams: 32 bytes of values and 4 bytes of metadata per lane and stage,
//     contiguous over the wave (rows of a 64-k block are 64 and 8 bytes apart).
// ROW and TENSOR scopes sum squares along the whole row; every workgroup leaves the sums of its K range
// beside its partial plane and lora_reduce_kernel adds them up in range order as well.
#include "rtl_internal.h"
#include "select.h"

namespace rtl {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

union Chunk {
    uint4 u;
    bf16x8 v;
};

constexpr int kRows = 128;                    // rows of a workgroup
constexpr int kStages = 3;                    // ring depth
constexpr int kXBytes = kRows * 128;          // X tile of a stage
constexpr int kBBytes = kLoraRank * 128;      // L_B tile of a stage
constexpr int kStageBytes = kXBytes + kBBytes;
constexpr int kLds = kStages * kStageBytes;   // 72 KiB: two workgroups per compute unit

// Rows of 8 chunks (128 bytes): the 16 consecutive rows a 16-byte read serves together must land in
// 16 different 16-byte slots modulo 256 bytes: the row parity picks the half, the chunk index is XORed
// with bits 1..3 of the row.
__device__ __forceinline__ int swz(int row, int c) { return row * 128 + ((c ^ ((row >> 1) & 7)) << 4); }

// lane l of a wave-wide direct-to-LDS load fetches 16 bytes from its own address; the hardware writes
// them to lds_base + 16 l (lds_base wave-uniform, in M0)
__device__ __forceinline__ void dma16(const void* gaddr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_base), "v"(gaddr) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vm() {   // at most N loads of this wave outstanding, LDS reads returned
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 0xF) | ((N >> 4) << 14));
}

// FP8: the kept values leave as E4M3 codes of (s x) / x_scale[0] in the FP8 form of the k-major layout
// (blocks of 128 dense k: 64 codes and a 16-byte metadata record per row; a stage is half a block).
template <int COMP, bool FP8>
__global__ __launch_bounds__(256) void pack_down_kernel(const uint16_t* __restrict__ X, int64_t M, int KT, int64_t ldx,
                                                           float eps, const float* __restrict__ x_scale,
                                                           const uint16_t* __restrict__ LB, int64_t ldlb,
                                                           uint8_t* __restrict__ vals_km, uint8_t* __restrict__ meta_km,
                                                           int64_t Mpad, float* __restrict__ partials,
                                                           float* __restrict__ sums, int per) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)smem;
    const int64_t m0 = (int64_t)blockIdx.x * kRows;
    const int split = blockIdx.y;
    const int kt0 = split * per;                         // first 64-k block of this workgroup
    const int nst = min(per, KT - kt0);                  // >= 1 by the launcher's choice of `per`

    // ---- global -> LDS: every lane owns fixed chunks of the two tiles; rows past M are clamped to the
    //      last row (their results are never stored) -------------------------------------------------
    // X tile: 1024 chunks = 16 wave-wide loads, four per wave; L_B tile: 512 chunks, two per wave
    const uint8_t* gx[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int p = (wave * 4 + s) * 64 + lane;        // chunk position in the swizzled tile
        const int row = p >> 3, c = (p & 7) ^ ((row >> 1) & 7);
        gx[s] = reinterpret_cast<const uint8_t*>(X + min(m0 + row, M - 1) * ldx + (int64_t)kt0 * 64) + c * 16;
    }
    const uint8_t* gb[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int p = (wave * 2 + s) * 64 + lane;
        const int row = p >> 3, c = (p & 7) ^ ((row >> 1) & 7);
        gb[s] = reinterpret_cast<const uint8_t*>(LB + (int64_t)row * ldlb + (int64_t)kt0 * 64) + c * 16;
    }
    auto request = [&](int st) {                         // stage st of this workgroup into ring buffer st % kStages
        const uint32_t base = lds0 + (st % kStages) * kStageBytes;
#pragma unroll
        for (int s = 0; s < 4; ++s) dma16(gx[s] + (int64_t)st * 128, base + (wave * 4 + s) * 1024);
#pragma unroll
        for (int s = 0; s < 2; ++s) dma16(gb[s] + (int64_t)st * 128, base + kXBytes + (wave * 2 + s) * 1024);
    };
    constexpr int kLoads = 6;                            // requests per wave and stage

    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    float num = 0.f, den = 0.f;        // ROW / TENSOR: sums of squares of this lane's half of its row, all / kept

    const int li = lane & 31, kb = lane >> 5;
    const int64_t row = m0 + wave * 32 + li;             // < Mpad: the k-major buffers are padded to whole 256-row tiles
    uint8_t* vrow = vals_km + ((int64_t)kt0 * Mpad + row) * 64 + kb * 32;      // bf16 form
    uint8_t* mrow = meta_km + ((int64_t)kt0 * Mpad + row) * 8 + kb * 4;
    float inv = 1.0f;
    if constexpr (FP8) inv = 1.0f / x_scale[0];

    // ---- prologue: two stages in flight ---------------------------------------------------------------
    request(0);
    if (nst > 1) request(1);
    for (int st = 0; st < nst; ++st) {
        // stage st has landed (the younger stage st + 1 may still be in flight)
        if (st + 1 < nst) wait_vm<kLoads>(); else wait_vm<0>();
        __builtin_amdgcn_s_barrier();                    // ... for every wave; and nobody reads stage st - 1 any more
        if (st + 2 < nst) request(st + 2);               // into the buffer of stage st - 1
        const uint8_t* bx = smem + (st % kStages) * kStageBytes;
        const uint8_t* bb = bx + kXBytes;
        Chunk a[4], b[2][4];
#pragma unroll
        for (int s = 0; s < 4; ++s) a[s].u = *reinterpret_cast<const uint4*>(bx + swz(wave * 32 + li, 4 * kb + s));
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int s = 0; s < 4; ++s) b[j][s].u = *reinterpret_cast<const uint4*>(bb + swz(j * 32 + li, 4 * kb + s));
        // ---- T += X L_B^T on the matrix cores ----
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s].v, b[j][s].v, acc[j], 0, 0, 0);
        // ---- select, compensate, compress the same four chunks (eight groups of four) ----
        uint32_t kept[8], nib = 0;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const GroupOut g0 = select_group<COMP, FP8>(a[s].u.x, a[s].u.y, eps, inv);
            const GroupOut g1 = select_group<COMP, FP8>(a[s].u.z, a[s].u.w, eps, inv);
            if constexpr (COMP == RTL_COMP_ROW || COMP == RTL_COMP_TENSOR) {
                num += g0.num + g1.num;
                den += g0.den + g1.den;
            }
            kept[2 * s] = g0.packed;
            kept[2 * s + 1] = g1.packed;
            nib |= (g0.nibble | (g1.nibble << 4)) << (8 * s);
        }
        if constexpr (FP8) {
            // stage kt0 + st is half `h` of the 128-k block (kt0 + st) / 2: 16 codes at 32 h + 16 kb of the
            // row's 64, 4 metadata bytes at 8 h + 4 kb of its 16
            const int kt = kt0 + st, h = kt & 1;
            const int64_t rec = (int64_t)(kt >> 1) * Mpad + row;
            *reinterpret_cast<uint4*>(vals_km + rec * 64 + h * 32 + kb * 16) =
                make_uint4(kept[0] | (kept[1] << 16), kept[2] | (kept[3] << 16), kept[4] | (kept[5] << 16),
                           kept[6] | (kept[7] << 16));
            *reinterpret_cast<uint32_t*>(meta_km + rec * 16 + h * 8 + kb * 4) = nib;
        } else {
            uint8_t* vdst = vrow + (int64_t)st * Mpad * 64;
            *reinterpret_cast<uint4*>(vdst) = make_uint4(kept[0], kept[1], kept[2], kept[3]);
            *reinterpret_cast<uint4*>(vdst + 16) = make_uint4(kept[4], kept[5], kept[6], kept[7]);
            *reinterpret_cast<uint32_t*>(mrow + (int64_t)st * Mpad * 8) = nib;
        }
    }

    // ---- fp32 partial plane of this K range: register r of a lane is row 8 (r / 4) + 4 kb + r % 4 of
    //      column li of the wave's 32 x 32 block ------------------------------------------------------
    float* out = partials + (int64_t)split * M * kLoraRank;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t orow = m0 + wave * 32 + 8 * (r / 4) + 4 * kb + (r % 4);
            if (orow < M) out[orow * kLoraRank + j * 32 + li] = acc[j][r];
        }
    // ROW / TENSOR: the two lanes of a row add their halves; sums of this K range, [splits][M][2]
    if constexpr (COMP == RTL_COMP_ROW || COMP == RTL_COMP_TENSOR) {
        num += __shfl_xor(num, 32, 64);
        den += __shfl_xor(den, 32, 64);
        if (kb == 0 && row < M) {
            float* sd = sums + ((int64_t)split * M + row) * 2;
            sd[0] = num;
            sd[1] = den;
        }
    }
}

// Ordered sum of the partial planes, T stored as two bf16 planes [2][M][64]: hi = bf16(T), lo =
// bf16(T - hi) (the matrix unit takes bf16 operands; the pair keeps 16 significant bits). ROW / TENSOR:
// the first M threads also add the row sums of the K ranges in order and emit the row's factor
// s = sqrt(|X|^2 / (|X~|^2 + eps)) (ROW) or the row's two sums for the tensor-wide factor (TENSOR).
__global__ __launch_bounds__(256) void lora_reduce_kernel(const float* __restrict__ partials, int splits, int64_t M,
                                                          uint16_t* __restrict__ T, const float* __restrict__ sums,
                                                          int comp, float eps, float* __restrict__ scale,
                                                          float* __restrict__ rowsums) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= M * kLoraRank) return;
    float acc = 0.f;
    for (int sp0 = 0; sp0 < splits; sp0 += 8) {          // the loads of up to eight ranges in flight together
        float p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) p[u] = sp0 + u < splits ? partials[(int64_t)(sp0 + u) * M * kLoraRank + e] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (sp0 + u < splits) acc += p[u];
    }
    const uint32_t hi = f32_to_bf16_rne(acc);
    T[e] = (uint16_t)hi;
    T[M * kLoraRank + e] = (uint16_t)f32_to_bf16_rne(acc - __uint_as_float(hi << 16));
    if ((comp == RTL_COMP_ROW || comp == RTL_COMP_TENSOR) && e < M) {
        float n = 0.f, d = 0.f;
        for (int sp = 0; sp < splits; ++sp) {
            n += sums[((int64_t)sp * M + e) * 2];
            d += sums[((int64_t)sp * M + e) * 2 + 1];
        }
        if (comp == RTL_COMP_ROW) {
            scale[e] = sqrtf(n / (d + eps));
        } else {
            rowsums[2 * e] = n;
            rowsums[2 * e + 1] = d;
        }
    }
}

}  // namespace

hipError_t prepare_pack_lora_kernels() {
    hipError_t e = hipSuccess;
    auto run = [&](const void* k) {
        if (e == hipSuccess) e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    };
    run(reinterpret_cast<const void*>(pack_down_kernel<RTL_COMP_NONE, false>));
    run(reinterpret_cast<const void*>(pack_down_kernel<RTL_COMP_GROUP, false>));
    run(reinterpret_cast<const void*>(pack_down_kernel<RTL_COMP_ROW, false>));
    run(reinterpret_cast<const void*>(pack_down_kernel<RTL_COMP_TENSOR, false>));
    run(reinterpret_cast<const void*>(pack_down_kernel<RTL_COMP_NONE, true>));
    run(reinterpret_cast<const void*>(pack_down_kernel<RTL_COMP_GROUP, true>));
    run(reinterpret_cast<const void*>(pack_down_kernel<RTL_COMP_ROW, true>));
    run(reinterpret_cast<const void*>(pack_down_kernel<RTL_COMP_TENSOR, true>));
    return e;
}

// K ranges of the fused sweep: enough workgroups (128 rows each) to give every compute unit two, at
// least 8 ranges (workgroups that walk different parts of K touch different memory channels at any
// moment), at most 16 (partial-plane traffic), every range at least one 64-k block.
static int pack_down_ranges(int64_t M, int64_t K, int* per_out) {
    const int64_t tiles = (M + kRows - 1) / kRows;
    const int KT = (int)(K / 64);
    int want = (int)((512 + tiles - 1) / tiles);
    want = want < 8 ? 8 : (want > 16 ? 16 : want);
    if (want > KT) want = KT;
    const int per = (KT + want - 1) / want;
    if (per_out) *per_out = per;
    return (KT + per - 1) / per;
}
int pack_down_splits(int64_t M, int64_t K) { return pack_down_ranges(M, K, nullptr); }

size_t pack_down_scratch_bytes(int64_t M, int64_t K) {     // partial planes, then the row sums of the K ranges
    return (size_t)pack_down_splits(M, K) * (size_t)M * (kLoraRank + 2) * sizeof(float);
}

hipError_t launch_pack_down(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp, float eps,
                            const uint16_t* LB, int64_t ldlb, uint8_t* vals_km, uint8_t* meta_km, float* scratch,
                            uint16_t* T, float* scale, float* rowsums, hipStream_t stream, const float* x_scale,
                            float* fused_scale) {
    int per = 1;
    const int splits = pack_down_ranges(M, K, &per);
    const dim3 grid((unsigned)((M + kRows - 1) / kRows), (unsigned)splits);
    const int64_t Mpad = kmajor_rows(M);
    float* partials = scratch;
    float* sums = scratch + (size_t)splits * (size_t)M * kLoraRank;
    const bool fp8 = x_scale != nullptr;
#define RTL_PACK_DOWN(C)                                                                                              \
    do {                                                                                                              \
        if (fp8)                                                                                                      \
            hipLaunchKernelGGL((pack_down_kernel<C, true>), grid, dim3(256), kLds, stream, X, M, (int)(K / 64), ldx,  \
                               eps, x_scale, LB, ldlb, vals_km, meta_km, Mpad, partials, sums, per);                  \
        else                                                                                                          \
            hipLaunchKernelGGL((pack_down_kernel<C, false>), grid, dim3(256), kLds, stream, X, M, (int)(K / 64), ldx, \
                               eps, x_scale, LB, ldlb, vals_km, meta_km, Mpad, partials, sums, per);                  \
    } while (0)
    switch (comp) {
        case RTL_COMP_NONE: RTL_PACK_DOWN(RTL_COMP_NONE); break;
        case RTL_COMP_GROUP: RTL_PACK_DOWN(RTL_COMP_GROUP); break;
        case RTL_COMP_ROW: RTL_PACK_DOWN(RTL_COMP_ROW); break;
        case RTL_COMP_TENSOR: RTL_PACK_DOWN(RTL_COMP_TENSOR); break;
    }
#undef RTL_PACK_DOWN
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t n = M * kLoraRank;
    hipLaunchKernelGGL(lora_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, partials, splits,
                       M, T, sums, (int)comp, eps, scale, rowsums);
    e = hipGetLastError();
    if (e != hipSuccess || comp != RTL_COMP_TENSOR) return e;
    return launch_tensor_scale(rowsums, M, eps, scale, stream, x_scale, fused_scale);
}

}  // namespace rtl
