// Linear layers on the gfx950 matrix cores.
//
//   dense : Y = X W^T                       (paper Eq. linear_layer; v_mfma_f32_32x32x16_bf16)
//   sparse: Y = S(X) W^T, S(X) compressed   (Alg. 1 "Y_s <- S(X) W^T", operand format of App. A;
//                                            v_smfmac_f32_32x32x32_bf16)
//
// Both share one LDS-staged, double-buffered tile loop. A workgroup owns a BM x BN tile of Y and
// walks K in steps of 64. The compressed activation is the FIRST matrix operand of SMFMAC (the
// one that carries 2-of-4 structure along K), so tokens map to the instruction's rows and the
// weight rows (K contiguous) map to its columns: no transposition of either tensor is needed.
//
// Operand layout of v_smfmac_f32_32x32x32_bf16 (measured on the device with one-hot operands):
//   lane l: i = l % 32, kb = l / 32
//   A (8 bf16)  : row i, the kept values of dense k in [16 kb, 16 kb + 16) in order
//   idx (16 bit): ABID picks the 16-bit half of the lane's own index register; nibble g holds
//                 pos0 | pos1 << 2 of the lane's g-th group
//   B (16 bf16) : column i; element u < 8 is dense k = 8 kb + u, u >= 8 is k = 16 + 8 kb + (u - 8)
//   D (16 fp32) : column i, register r is row 8 (r / 4) + 4 kb + r % 4
// The labelling of k inside a 64-wide step is free as long as both operands agree; it is chosen
// so that a lane reads 16-byte chunks from LDS and one 32-bit word of metadata per step.
#include "rtl_internal.h"

namespace rtl {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BK = 64;  // dense k per main-loop step

union Frag8 {
    uint4 u;
    bf16x8 v;
};
union Frag16 {
    uint4 u[2];
    bf16x16 v;
};

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x40u;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? nan : r;
}

template <bool SPARSE, int BM, int BN>
struct Smem {
    static constexpr int kABytes = SPARSE ? BM * 64 : BM * 128;
    static constexpr int kMetaBytes = SPARSE ? BM * 8 : 0;
    static constexpr int kBBytes = BN * 128;
    static constexpr int kStage = kABytes + kMetaBytes + kBBytes;
    static constexpr int kTotal = 2 * kStage;
};

// Byte offset of 16-byte chunk c of a row inside a tile whose rows hold 8 chunks (128 bytes).
__device__ __forceinline__ int swz8(int row, int c) { return row * 128 + ((c ^ (row & 7)) << 4); }
// Same for rows of 4 chunks (64 bytes, the compressed activation): two rows share a 128-byte line.
__device__ __forceinline__ int swz4(int row, int c) {
    const int q = row * 4 + c;
    const int line = q >> 3;
    return (line * 8 + ((q & 7) ^ (line & 7))) << 4;
}

// Tile order: consecutive workgroup ids land on different XCDs (round robin), so ids are first
// regrouped per XCD, then walked in groups of 8 tile-rows so that the ~32 tiles an XCD runs at a
// time share few activation and weight panels in its L2.
__device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int& pm, int& pn) {
    const int nblk = tiles_m * tiles_n;
    const int q = nblk / 8, r = nblk % 8;
    const int xcd = pid % 8, local = pid / 8;
    const int t = (xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q) + local;
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = t / per_group;
    const int first_m = group * GM;
    const int gsize = min(tiles_m - first_m, GM);
    pm = first_m + (t % per_group) % gsize;
    pn = (t % per_group) / gsize;
}

template <bool SPARSE, int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_kernel(const GemmArgs a) {
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 blocks");
    using L = Smem<SPARSE, BM, BN>;
    constexpr int A_CHUNKS = SPARSE ? BM * 4 : BM * 8;
    constexpr int B_CHUNKS = BN * 8;
    static_assert(A_CHUNKS % NT == 0 && B_CHUNKS % NT == 0, "tile loads must divide evenly");
    constexpr int A_PER_T = A_CHUNKS / NT, B_PER_T = B_CHUNKS / NT;
    constexpr int A_CPR = SPARSE ? 4 : 8;          // 16-byte chunks per row per step
    constexpr int A_STEP = SPARSE ? 32 : 64;       // elements of A consumed per step

    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    int pm, pn;
    tile_coords(blockIdx.x, tiles_m, tiles_n, pm, pn);
    const int64_t m0 = (int64_t)pm * BM, n0 = (int64_t)pn * BN;
    const int KT = (int)(a.K / BK);

    // ---- global -> register staging (one 16-byte chunk per slot) ---------------------------
    const uint16_t* pa[A_PER_T];
    bool va[A_PER_T];
    int la[A_PER_T];
#pragma unroll
    for (int s = 0; s < A_PER_T; ++s) {
        const int id = tid + s * NT;
        const int row = id / A_CPR, c = id % A_CPR;
        va[s] = (m0 + row) < a.M;
        pa[s] = a.A + (va[s] ? (m0 + row) : 0) * a.lda + c * 8;
        la[s] = SPARSE ? swz4(row, c) : swz8(row, c);
    }
    const uint16_t* pb[B_PER_T];
    bool vb[B_PER_T];
    int lb[B_PER_T];
#pragma unroll
    for (int s = 0; s < B_PER_T; ++s) {
        const int id = tid + s * NT;
        const int row = id / 8, c = id % 8;
        vb[s] = (n0 + row) < a.N;
        pb[s] = a.W + (vb[s] ? (n0 + row) : 0) * a.ldw + c * 8;
        lb[s] = L::kABytes + L::kMetaBytes + swz8(row, c);
    }
    const uint8_t* pmeta = nullptr;
    bool vmeta = false;
    if constexpr (SPARSE) {
        vmeta = tid < BM && (m0 + tid) < a.M;
        pmeta = a.meta + (vmeta ? (m0 + tid) : 0) * (a.K / 8);
    }

    uint4 ra[A_PER_T], rb[B_PER_T];
    uint2 rmeta = make_uint2(0, 0);

    auto gload = [&](int kt) {
#pragma unroll
        for (int s = 0; s < A_PER_T; ++s) {
            ra[s] = make_uint4(0, 0, 0, 0);
            if (va[s]) ra[s] = *reinterpret_cast<const uint4*>(pa[s] + (int64_t)kt * A_STEP);
        }
#pragma unroll
        for (int s = 0; s < B_PER_T; ++s) {
            rb[s] = make_uint4(0, 0, 0, 0);
            if (vb[s]) rb[s] = *reinterpret_cast<const uint4*>(pb[s] + (int64_t)kt * BK);
        }
        if constexpr (SPARSE) {
            rmeta = make_uint2(0, 0);
            if (vmeta) rmeta = *reinterpret_cast<const uint2*>(pmeta + (int64_t)kt * 8);
        }
    };
    auto lstore = [&](int stage) {
        uint8_t* base = smem + stage * L::kStage;
#pragma unroll
        for (int s = 0; s < A_PER_T; ++s) *reinterpret_cast<uint4*>(base + la[s]) = ra[s];
#pragma unroll
        for (int s = 0; s < B_PER_T; ++s) *reinterpret_cast<uint4*>(base + lb[s]) = rb[s];
        if constexpr (SPARSE) {
            if (tid < BM) *reinterpret_cast<uint2*>(base + L::kABytes + tid * 8) = rmeta;
        }
    };

    // ---- accumulators -------------------------------------------------------------------------
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int li = lane & 31, kb = lane >> 5;
    const int arow0 = wm * WTM + li;   // + tm * 32
    const int brow0 = wn * WTN + li;   // + tn * 32

    auto compute = [&](int stage) {
        const uint8_t* base = smem + stage * L::kStage;
        const uint8_t* bB = base + L::kABytes + L::kMetaBytes;
        if constexpr (SPARSE) {
            const uint8_t* bM = base + L::kABytes;
            int idx[TM];
            Frag8 fa[TM][2];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = arow0 + i * 32;
                idx[i] = *reinterpret_cast<const int*>(bM + row * 8 + kb * 4);
                fa[i][0].u = *reinterpret_cast<const uint4*>(base + swz4(row, 2 * kb));
                fa[i][1].u = *reinterpret_cast<const uint4*>(base + swz4(row, 2 * kb + 1));
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = brow0 + j * 32;
                Frag16 f0, f1;
                f0.u[0] = *reinterpret_cast<const uint4*>(bB + swz8(row, kb));
                f0.u[1] = *reinterpret_cast<const uint4*>(bB + swz8(row, 4 + kb));
                f1.u[0] = *reinterpret_cast<const uint4*>(bB + swz8(row, 2 + kb));
                f1.u[1] = *reinterpret_cast<const uint4*>(bB + swz8(row, 6 + kb));
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(fa[i][0].v, f0.v, acc[i][j],
                                                                          idx[i], 0, 0);
                    acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(fa[i][1].v, f1.v, acc[i][j],
                                                                          idx[i], 0, 1);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag8 fa[TM], fb[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[i].u = *reinterpret_cast<const uint4*>(base + swz8(arow0 + i * 32, 4 * kb + s));
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[j].u = *reinterpret_cast<const uint4*>(bB + swz8(brow0 + j * 32, 4 * kb + s));
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i][j],
                                                                            0, 0, 0);
            }
        }
    };

    // ---- main loop: LDS double buffer, next tile in flight in registers ----------------------
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) gload(kt + 1);
        compute(cur);
        if (kt + 1 < KT) lstore(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: optional fp32 scales, bias, bf16 RNE store -------------------------------
    const float ts = a.tensor_scale ? a.tensor_scale[0] : 1.0f;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int64_t col = n0 + wn * WTN + j * 32 + li;
        if (col >= a.N) continue;
        const float bv = a.bias ? __uint_as_float((uint32_t)a.bias[col] << 16) : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * kb + (r % 4);
                if (row >= a.M) continue;
                float v = acc[i][j][r];
                if (a.row_scale) v *= a.row_scale[row];
                if (a.tensor_scale) v *= ts;
                if (a.bias) v += bv;
                a.Y[row * a.ldy + col] = (uint16_t)f32_to_bf16_rne(v);
            }
        }
    }
}

template <bool SPARSE, int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t stream) {
    using L = Smem<SPARSE, BM, BN>;
    auto kern = gemm_kernel<SPARSE, BM, BN, WAVES_M, WAVES_N>;
    static bool attr_set = false;   // per instantiation; idempotent, so a race is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, L::kTotal);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(WAVES_M * WAVES_N * 64), L::kTotal, stream, a);
    return hipGetLastError();
}

}  // namespace

size_t gemm_workspace_bytes(bool, int64_t, int64_t, int64_t) { return 0; }

hipError_t launch_gemm(bool sparse, const GemmArgs& a, hipStream_t stream) {
    if (sparse) return launch_cfg<true, 256, 256, 2, 4>(a, stream);
    return launch_cfg<false, 256, 256, 2, 4>(a, stream);
}

}  // namespace rtl
