// Linear layers on the gfx950 matrix cores.
//
//   dense : Y = X W^T                       (paper Eq. linear_layer; v_mfma_f32_32x32x16_bf16)
//   sparse: Y = S(X) W^T, S(X) compressed   (Alg. 1 "Y_s <- S(X) W^T", operand format of App. A;
//                                            v_smfmac_f32_32x32x32_bf16)
//
// Both share one tile loop. A workgroup owns a BM x BN tile of Y and walks K in stages; a stage is
// two matrix-instruction sub-steps deep (64 dense k for the sparse kernel, 32 for the dense one, so
// both spend the same number of matrix cycles per stage). Stages travel HBM/L2 -> LDS with
// direct-to-LDS loads (no register staging) through a ring of LDS buffers, and each wave keeps the
// operand fragments of the next sub-step in flight while the matrix core works on the current one.
// The sparse kernel reads its compressed operand in the k-major layout the pack sweep writes
// (values and metadata of a 256-row tile contiguous per stage: whole 128-byte lines only); the
// dense operands X and W are the caller's row-major tensors.
//
// The compressed activation is the FIRST matrix operand of SMFMAC (the one that carries 2-of-4
// structure along K), so tokens map to the instruction's rows and the weight rows (K contiguous)
// map to its columns: no transposition of either tensor is needed.
//
// Operand layout of v_smfmac_f32_32x32x32_bf16 (measured on the device with one-hot operands):
//   lane l: i = l % 32, kb = l / 32
//   A (8 bf16)  : row i, the kept values of dense k in [16 kb, 16 kb + 16) in order
//   idx (16 bit): ABID picks the 16-bit half of the lane's own index register; nibble g holds
//                 pos0 | pos1 << 2 of the lane's g-th group
//   B (16 bf16) : column i; element u < 8 is dense k = 8 kb + u, u >= 8 is k = 16 + 8 kb + (u - 8)
//   D (16 fp32) : column i, register r is row 8 (r / 4) + 4 kb + r % 4
// v_mfma_f32_32x32x16_bf16: A and B (8 bf16) hold k = 8 kb + v of row / column i; D as above.
// The labelling of k inside a stage is free as long as both operands agree; it is chosen so that
// a lane reads whole 16-byte chunks from LDS and one 32-bit word of metadata per stage.
//
// FP8 variant of the sparse kernel (E4M3 codes on both operands, the W8A8 composition of the
// implementation-details section): v_smfmac_f32_32x32x64_fp8_fp8, measured the same way:
//   A (16 fp8)  : row i, the kept values of dense k in [32 kb, 32 kb + 32) in order
//   idx (32 bit): the whole register, nibble g = pos0 | pos1 << 2 of the lane's g-th group
//   B (32 fp8)  : column i; element u < 16 is dense k = 16 kb + u, u >= 16 is k = 32 + 16 kb + (u - 16)
//   D           : as above
// In bytes this is the bf16 geometry (16-byte A chunk, two 16-byte B chunks at the same chunk
// indices), so a stage simply covers 128 dense k instead of 64 and the kernel differs only in the
// instruction and in the metadata record (16 bytes per row and stage, one 32-bit word per sub-step).
#include <mutex>
#include <type_traits>
#include <vector>
#include "rtl_internal.h"

namespace rtl {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

union Frag8 {
    uint4 u;
    bf16x8 v;
    i32x4 q;     // 16 fp8
};
union Frag16 {
    uint4 u[2];
    bf16x16 v;
    i32x8 q;     // 32 fp8
};

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x40u;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? nan : r;
}

// Direct-to-LDS load of one wave: lane l fetches `bytes` (16 or 4) from its own global address and
// the hardware writes them to LDS address lds_base + l * bytes (lds_base is wave-uniform and
// travels in M0). Written as inline assembly so that the outstanding-load counter stays under
// the kernel's own control: the loads of a stage are awaited with an explicit vmcnt wait right
// before the barrier that publishes the stage, and reads of older stages never wait for them.
__device__ __forceinline__ void lds_dma16(const void* gaddr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_base), "v"(gaddr) : "memory", "m0");
}
__device__ __forceinline__ void lds_dma4(const void* gaddr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                 :: "s"(lds_base), "v"(gaddr) : "memory", "m0");
}
// Same with a wave-uniform 64-bit base (SGPR pair) plus a 32-bit per-lane byte offset: the per-lane
// state of a stream shrinks to one register and the walk along K is a scalar addition.
__device__ __forceinline__ uint64_t uniform64(const void* p) {   // pin a wave-uniform pointer to SGPRs
    const uint64_t b = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ void lds_dma16_so(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(voff), "s"(uniform64(sbase)) : "memory", "m0");
}
__device__ __forceinline__ void lds_dma4_so(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(lds_base), "v"(voff), "s"(uniform64(sbase)) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt_lgkm0() {   // vmcnt <= N, all LDS reads returned
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 0xF) | ((N >> 4) << 14));
}

// Per-stage LDS footprint. Rows of the A tile hold 64 bytes in both kernels (32 kept bf16 of 64
// dense k, or 32 dense k); rows of the B tile hold 128 bytes (sparse) or 64 bytes (dense).
// D64 (dense only): stages of 64 dense k, 128-byte rows on both sides, so that every L2 request
// of the row-major operands is a whole line; a sub-step is then two matrix instructions deep.
template <bool SPARSE, int BM, int BN, int STAGES, int WAVES_M = 1, int WAVES_N = 1, bool FP8 = false,
          bool D64 = false>
struct Smem {
    static constexpr int kABytes = BM * (D64 ? 128 : 64);
    static constexpr int kMetaRec = FP8 ? 16 : 8;   // metadata bytes per row and stage
    static constexpr int kMetaBytes = SPARSE ? BM * kMetaRec : 0;
    static constexpr int kBBytes = (SPARSE || D64) ? BN * 128 : BN * 64;
    static constexpr int kStage = kABytes + kMetaBytes + kBBytes;
    static constexpr int kRing = STAGES * kStage;
    // epilogue staging: every wave owns (BM / WAVES_M) rows of (BN / WAVES_N) bf16 plus 16 bytes
    // of padding per row (keeps rows 4 apart, written together, in different banks)
    static constexpr int kEpiRowBytes = (BN / WAVES_N) * 2 + 16;
    static constexpr int kEpi = WAVES_M * WAVES_N * (BM / WAVES_M) * kEpiRowBytes;
    static constexpr int kTotal = kRing > kEpi ? kRing : kEpi;
    static_assert(kTotal <= 160 * 1024, "LDS budget of a CU");
};

// LDS swizzles. A 16-byte read of a wave is served 16 lanes at a time over 64 four-byte banks, so
// the 16 consecutive tile rows those lanes address (same logical chunk c) must land in 16 different
// 16-byte slots modulo 256 bytes.
// Rows of 8 chunks (128 bytes): two rows per 256 bytes; the row parity picks the half, c is XORed
// with bits 1..3 of the row.
__device__ __forceinline__ int swz8(int row, int c) { return row * 128 + ((c ^ ((row >> 1) & 7)) << 4); }
// Rows of 4 chunks (64 bytes): four rows per 256 bytes; c is XORed with bits 2..3 of the row.
__device__ __forceinline__ int swz4(int row, int c) { return row * 64 + ((c ^ ((row >> 2) & 3)) << 4); }
// Inverse maps: which (row, c) lives at chunk position p of the tile.
__device__ __forceinline__ void unswz8(int p, int& row, int& c) {
    row = p >> 3;
    c = (p & 7) ^ ((row >> 1) & 7);
}
__device__ __forceinline__ void unswz4(int p, int& row, int& c) {
    row = p >> 2;
    c = (p & 3) ^ ((row >> 2) & 3);
}

// Tile order: consecutive workgroup ids land on different XCDs (round robin), so ids are first
// regrouped per XCD (XCD x works through a contiguous share of the tile list), and the list walks
// the tile grid in groups of 8 tile-rows so that the ~32 tiles an XCD runs at a time share few
// activation and weight panels in its L2.
__device__ __forceinline__ int xcd_share_start(int n, int xcd) {   // first list index of XCD xcd's share of n tiles
    return xcd * (n / 8) + min(xcd, n % 8);
}
__device__ __forceinline__ void tile_walk(int t, int tiles_m, int tiles_n, int& pm, int& pn) {
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = t / per_group;
    const int first_m = group * GM;
    const int gsize = min(tiles_m - first_m, GM);
    pm = first_m + (t % per_group) % gsize;
    pn = (t % per_group) / gsize;
}

// MODE 0: plain linear. MODE 1 (sparse only): LoRA tail, the accumulators also receive T L_A^T before
// the epilogue.
// `tile`: index of this workgroup's output tile in the walk of the (M / BM) x (N / BN) tile grid.
template <bool SPARSE, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int MODE = 0, bool FP8 = false,
          bool D64 = false>
__device__ __forceinline__ void gemm_tile(const GemmArgs a, const int tile) {
    static_assert(!D64 || (!SPARSE && MODE != 1), "64-k stages: dense kernels only");
    static_assert(MODE == 0 || (MODE == 1 && SPARSE), "mode/operand combination");
    static_assert(!FP8 || SPARSE, "FP8 operands: sparse kernels only");
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 blocks");
    using L = Smem<SPARSE, BM, BN, STAGES, WAVES_M, WAVES_N, FP8, D64>;
    constexpr int ESZ = FP8 ? 1 : 2;                  // bytes per operand element
    constexpr int KSTAGE = SPARSE ? 128 / ESZ : (D64 ? 64 : 32);   // dense k per stage
    constexpr int A_ELEMS = D64 ? 64 : 64 / ESZ;      // elements of an A row per stage: 64 bytes (D64: 128)
    constexpr int NMMA = D64 ? 2 * TM * TN : TM * TN; // matrix instructions of a sub-step
    constexpr int MREC = L::kMetaRec;                 // metadata bytes per row and stage
    constexpr int IXW = FP8 ? 2 : 1;                  // metadata words a lane holds per stage and row block
    // one wave-wide direct-to-LDS load moves 64 chunks of 16 bytes = 1 KiB
    constexpr int A_LOADS = L::kABytes / 1024;
    static_assert(A_LOADS % NW == 0, "tile loads must divide over the waves");
    // The B tile is dealt to the waves in runs of B_CH 16-byte chunks. When that is an odd
    // multiple of 32 (192-row dense tile: 96 chunks), a wave's last load runs with its upper half
    // masked off, so every wave still issues the same number of loads.
    constexpr int B_CH = L::kBBytes / 16 / NW;
    static_assert((L::kBBytes / 16) % NW == 0 && B_CH % 32 == 0, "B tile must divide over the waves");
    constexpr int A_PER_W = A_LOADS / NW, B_PER_W = (B_CH + 63) / 64;
    constexpr bool B_HALF = (B_CH % 64) != 0;
    constexpr int M_LOADS = SPARSE ? (BM * MREC) / 256 : 0;  // metadata: 4 bytes per lane per load
    static_assert(!SPARSE || M_LOADS % NW == 0, "metadata loads must divide over the waves");
    constexpr int M_PER_W = M_LOADS / NW;

    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, lives in an SGPR
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)smem;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    int pm, pn;
    tile_walk(tile, tiles_m, tiles_n, pm, pn);
    const int64_t m0 = (int64_t)pm * BM, n0 = (int64_t)pn * BN;
    const int KT = (int)(a.K / KSTAGE);

    // ---- global -> LDS: every lane owns fixed chunks; rows past the edge are clamped to the last
    //      valid row (their products only reach outputs that are never stored) -----------------
    // wave-uniform bases of this tile's three streams, already advanced to the first stage
    // Sparse A is the k-major value buffer: 64 bytes per row and stage, the rows of a stage
    // contiguous, so the tile's stage is one 16 KiB run; dense A is row-major X.
    const int64_t rows_pad = a.rows_pad;    // rows per k block of the k-major operand (whole activation)
    const int64_t a_stride = SPARSE ? rows_pad * 64 : (int64_t)(A_ELEMS * ESZ);   // bytes between stages
    const uint8_t* base_a = SPARSE
        ? static_cast<const uint8_t*>(a.A) + m0 * 64
        : static_cast<const uint8_t*>(a.A) + m0 * a.lda * ESZ;
    const uint8_t* base_b = static_cast<const uint8_t*>(a.W) + n0 * a.ldw * ESZ;
    const int64_t rows_a = a.M - m0, rows_b = a.N - n0;     // valid rows from the tile's first row
    uint32_t oa[A_PER_W];
#pragma unroll
    for (int s = 0; s < A_PER_W; ++s) {
        const int p = (wave * A_PER_W + s) * 64 + lane;
        int row, c;
        if constexpr (D64) unswz8(p, row, c); else unswz4(p, row, c);
        const int64_t gr = min((int64_t)row, rows_a - 1);
        // (the k-major buffer is padded to whole tiles: rows past M hold unspecified bytes whose
        //  products only reach outputs that are never stored)
        oa[s] = SPARSE ? (uint32_t)(row * 64 + c * 16) : (uint32_t)(gr * a.lda * ESZ + c * 16);
    }
    uint32_t ob[B_PER_W];
#pragma unroll
    for (int s = 0; s < B_PER_W; ++s) {
        const int p = wave * B_CH + min(s * 64 + lane, B_CH - 1);   // masked lanes of a half load: any valid chunk
        int row, c;
        if constexpr (SPARSE || D64) unswz8(p, row, c); else unswz4(p, row, c);
        const int64_t gr = min((int64_t)row, rows_b - 1);
        ob[s] = (uint32_t)(gr * a.ldw * ESZ + c * 16);
    }
    const uint8_t* base_m = nullptr;
    uint32_t om = 0;
    if constexpr (SPARSE) {
        // k-major records: the rows of this tile are one contiguous run per stage (2 KiB, 4 KiB with
        // FP8 operands) and wave w moves M_PER_W 256-byte pieces of it, 4 bytes per lane
        base_m = a.meta + m0 * MREC;
        om = (uint32_t)(wave * M_PER_W * 256 + lane * 4);
    }

    const int64_t meta_stride = rows_pad * MREC;   // bytes between stage blocks
    // Load number n (0 .. LOADS_PER_STAGE-1) of this wave for stage kt into ring buffer `stage`.
    // The loads of a stage are issued one at a time between matrix instructions: the texture
    // addresser takes a wave-wide 1 KiB request every ~16 cycles and a wave stalls at a request
    // that finds it busy, so a burst of requests from all waves would leave the matrix cores idle.
    auto gload_one = [&](int kt, int stage, auto n_tag) {
        constexpr int n = decltype(n_tag)::value;
        const uint32_t base = lds0 + stage * L::kStage;
        if constexpr (n < A_PER_W) {
            lds_dma16_so(base_a + (int64_t)kt * a_stride, oa[n], base + (wave * A_PER_W + n) * 1024);
        } else if constexpr (n < A_PER_W + B_PER_W) {
            constexpr int s = n - A_PER_W;
            const uint32_t dst = base + L::kABytes + L::kMetaBytes + (wave * B_CH + s * 64) * 16;
            if constexpr (B_HALF && s == B_PER_W - 1) {
                if (lane < 32) lds_dma16_so(base_b + (int64_t)kt * (KSTAGE * ESZ), ob[s], dst);
            } else {
                lds_dma16_so(base_b + (int64_t)kt * (KSTAGE * ESZ), ob[s], dst);
            }
        } else if constexpr (SPARSE && n < A_PER_W + B_PER_W + M_PER_W) {
            constexpr int s = n - A_PER_W - B_PER_W;
            lds_dma4_so(base_m + (int64_t)kt * meta_stride + s * 256, om,
                        base + L::kABytes + (wave * M_PER_W + s) * 256);
        }
    };
    auto gload = [&](int kt, int stage) {
        gload_one(kt, stage, std::integral_constant<int, 0>{});
        gload_one(kt, stage, std::integral_constant<int, 1>{});
        gload_one(kt, stage, std::integral_constant<int, 2>{});
        gload_one(kt, stage, std::integral_constant<int, 3>{});
        gload_one(kt, stage, std::integral_constant<int, 4>{});
        gload_one(kt, stage, std::integral_constant<int, 5>{});
        gload_one(kt, stage, std::integral_constant<int, 6>{});
        gload_one(kt, stage, std::integral_constant<int, 7>{});
        gload_one(kt, stage, std::integral_constant<int, 8>{});
        gload_one(kt, stage, std::integral_constant<int, 9>{});
        gload_one(kt, stage, std::integral_constant<int, 10>{});
        gload_one(kt, stage, std::integral_constant<int, 11>{});
        gload_one(kt, stage, std::integral_constant<int, 12>{});
        gload_one(kt, stage, std::integral_constant<int, 13>{});
        gload_one(kt, stage, std::integral_constant<int, 14>{});
        gload_one(kt, stage, std::integral_constant<int, 15>{});
    };
    constexpr int LOADS_PER_STAGE = A_PER_W + B_PER_W + (SPARSE ? M_PER_W : 0);
    static_assert(LOADS_PER_STAGE <= 16 && (LOADS_PER_STAGE + 1) / 2 <= NMMA, "loads are paired with matrix instructions");

    // ---- accumulators -------------------------------------------------------------------------
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int li = lane & 31, kb = lane >> 5;
    const int arow0 = wm * WTM + li;   // + i * 32
    const int brow0 = wn * WTN + li;   // + j * 32

    // operand fragments of one sub-step
    struct Frags {
        std::conditional_t<D64, Frag16, Frag8> a[TM];   // D64: two 16-k halves
        Frag16 b[TN];   // dense kernel with 32-k stages uses b[j].u[0] only
    };
    // metadata words of the current / next stage (sparse only); FP8: word 2 i + sub of row block i
    int ix_cur[TM * IXW], ix_nxt[TM * IXW];

    auto read_frags = [&](int stage, int sub, Frags& f) {
        const uint8_t* base = smem + stage * L::kStage;
        const uint8_t* bB = base + L::kABytes + L::kMetaBytes;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if constexpr (D64) {
                f.a[i].u[0] = *reinterpret_cast<const uint4*>(base + swz8(arow0 + i * 32, 4 * sub + kb));
                f.a[i].u[1] = *reinterpret_cast<const uint4*>(base + swz8(arow0 + i * 32, 4 * sub + 2 + kb));
            } else {
                f.a[i].u = *reinterpret_cast<const uint4*>(base + swz4(arow0 + i * 32, 2 * (SPARSE ? kb : sub) + (SPARSE ? sub : kb)));
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int row = brow0 + j * 32;
            if constexpr (D64) {
                f.b[j].u[0] = *reinterpret_cast<const uint4*>(bB + swz8(row, 4 * sub + kb));
                f.b[j].u[1] = *reinterpret_cast<const uint4*>(bB + swz8(row, 4 * sub + 2 + kb));
            } else if constexpr (SPARSE) {
                f.b[j].u[0] = *reinterpret_cast<const uint4*>(bB + swz8(row, 2 * sub + kb));
                f.b[j].u[1] = *reinterpret_cast<const uint4*>(bB + swz8(row, 4 + 2 * sub + kb));
            } else {
                f.b[j].u[0] = *reinterpret_cast<const uint4*>(bB + swz4(row, 2 * sub + kb));
            }
        }
    };
    auto read_idx = [&](int stage, int (&ix)[TM * IXW]) {
        if constexpr (SPARSE) {
            const uint8_t* bM = smem + stage * L::kStage + L::kABytes;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if constexpr (FP8) {
                    const int2 w = *reinterpret_cast<const int2*>(bM + (arow0 + i * 32) * 16 + kb * 8);
                    ix[2 * i] = w.x;
                    ix[2 * i + 1] = w.y;
                } else {
                    ix[i] = *reinterpret_cast<const int*>(bM + (arow0 + i * 32) * 8 + kb * 4);
                }
            }
        }
    };
    // Read number n of the fragment set of (stage, SUB), in the order the matrix instructions need
    // them: metadata words (sub-step 0 only), A fragments, then B fragments column block by block.
    auto read_one = [&](int stage, auto sub_tag, Frags& f, int (&ix)[TM * IXW], auto n_tag) {
        constexpr int SUB = decltype(sub_tag)::value, n = decltype(n_tag)::value;
        constexpr int NI = (SPARSE && SUB == 0) ? TM : 0;     // metadata reads first
        const uint8_t* base = smem + stage * L::kStage;
        const uint8_t* bB = base + L::kABytes + L::kMetaBytes;
        if constexpr (n < NI) {
            if constexpr (FP8) {
                const int2 w = *reinterpret_cast<const int2*>(base + L::kABytes + (arow0 + n * 32) * 16 + kb * 8);
                ix[2 * n] = w.x;
                ix[2 * n + 1] = w.y;
            } else {
                ix[n] = *reinterpret_cast<const int*>(base + L::kABytes + (arow0 + n * 32) * 8 + kb * 4);
            }
        } else if constexpr (D64) {
            // 16-k half h of every fragment, first halves first (the order the instructions use them)
            constexpr int h = n / (TM + TN), m = n % (TM + TN);
            if constexpr (h < 2 && m < TM)
                f.a[m].u[h] = *reinterpret_cast<const uint4*>(base + swz8(arow0 + m * 32, 4 * SUB + 2 * h + kb));
            else if constexpr (h < 2)
                f.b[m - TM].u[h] = *reinterpret_cast<const uint4*>(bB + swz8(brow0 + (m - TM) * 32, 4 * SUB + 2 * h + kb));
        } else if constexpr (n < NI + TM) {
            constexpr int i = n - NI;
            f.a[i].u = *reinterpret_cast<const uint4*>(
                base + swz4(arow0 + i * 32, SPARSE ? 2 * kb + SUB : 2 * SUB + kb));
        } else if constexpr (SPARSE && n < NI + TM + 2 * TN) {
            constexpr int m = n - NI - TM, j = m / 2, h = m % 2;
            f.b[j].u[h] = *reinterpret_cast<const uint4*>(bB + swz8(brow0 + j * 32, 4 * h + 2 * SUB + kb));
        } else if constexpr (!SPARSE && n < TM + TN) {
            constexpr int j = n - TM;
            f.b[j].u[0] = *reinterpret_cast<const uint4*>(bB + swz4(brow0 + j * 32, 2 * SUB + kb));
        }
    };
    auto mma_one = [&](const Frags& f, const int (&ix)[TM * IXW], auto sub_tag, auto n_tag) {
        constexpr int SUB = decltype(sub_tag)::value;
        constexpr int n = decltype(n_tag)::value;
        constexpr int blk = n % (TM * TN), half = n / (TM * TN);   // half: 16-k half of a D64 sub-step
        constexpr int i = blk % TM, j = blk / TM;
        if constexpr (D64) {
            if constexpr (n < NMMA) {
                if constexpr (half == 0)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf16x8(f.a[i].v.lo), bf16x8(f.b[j].v.lo),
                                                                        acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf16x8(f.a[i].v.hi), bf16x8(f.b[j].v.hi),
                                                                        acc[i][j], 0, 0, 0);
            }
        } else {
            if constexpr (n < TM * TN) {
                if constexpr (FP8)
                    acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(f.a[i].q, f.b[j].q, acc[i][j],
                                                                             ix[2 * i + SUB], 0, 0);
                else if constexpr (SPARSE)
                    acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(f.a[i].v, f.b[j].v, acc[i][j],
                                                                          ix[i], 0, SUB);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i].v, bf16x8(f.b[j].v.lo),
                                                                        acc[i][j], 0, 0, 0);
            }
        }
    };
    // Matrix work of sub-step SUB on fragments f. After each matrix instruction the wave issues two
    // LDS reads of the NEXT fragment set (rstage, RSUB) into rf / rix (when READ), and one of the
    // ring-refill requests LO <= n < HI of stage kt_load into ring buffer buf. Spreading both keeps
    // the LDS command queue and the texture addresser from filling up, which would stall the wave
    // in front of its next matrix instruction.
    auto mma = [&](const Frags& f, const int (&ix)[TM * IXW], auto sub_tag, auto read_tag, auto rsub_tag,
                   int rstage, Frags& rf, int (&rix)[TM * IXW], auto lo_tag, auto hi_tag, int kt_load, int buf) {
        constexpr int LO = decltype(lo_tag)::value, HI = decltype(hi_tag)::value;
        constexpr bool READ = decltype(read_tag)::value;
        static_assert(NMMA <= 16 && HI - LO <= NMMA, "unrolled by hand up to 16 matrix instructions");
        static_assert(((SPARSE || D64) ? 2 * TM + 2 * TN : TM + TN) <= 2 * NMMA + 2, "two reads per matrix instruction must cover a fragment set");
#define RTL_MMA_STEP(N)                                                                       \
        mma_one(f, ix, sub_tag, std::integral_constant<int, N>{});                            \
        if constexpr (N < NMMA) {                                                             \
            if constexpr (READ) {                                                             \
                read_one(rstage, rsub_tag, rf, rix, std::integral_constant<int, 2 * N>{});     \
                read_one(rstage, rsub_tag, rf, rix, std::integral_constant<int, 2 * N + 1>{}); \
                if constexpr (N == NMMA - 1) {                                                \
                    read_one(rstage, rsub_tag, rf, rix, std::integral_constant<int, 2 * N + 2>{}); \
                    read_one(rstage, rsub_tag, rf, rix, std::integral_constant<int, 2 * N + 3>{}); \
                }                                                                             \
            }                                                                                 \
            if constexpr (LO + N < HI) gload_one(kt_load, buf, std::integral_constant<int, LO + N>{}); \
            __builtin_amdgcn_sched_barrier(0);                                                \
        }
        RTL_MMA_STEP(0) RTL_MMA_STEP(1) RTL_MMA_STEP(2) RTL_MMA_STEP(3)
        RTL_MMA_STEP(4) RTL_MMA_STEP(5) RTL_MMA_STEP(6) RTL_MMA_STEP(7)
        RTL_MMA_STEP(8) RTL_MMA_STEP(9) RTL_MMA_STEP(10) RTL_MMA_STEP(11)
        RTL_MMA_STEP(12) RTL_MMA_STEP(13) RTL_MMA_STEP(14) RTL_MMA_STEP(15)
#undef RTL_MMA_STEP
    };

    // ---- prologue: the whole ring in flight, stage 0 visible ----------------------------------
#pragma unroll
    for (int s = 0; s < STAGES; ++s)
        if (s < KT) gload(s, s);
    if (KT >= STAGES) wait_vmcnt_lgkm0<(STAGES - 1) * LOADS_PER_STAGE>();
    else wait_vmcnt_lgkm0<0>();
    __builtin_amdgcn_s_barrier();

    Frags f0, f1;
    read_frags(0, 0, f0);
    read_idx(0, ix_cur);
    wait_vmcnt_lgkm0<63>();            // fragments of sub-step 0 are in registers

    // One stage of the main loop. Schedule inside a stage kt:
    //   read fragments of sub-step 1 |
    //   matrix work of sub-step 0, interleaved with the second part of the requests of stage
    //   kt+STAGES-1 (its buffer, the one of stage kt-1, was released by the previous barrier) |
    //   wait: own reads of stage kt done, stage kt+1 landed | barrier |
    //   read fragments of stage kt+1 sub-step 0 |
    //   matrix work of sub-step 1, interleaved with the first part of the requests of stage
    //   kt+STAGES (into the buffer of stage kt, which nobody reads any more).
    // Every stage has about two stage times to arrive and the request stream never bursts.
    // PENDING: whole stages younger than kt+1 in flight at the wait (compile-time per phase).
    // requests issued in the second half. A ring of two has no buffer to spare for the early part:
    // all requests of stage kt+2 go out after the barrier of stage kt, one stage time ahead.
    constexpr int SPLIT = STAGES == 2 ? LOADS_PER_STAGE : (LOADS_PER_STAGE + 1) / 2;
    using c0 = std::integral_constant<int, 0>;
    using cS = std::integral_constant<int, SPLIT>;
    using cL = std::integral_constant<int, LOADS_PER_STAGE>;
    using T = std::true_type;
    using F = std::false_type;
    int cur = 0;                       // LDS buffer of stage kt
    auto stage_step = [&](int kt, auto load_a, auto load_b, auto has_next, auto pending) {
        constexpr bool LOAD_A = decltype(load_a)::value, LOAD_B = decltype(load_b)::value;
        constexpr bool HAS_NEXT = decltype(has_next)::value;
        constexpr int PENDING = decltype(pending)::value;
        const int nxt = cur + 1 == STAGES ? 0 : cur + 1;
        const int prv = cur == 0 ? STAGES - 1 : cur - 1;
        using s0 = std::integral_constant<int, 0>;
        using s1 = std::integral_constant<int, 1>;
        // sub-step 0 runs while the fragments of sub-step 1 are fetched
        if constexpr (LOAD_A) mma(f0, ix_cur, s0{}, T{}, s1{}, cur, f1, ix_nxt, cS{}, cL{}, kt + STAGES - 1, prv);
        else mma(f0, ix_cur, s0{}, T{}, s1{}, cur, f1, ix_nxt, c0{}, c0{}, 0, 0);
        wait_vmcnt_lgkm0<PENDING * LOADS_PER_STAGE>();
        __builtin_amdgcn_s_barrier();
        // sub-step 1 runs while the first fragments (and metadata) of stage kt+1 are fetched
        if constexpr (LOAD_B) mma(f1, ix_cur, s1{}, std::integral_constant<bool, HAS_NEXT>{}, s0{}, nxt, f0, ix_nxt, c0{}, cS{}, kt + STAGES, cur);
        else mma(f1, ix_cur, s1{}, std::integral_constant<bool, HAS_NEXT>{}, s0{}, nxt, f0, ix_nxt, c0{}, c0{}, 0, 0);
        if constexpr (SPARSE && HAS_NEXT) {
#pragma unroll
            for (int i = 0; i < TM * IXW; ++i) ix_cur[i] = ix_nxt[i];
        }
        cur = nxt;
    };
    static_assert(STAGES == 2 || STAGES == 3 || STAGES == 4, "ring depth");
    using P = std::integral_constant<int, STAGES - 2>;
    int kt = 0;
    if (KT > STAGES) {
        // stage 0 has no half-requested predecessor; from then on both halves carry requests
        stage_step(kt, F{}, T{}, T{}, P{});
        for (kt = 1; kt < KT - STAGES; ++kt) stage_step(kt, T{}, T{}, T{}, P{});
        // second part of the last stage; nothing new afterwards
        stage_step(kt, T{}, F{}, T{}, P{});
        ++kt;
    }
    // drain (and short K): stages kt+1 .. KT-1 are all requested; fewer remain in flight each step
    if constexpr (STAGES >= 4) {
        if (kt == KT - 4) { stage_step(kt, F{}, F{}, T{}, std::integral_constant<int, 2>{}); ++kt; }
    }
    if constexpr (STAGES >= 3) {
        if (kt == KT - 3) { stage_step(kt, F{}, F{}, T{}, std::integral_constant<int, 1>{}); ++kt; }
    }
    if (kt == KT - 2) { stage_step(kt, F{}, F{}, T{}, std::integral_constant<int, 0>{}); ++kt; }
    stage_step(kt, F{}, F{}, F{}, std::integral_constant<int, 0>{});

    const float ts = a.tensor_scale ? a.tensor_scale[0] : 1.0f;

    if constexpr (MODE == 1) {
        // ---- LoRA tail (Alg. 1: Y <- Y_s + Y_r, accumulated on chip) --------------------------
        // The ROW / TENSOR factors belong to the sparse product only, so they are applied to the
        // accumulators first. Then Y_r = T L_A^T, T = X L_B^T (bf16 [M,64]), is added by four dense
        // matrix-instruction steps over the rank; SMFMAC and MFMA 32x32 share one accumulator layout.
        if (a.row_scale || a.tensor_scale) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = min(m0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * kb + (r % 4), a.M - 1);
                    const float f = (a.row_scale ? a.row_scale[row] : 1.0f) * ts;
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[i][j][r] *= f;
                }
        }
        wait_vmcnt_lgkm0<0>();
        __builtin_amdgcn_s_barrier();          // the ring is free: reuse it for the two rank tiles
        constexpr int T_LOADS = BM * 128 / 1024, LA_LOADS = BN * 128 / 1024;   // rows of 64 bf16
        static_assert(T_LOADS % NW == 0 && LA_LOADS % NW == 0, "rank tiles must divide over the waves");
        static_assert((2 * BM + BN) * 128 <= L::kTotal, "rank tiles fit in the ring");
        const int64_t plane = a.t_plane;                // T is two bf16 planes: hi, lo
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int s = 0; s < T_LOADS / NW; ++s) {
                const int p = (wave * (T_LOADS / NW) + s) * 64 + lane;
                int row, c;
                unswz8(p, row, c);
                lds_dma16(a.T + h * plane + min(m0 + row, a.M - 1) * kLoraRank + c * 8,
                          lds0 + h * BM * 128 + (wave * (T_LOADS / NW) + s) * 1024);
            }
#pragma unroll
        for (int s = 0; s < LA_LOADS / NW; ++s) {
            const int p = (wave * (LA_LOADS / NW) + s) * 64 + lane;
            int row, c;
            unswz8(p, row, c);
            lds_dma16(a.LA + min(n0 + row, a.N - 1) * a.ldla + c * 8,
                      lds0 + 2 * BM * 128 + (wave * (LA_LOADS / NW) + s) * 1024);
        }
        wait_vmcnt_lgkm0<0>();
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int sub = 0; sub < kLoraRank / 16; ++sub) {
            Frag8 th[TM], tl[TM], lb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                th[i].u = *reinterpret_cast<const uint4*>(smem + swz8(arow0 + i * 32, 2 * sub + kb));
                tl[i].u = *reinterpret_cast<const uint4*>(smem + BM * 128 + swz8(arow0 + i * 32, 2 * sub + kb));
            }
#pragma unroll
            for (int j = 0; j < TN; ++j)
                lb[j].u = *reinterpret_cast<const uint4*>(smem + 2 * BM * 128 + swz8(brow0 + j * 32, 2 * sub + kb));
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tl[i].v, lb[j].v, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(th[i].v, lb[j].v, acc[i][j], 0, 0, 0);
                }
        }
    }

    // ---- epilogue: optional fp32 scales, bias, bf16 RNE, store --------------------------------
    auto finish = [&](float v, int64_t row, float bv) {
        if constexpr (MODE != 1) {
            if (a.row_scale) v *= a.row_scale[row];
            if (a.tensor_scale) v *= ts;
        }
        if (a.bias) v += bv;
        return (uint16_t)f32_to_bf16_rne(v);
    };
    const bool wide_ok = ((reinterpret_cast<uintptr_t>(a.Y) & 15) == 0) && (a.ldy % 8 == 0);
    if (wide_ok) {
        // The accumulator layout gives a lane one column and scattered rows, i.e. 2-byte stores.
        // Each wave therefore transposes its tile through a private LDS region (the ring is no
        // longer needed) and writes whole 16-byte row segments.
        constexpr int ROWB = L::kEpiRowBytes;
        wait_vmcnt_lgkm0<0>();
        __builtin_amdgcn_s_barrier();     // every wave is done reading the ring
        uint8_t* ep = smem + wave * (WTM * ROWB);
        // Two accumulator registers (rows r, r + 1 of one column) are converted by one packed
        // fp32 -> bf16 instruction (round to nearest even) and leave as two 16-bit LDS writes. The
        // plain case (no factors, no bias) is kept free of any other per-element work: with 128
        // elements per lane the epilogue is otherwise bound by its vector ALU work, not by stores.
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        // A lane holds rows rl, rl + 1 of ONE column; its neighbour (lane ^ 1) holds the same rows
        // of the next column. The pair swaps halves (one DPP move, one byte permute) so that the
        // even lane owns row rl and the odd lane row rl + 1 of BOTH columns: one 32-bit LDS write
        // per lane instead of two 16-bit ones.
        const bool odd = lane & 1;
        const uint32_t sel = odd ? 0x03020706u : 0x05040100u;   // v_perm_b32: bytes 0-3 = own, 4-7 = partner
        const int rsel = odd ? ROWB : 0;                        // odd lanes write the row below
        auto put2 = [&](float v0, float v1, int rl, int cl) {
            const f32x2 pv = {v0, v1};
            const uint32_t own = __builtin_bit_cast(uint32_t, __builtin_convertvector(pv, bf16x2));
            const uint32_t partner = (uint32_t)__builtin_amdgcn_mov_dpp((int)own, 0xB1, 0xF, 0xF, true);
            // even: (own.lo, partner.lo) = row rl, columns (cl, cl + 1)
            // odd : (partner.hi, own.hi) = row rl + 1, columns (cl - 1, cl)
            const uint32_t w = __builtin_amdgcn_perm(partner, own, sel);
            *reinterpret_cast<uint32_t*>(ep + rl * ROWB + rsel + (cl & ~1) * 2) = w;
        };
        const bool scaled = MODE != 1 && (a.row_scale || a.tensor_scale);
        if (!scaled && !a.bias) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; r += 2)
                        put2(acc[i][j][r], acc[i][j][r + 1], i * 32 + 8 * (r / 4) + 4 * kb + (r % 4), j * 32 + li);
        } else {
            // the factors of the lane's 16 rows per row block are fetched once, not once per column block,
            // four consecutive rows per load, all loads in flight together
            float bv[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t col = min(n0 + wn * WTN + j * 32 + li, a.N - 1);
                bv[j] = a.bias ? __uint_as_float((uint32_t)a.bias[col] << 16) : 0.f;
            }
            float f[TM][16];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {       // registers 4 q .. 4 q + 3 are four consecutive rows
                    const int64_t row = m0 + wm * WTM + i * 32 + 8 * q + 4 * kb;
                    if (!scaled || !a.row_scale) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) f[i][4 * q + e] = 1.0f;
                    } else if (row + 3 < a.M && (reinterpret_cast<uintptr_t>(a.row_scale + row) & 15) == 0) {
                        const float4 v = *reinterpret_cast<const float4*>(a.row_scale + row);
                        f[i][4 * q] = v.x; f[i][4 * q + 1] = v.y; f[i][4 * q + 2] = v.z; f[i][4 * q + 3] = v.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) f[i][4 * q + e] = a.row_scale[min(row + e, a.M - 1)];
                    }
                }
            const float tsf = scaled ? ts : 1.0f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; r += 2)
                        put2(acc[i][j][r] * (f[i][r] * tsf) + bv[j], acc[i][j][r + 1] * (f[i][r + 1] * tsf) + bv[j],
                             i * 32 + 8 * (r / 4) + 4 * kb + (r % 4), j * 32 + li);
        }
        // same wave reads back what it wrote: LDS operations of a wave complete in order
        constexpr int CPR = WTN / 8;               // 16-byte chunks per tile row
        constexpr int CHUNKS = WTM * CPR;
#pragma unroll
        for (int q0 = 0; q0 < CHUNKS; q0 += 64) {
            const int q = q0 + lane;
            if (q < CHUNKS) {
                const int rl = q / CPR, c = q % CPR;
                const int64_t row = m0 + wm * WTM + rl, col = n0 + wn * WTN + c * 8;
                if (row < a.M && col < a.N) {
                    const uint4 v = *reinterpret_cast<const uint4*>(ep + rl * ROWB + c * 16);
                    uint16_t* dst = a.Y + row * a.ldy + col;
                    if (col + 8 <= a.N) {
                        *reinterpret_cast<uint4*>(dst) = v;
                    } else {
                        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                        for (int e = 0; e < 8 && col + e < a.N; ++e)
                            dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                    }
                }
            }
        }
    } else {
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
                    a.Y[row * a.ldy + col] = finish(acc[i][j][r], row, bv);
                }
            }
        }
    }
}

// Two tile shapes in one launch (the "block-parallel" balancing of the method section's kernel
// paragraph, done with tile shapes instead of split contractions): rows [0, m_split) of the output
// are cut into 256 x BN body tiles, rows [m_split, M) into 256 x 128 tail tiles. Uniform tiles
// leave the chip's last round of workgroups mostly empty for many layer shapes (e.g. 792 tiles on
// 256 compute units: 3.09 rounds cost 4); smaller tiles at the end fill that round at 0.6 of a
// body tile's time. Every XCD works through its share of the body tiles first, then its share of
// the tail tiles (workgroups are dispatched in id order). tail_tiles == 0: a plain one-shape launch.
constexpr int kTailBN = 128;
template <bool SPARSE, int BN, int WAVES_M, int WAVES_N, int STAGES, int MODE = 0, bool FP8 = false, bool D64 = false>
__global__ __launch_bounds__(512) void gemm_mixed_kernel(const GemmArgs a) {
    static_assert(WAVES_M * WAVES_N == 8, "both tile shapes run with eight waves");
    const int xcd = (int)blockIdx.x % 8, local = (int)blockIdx.x / 8;
    const int nb = a.body_tiles, nt = a.tail_tiles;
    const int nb_x = nb / 8 + (xcd < nb % 8);
    if (local < nb_x) {
        GemmArgs b = a;
        if (nt > 0) b.M = a.m_split;
        gemm_tile<SPARSE, 256, BN, WAVES_M, WAVES_N, STAGES, MODE, FP8, D64>(b, xcd_share_start(nb, xcd) + local);
    } else {
        // the tail region as a problem of its own: same operands, shifted by m_split rows
        constexpr int ESZ = FP8 ? 1 : 2;
        GemmArgs t = a;
        t.M = a.M - a.m_split;
        t.A = static_cast<const uint8_t*>(a.A) + (SPARSE ? a.m_split * 64 : a.m_split * a.lda * ESZ);
        if constexpr (SPARSE) t.meta = a.meta + a.m_split * (FP8 ? 16 : 8);
        t.Y = a.Y + a.m_split * a.ldy;
        if (a.row_scale) t.row_scale = a.row_scale + a.m_split;
        if constexpr (MODE == 1) t.T = a.T + a.m_split * kLoraRank;
        const int idx = xcd_share_start(nb + nt, xcd) - xcd_share_start(nb, xcd) + (local - nb_x);
        gemm_tile<SPARSE, 256, kTailBN, 2, 4, STAGES, MODE, FP8, D64>(t, idx);
    }
}

// The tile loops need more dynamic LDS than the default limit of a launch: the limit is raised once
// per kernel by the prepare functions (called for every configuration from prepare_gemm_kernels, i.e.
// from rtl_init or from the first entry-point call on a device), never from a launch, so that launches
// consist of the kernel node only and can be recorded into a HIP graph.
template <bool SPARSE, int BN, int WAVES_M, int WAVES_N, int STAGES, int MODE = 0, bool FP8 = false, bool D64 = false>
struct Mixed {
    using LB = Smem<SPARSE, 256, BN, STAGES, WAVES_M, WAVES_N, FP8, D64>;
    using LT = Smem<SPARSE, 256, kTailBN, STAGES, 2, 4, FP8, D64>;
    static constexpr int kLds = LB::kTotal > LT::kTotal ? LB::kTotal : LT::kTotal;
    static hipError_t prepare() {
        auto kern = gemm_mixed_kernel<SPARSE, BN, WAVES_M, WAVES_N, STAGES, MODE, FP8, D64>;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    }
    // a.m_split, a.body_tiles and a.tail_tiles come from the planner
    static hipError_t launch(const GemmArgs& a, hipStream_t stream) {
        auto kern = gemm_mixed_kernel<SPARSE, BN, WAVES_M, WAVES_N, STAGES, MODE, FP8, D64>;
        hipLaunchKernelGGL(kern, dim3((unsigned)(a.body_tiles + a.tail_tiles)), dim3(512), kLds, stream, a);
        return hipGetLastError();
    }
};

}  // namespace

size_t gemm_workspace_bytes(bool, int64_t, int64_t, int64_t) { return 0; }

// ---- tile plan ---------------------------------------------------------------------------------
// A launch cuts rows [0, m_split) of the output into 256 x BN body tiles (BN = 256 or 192) and the
// remaining rows into 256 x 128 tail tiles. The main loop is bound by the rate at which a CU can pull
// operand stages out of L2, so a tile's time goes with its bytes per stage: 256x256 moves 51 KB,
// 256x192 43 KB (dense kernel: 64 and 56 KB per 64-k stage); a 256x128 tile was measured at 0.60 to
// 0.66 of a 256x256 tile. The plan is the (BN, m_split) whose simulated schedule ends first: per XCD
// (32 compute units, one workgroup each), workgroups in id order, each to the unit that frees first.
struct TilePlan {
    bool use_192;
    int64_t m_split;     // rows covered by body tiles (a multiple of 256, or M when there is no tail)
    int body_tiles, tail_tiles;
};

static double simulate_schedule(int64_t nb, int64_t nt, double cb, double ct) {
    double worst = 0.0;
    for (int x = 0; x < 8; ++x) {
        const int64_t tot = nb + nt;
        const int64_t nbx = nb / 8 + (x < nb % 8), cx = tot / 8 + (x < tot % 8);
        double unit[32] = {0};
        for (int64_t i = 0; i < cx; ++i) {
            int best = 0;
            for (int u = 1; u < 32; ++u)
                if (unit[u] < unit[best]) best = u;
            unit[best] += i < nbx ? cb : ct;
        }
        for (int u = 0; u < 32; ++u) worst = unit[u] > worst ? unit[u] : worst;
    }
    return worst;
}

static TilePlan make_plan(int64_t M, int64_t N, bool dense) {
    const double c256 = dense ? 64 : 51, c192 = dense ? 56 : 43, c128 = 0.64 * c256;
    const int64_t tm = (M + 255) / 256;
    const int64_t n256 = (N + 255) / 256, n192 = (N + 191) / 192, n128 = (N + kTailBN - 1) / kTailBN;
    if (tm * n128 > (int64_t)1 << 16) {
        // very large grids: many rounds, the last one no longer matters; pick the cheaper uniform shape
        // by rounds x bytes per stage and skip the simulation (it is linear in the number of tiles)
        const double r256 = (double)((tm * n256 + 255) / 256) * c256, r192 = (double)((tm * n192 + 255) / 256) * c192;
        return r192 < r256 ? TilePlan{true, M, (int)(tm * n192), 0} : TilePlan{false, M, (int)(tm * n256), 0};
    }
    TilePlan best{false, M, (int)(tm * n256), 0};
    double best_cost = simulate_schedule(tm * n256, 0, c256, c128);
    auto consider = [&](bool use_192, int64_t p) {
        if (p < 0 || p > tm) return;
        const int64_t nb = p * (use_192 ? n192 : n256), nt = (tm - p) * n128;
        double cost = simulate_schedule(nb, nt, use_192 ? c192 : c256, c128);
        if (nt > 0) cost *= 1.03;          // a tail has to pay for itself
        if (cost < best_cost - 1e-9) {
            best_cost = cost;
            best = TilePlan{use_192, p == tm ? M : p * 256, (int)nb, (int)nt};
        }
    };
    consider(true, tm);
    // body sizes that fill whole rounds of the chip, and a few panels around them
    for (int use_192 = 0; use_192 < 2; ++use_192) {
        const int64_t tn = use_192 ? n192 : n256;
        const int64_t rounds = tm * tn / 256;
        for (int64_t r = rounds; r >= rounds - 1 && r >= 0; --r)
            for (int64_t d = -2; d <= 1; ++d) consider(use_192 != 0, r * 256 / tn + d);
    }
    return best;
}

// Plans are cached per (M, N, kind): the simulation costs tens of microseconds on the host.
static TilePlan plan_for(int64_t M, int64_t N, bool dense) {
    struct Entry { int64_t M, N; bool dense; TilePlan plan; };
    static std::mutex mu;
    static std::vector<Entry> cache;
    std::lock_guard<std::mutex> lock(mu);
    for (const Entry& e : cache)
        if (e.M == M && e.N == N && e.dense == dense) return e.plan;
    const TilePlan p = make_plan(M, N, dense);
    if (cache.size() < 4096) cache.push_back(Entry{M, N, dense, p});
    return p;
}

void tile_plan(int64_t M, int64_t N, bool dense, int64_t out[4]) {
    const TilePlan p = plan_for(M, N, dense);
    out[0] = p.use_192 ? 192 : 256;
    out[1] = p.m_split;
    out[2] = p.body_tiles;
    out[3] = p.tail_tiles;
}

// Every configuration launch_gemm can pick.
hipError_t prepare_gemm_kernels() {
    hipError_t e = hipSuccess;
    auto run = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    run(Mixed<true, 192, 4, 2, 3, 0, true>::prepare());
    run(Mixed<true, 256, 2, 4, 3, 0, true>::prepare());
    run(Mixed<true, 192, 4, 2, 3, 1, true>::prepare());
    run(Mixed<true, 256, 2, 4, 3, 1, true>::prepare());
    run(Mixed<true, 192, 4, 2, 3, 1>::prepare());
    run(Mixed<true, 192, 4, 2, 3>::prepare());
    run(Mixed<true, 256, 2, 4, 3, 1>::prepare());
    run(Mixed<true, 256, 2, 4, 3>::prepare());
    run(Mixed<false, 192, 4, 2, 2, 0, false, true>::prepare());
    run(Mixed<false, 256, 2, 4, 2, 0, false, true>::prepare());
    return e;
}

hipError_t launch_gemm(bool sparse, const GemmArgs& a_in, hipStream_t stream) {
    GemmArgs a = a_in;
    const TilePlan plan = plan_for(a.M, a.N, !sparse);
    a.m_split = plan.m_split;
    a.body_tiles = plan.body_tiles;
    a.tail_tiles = plan.tail_tiles;
    a.rows_pad = kmajor_rows(a.M);
    a.t_plane = a.M * kLoraRank;
    if (sparse && a.fp8) {
        if (a.T != nullptr) {          // LoRA tail in bf16 on top of the FP8 product
            if (plan.use_192) return Mixed<true, 192, 4, 2, 3, 1, true>::launch(a, stream);
            return Mixed<true, 256, 2, 4, 3, 1, true>::launch(a, stream);
        }
        if (plan.use_192) return Mixed<true, 192, 4, 2, 3, 0, true>::launch(a, stream);
        return Mixed<true, 256, 2, 4, 3, 0, true>::launch(a, stream);
    }
    if (sparse) {
        const bool lora = a.T != nullptr;
        if (plan.use_192) {
            if (lora) return Mixed<true, 192, 4, 2, 3, 1>::launch(a, stream);
            return Mixed<true, 192, 4, 2, 3>::launch(a, stream);
        }
        if (lora) return Mixed<true, 256, 2, 4, 3, 1>::launch(a, stream);
        return Mixed<true, 256, 2, 4, 3>::launch(a, stream);
    }
    // dense: stages of 64 k (whole-line requests on the row-major operands), ring of two
    if (plan.use_192) return Mixed<false, 192, 4, 2, 2, 0, false, true>::launch(a, stream);
    return Mixed<false, 256, 2, 4, 2, 0, false, true>::launch(a, stream);
}

}  // namespace rtl
