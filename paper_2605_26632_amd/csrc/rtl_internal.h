// Internal declarations shared by the HIP translation units of librtlynx (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "rtlynx.h"

namespace rtl {

// ---- metadata layouts -----------------------------------------------------------------------
// canonical (ABI): meta[M][K/8] bytes, row-major.
// k-major (what the GEMM streams): for every block of 64 dense k, one 8-byte record per row,
// records of a block contiguous over rows: km[(k / 64) * Mpad + m] (8 bytes), Mpad = kmajor_rows(M).
// A 256-row tile of one block is then a single contiguous 2 KiB run instead of 256 scattered
// 8-byte pieces, which keeps the L2 -> CU traffic of the GEMM at its algorithmic size.
// With FP8 kept values (one stage = 128 dense k) the records are 16 bytes per row and 128-k block:
// km[(k / 128) * Mpad + m] (16 bytes). Either way a row contributes K / 8 bytes, so the buffer size
// is the same.
// The kept values the GEMM streams use the same blocking: 64 bytes per row and block (32 bf16 of a
// 64-k block, or 64 FP8 codes of a 128-k block), vals_km[(block * Mpad + m) * 64]. A 256-row tile of
// one stage is then one contiguous 16 KiB run of whole 128-byte lines; in the row-major form every
// row contributes a 64-byte half line per stage and the L2 sees twice the requests for it.
inline int64_t kmajor_rows(int64_t M) { return (M + 255) / 256 * 256; }
inline size_t kmajor_bytes(int64_t M, int64_t K) { return (size_t)(K / 64) * (size_t)kmajor_rows(M) * 8; }
// bytes of the k-major value buffer; val_bytes = 2 (bf16) or 1 (FP8)
inline size_t kmajor_val_bytes(int64_t M, int64_t K, size_t val_bytes) {
    return (size_t)kmajor_rows(M) * (size_t)(K / 2) * val_bytes;
}

// ---- sparsify + pack (pack.hip) -------------------------------------------------------------
// Launches the select/compensate/compress sweep. The canonical outputs (`vals`, `meta`) and the
// k-major ones (`vals_km`, `meta_km`, need K % 64 == 0) are each optional; `rowsums` ([M][2] fp32)
// is only touched for RTL_COMP_TENSOR. Returns the HIP launch status.
hipError_t launch_sparsify_pack(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                float eps, uint16_t* vals, uint8_t* meta, uint8_t* vals_km,
                                uint8_t* meta_km, float* scale, float* rowsums, hipStream_t stream);
// FP8 form (implementation details, "orthogonal validation with FP8 quantization"): kept values
// leave as E4M3 codes of (s * x) / x_scale[0] (vals8 [M,K/2] bytes); `meta_km` then uses the 16-byte
// records and `vals_km` 128-k blocks (need K % 128 == 0). `fused_scale` (nullable, [1]) receives
// x_scale[0] times the TENSOR factor (TENSOR scope only), the single multiplier the GEMM epilogue
// then needs.
hipError_t launch_sparsify_pack_fp8(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                    float eps, const float* x_scale, uint8_t* vals8, uint8_t* meta,
                                    uint8_t* vals_km, uint8_t* meta_km, float* scale, float* rowsums,
                                    float* fused_scale, hipStream_t stream);
// Direct cast of a bf16 matrix to E4M3 codes (round to nearest even, saturating), cols % 8 == 0.
hipError_t launch_quantize_fp8(const uint16_t* W, int64_t rows, int64_t cols, int64_t ld, uint8_t* Wq,
                               int64_t ldq, hipStream_t stream);
// canonical -> k-major copy of the compressed bf16 operand (values and metadata, K % 64 == 0).
hipError_t launch_operand_to_kmajor(const uint16_t* vals, const uint8_t* meta, int64_t M, int64_t K,
                                    uint8_t* vals_km, uint8_t* meta_km, hipStream_t stream);

// ---- GEMMs (gemm.hip) -----------------------------------------------------------------------
struct GemmArgs {
    // A and W are bf16 unless fp8 is set (sparse only): then both hold one-byte E4M3 codes and
    // lda / ldw still count elements.
    const void* A;          // dense: X [M,K] (lda); sparse: k-major kept values (lda unused)
    const uint8_t* meta;    // sparse only: k-major records, kmajor_rows(M) rows per block
    const void* W;          // [N,K] (ldw)
    const uint16_t* bias;   // nullable [N]
    const float* row_scale; // nullable [M]
    const float* tensor_scale; // nullable [1]
    uint16_t* Y;            // [M,N] (ldy)
    int64_t M, N, K, lda, ldw, ldy;
    // LoRA tail of the sparse kernel (Alg. 1 "Y_r <- X (L_A L_B)^T" as (X L_B^T) L_A^T):
    const uint16_t* T;      // nullable: X L_B^T as two bf16 planes (hi, lo), [2][M,64]
    const uint16_t* LA;     // L_A bf16 [N,64] (ldla)
    int64_t ldla;
    // filled in by launch_gemm (tile plan and strides of the whole problem):
    int64_t rows_pad;       // sparse: rows per k block of the k-major operand, kmajor_rows(M of the whole activation)
    int64_t t_plane;        // LoRA: elements between the hi and lo planes of T (M of the whole activation * 64)
    int64_t m_split;        // rows [0, m_split) are cut into body tiles, rows [m_split, M) into 256 x 128 tail tiles
    int body_tiles, tail_tiles;
    bool fp8;               // sparse only: E4M3 operands, K % 128 == 0, 16-byte metadata records
};
size_t gemm_workspace_bytes(bool sparse, int64_t M, int64_t N, int64_t K);
// One-time set-up per device (rtl_init, or the first entry-point call): raises the dynamic-LDS limit
// of every tile-loop kernel and makes the runtime load both code objects, so that later launches
// are plain kernel nodes (HIP-graph capture needs no warm-up call).
hipError_t prepare_gemm_kernels();
hipError_t prepare_pack_kernels();
hipError_t launch_gemm(bool sparse, const GemmArgs& a, hipStream_t stream);
// The tile plan launch_gemm uses for an [M, N] output: out = {body tile width (256 or 192), rows covered
// by body tiles, number of body tiles, number of 256 x 128 tail tiles}. Host arithmetic only.
void tile_plan(int64_t M, int64_t N, bool dense, int64_t out[4]);

constexpr int kLoraRank = 64;

// One pass over X for the LoRA branch (pack_lora.hip): the sweep writes the k-major compressed operand (as
// launch_sparsify_pack does) and, per K range, an fp32 partial plane of T = X L_B^T and (ROW / TENSOR) the
// row sums of squares, into `scratch` (pack_down_scratch_bytes(M, K) bytes); a second small kernel adds the
// ranges up in order into the two bf16 planes of T ([2][M][64]: hi, lo), the ROW factors `scale` [M] or
// the TENSOR row sums `rowsums` [M][2], from which launch_tensor_scale then forms scale[0].
size_t pack_down_scratch_bytes(int64_t M, int64_t K);
hipError_t prepare_pack_lora_kernels();
hipError_t launch_pack_down(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp, float eps,
                            const uint16_t* LB, int64_t ldlb, uint8_t* vals_km, uint8_t* meta_km, float* scratch,
                            uint16_t* T, float* scale, float* rowsums, hipStream_t stream,
                            const float* x_scale = nullptr, float* fused_scale = nullptr);
// (x_scale set: FP8 form: kept values as E4M3 codes of (s x) / x_scale[0] in the FP8 k-major layout, K % 128 == 0;
//  fused_scale [1] then receives x_scale[0] times the TENSOR factor, TENSOR scope only.)
// TENSOR scope: the single factor from the per-row sums [M][2] (fixed order, fp64), into scale[0]; `fused`
// (nullable) receives scale[0] * mul[0].
hipError_t launch_tensor_scale(const float* rowsums, int64_t M, float eps, float* scale, hipStream_t stream,
                               const float* mul = nullptr, float* fused = nullptr);

// ---- diagnostics (diag.hip) -------------------------------------------------------------------
// Issue-rate probe: `blocks` workgroups of four waves, each wave issuing 4 * iters matrix
// instructions (kind 0: dense 32x32x16 bf16, kind 1: structured-sparse 32x32x32 bf16) on register
// operands read once from `operands` (3072 bytes). clocks[0..1]: shader cycles and 100 MHz ticks
// of the first wave.
hipError_t launch_matrix_rate(int kind, const void* operands, int64_t iters, int blocks,
                              unsigned long long* clocks, float* sink, hipStream_t stream);
// Fill-rate probe: `blocks` workgroups of eight waves stream `region` into LDS with direct-to-LDS
// loads, 8 KiB per wave and iteration (bytes moved: blocks * 8 * iters * 8192). clocks as above.
hipError_t prepare_diag_kernels();
hipError_t launch_fill_rate(const void* region, size_t region_bytes, int64_t iters, int blocks,
                            unsigned long long* clocks, float* sink, hipStream_t stream);

}  // namespace rtl
