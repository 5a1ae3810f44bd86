/*
 * rtlynx.h - C ABI of the MI355X (gfx950) RT-Lynx hot path:
 *            online 2:4 activation sparsification + activation-sparse x dense-weight linear.
 *
 * Problem statement (paper, Preliminary: Eq. linear_layer / Eq. sparse_activation; Alg. 1):
 *     Y = S(X) W^T ,  X in R^{M x K} (tokens x D_in),  W in R^{N x K} (D_out x D_in),
 *     S(X) = s * TopK_{2:4}(X),  s = sqrt(|X|^2 / (|TopK(X)|^2 + eps)).
 *
 * General conventions
 *  - Every tensor pointer is a DEVICE pointer owned by the caller. The library never allocates,
 *    frees or synchronises; all work is enqueued on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream) and the call returns immediately. Calls consist of kernel
 *    launches only (no memset or copy nodes), so they may be recorded into a HIP graph; call
 *    rtl_init() on the device once before the capture starts (the one-time set-up of a device,
 *    which otherwise happens inside the first call, is not a stream operation).
 *  - bf16 tensors are row-major with the contraction dimension K contiguous; `ld*` are row
 *    strides in ELEMENTS. Inputs are never modified; outputs are fully overwritten.
 *  - All argument checks happen before any launch, so error paths touch no memory:
 *      RTL_ERR_NULL       a required pointer is NULL
 *      RTL_ERR_SHAPE      negative size, K not a multiple of the required granule, ld < extent,
 *                         M, N or K above 2^30, or a row stride of a GEMM operand above 2^22 elements
 *      RTL_ERR_ALIGN      a pointer or a row stride breaks the stated alignment
 *      RTL_ERR_WORKSPACE  workspace NULL or smaller than the matching *_workspace() query
 *      RTL_ERR_ARG        an enum value out of range, or eps negative / not finite
 *      RTL_ERR_HIP        the HIP runtime reports no usable device, or refused the set-up or a
 *                         launch (message via hipGetLastError)
 *      RTL_ERR_ARCH       the current device is not a gfx950 GPU (checked once per device, after
 *                         the argument checks and before anything is launched)
 *  - M == 0 or N == 0 is RTL_OK with no launch.
 *  - Arithmetic: bf16 operands, fp32 accumulation, fp32 -> bf16 round-to-nearest-even on store.
 */
#ifndef RTLYNX_H
#define RTLYNX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RTL_OK = 0,
    RTL_ERR_NULL = 1,
    RTL_ERR_SHAPE = 2,
    RTL_ERR_ALIGN = 3,
    RTL_ERR_WORKSPACE = 4,
    RTL_ERR_ARG = 5,
    RTL_ERR_HIP = 6,
    RTL_ERR_ARCH = 7
} rtl_status;

/* One-time set-up of the CURRENT device: checks that it is a gfx950 GPU (else RTL_ERR_ARCH) and
 * readies every kernel of the library for launch. Idempotent and thread-safe; every other entry
 * point performs the same set-up by itself on its first call on a device, so calling rtl_init is
 * only required before HIP-graph capture. Not a stream operation. */
rtl_status rtl_init(void);

/* Scope of the two norms in the compensation factor s (method section, "Norm-Compensated
 * Sparsification", and Alg. 1 step 4). The method section states it for one 1x4 group (GROUP,
 * the default reading); Alg. 1 writes one scalar for the whole activation (TENSOR); ROW is the
 * per-token reading in between. NONE is the naive "Sparse Activation" baseline of the paper. */
typedef enum {
    RTL_COMP_NONE = 0,
    RTL_COMP_GROUP = 1,
    RTL_COMP_ROW = 2,
    RTL_COMP_TENSOR = 3
} rtl_comp;

/* ---------------------------------------------------------------------------------------------
 * rtl_sparsify_pack - Alg. 1 steps "X~ <- TopK(X)" and "s, S(X) <- s X~", followed by the
 * compression into the operand format of the paper's App. A (kept values + 2-bit positions).
 *
 *   X      [M, K] bf16, row stride ldx (>= K). 16-byte aligned base, ldx % 8 == 0, K % 8 == 0.
 *   comp   scope of s (see rtl_comp); eps is the stabiliser inside the square root (paper: 1e-8).
 *   vals   [M, K/2] bf16, dense rows (stride K/2), 16-byte aligned. For every aligned group of four
 *          g = k/4 the two entries of largest magnitude, in ascending position order. Magnitude
 *          is compared on the bf16 bit pattern without its sign bit; ties keep the lower index.
 *          comp == GROUP: the stored values are bf16_rne(s_g * x) with
 *              s_g = sqrtf((((x0^2+x1^2)+x2^2)+x3^2) / ((ka^2+kb^2)+eps))   (fp32, this order);
 *          otherwise the stored values are the untouched inputs.
 *   meta   [M, K/8] bytes, 4-byte aligned (8-byte aligned if it is to be handed to
 *          rtl_packed_linear). Group g of a row sits in nibble (g & 1) of byte g/2;
 *          nibble = pos0 | pos1 << 2 with pos0 < pos1 the kept positions inside the group.
 *   scale  fp32 output, required for ROW ([M]) and TENSOR ([1]), ignored otherwise (may be NULL).
 *          The two norms are accumulated in fp32: a row whose sum of squares exceeds the fp32
 *          range (|x| around 1e17 and above) yields a NaN factor.
 *          s is constant along the contraction for these scopes, so it is handed out for an fp32
 *          multiplication of the GEMM result instead of being rounded into `vals`.
 *   workspace  device scratch of rtl_sparsify_pack_workspace(M, K, comp) bytes (0 unless TENSOR),
 *          256-byte aligned; contents are overwritten. May be NULL when the query returns 0.
 * ------------------------------------------------------------------------------------------- */
size_t rtl_sparsify_pack_workspace(int64_t M, int64_t K, rtl_comp comp);
rtl_status rtl_sparsify_pack(const void* X, int64_t M, int64_t K, int64_t ldx,
                             rtl_comp comp, float eps,
                             void* vals, void* meta, float* scale,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * rtl_packed_linear - Alg. 1 step "Y_s <- S(X) W^T" on an already compressed activation
 * (App. A: the 2-bit positions pick the matching rows of the dense operand), executed on the
 * structured-sparse matrix instructions; optional "+ b" of Alg. 2.
 *
 *   vals, meta  as written by rtl_sparsify_pack for an [M, K] activation (dense rows of K/2 values
 *          and K/8 bytes). K % 64 == 0; vals 16-byte aligned, meta 8-byte aligned.
 *   row_scale   NULL, or fp32 [M]: Y[m, :] is multiplied by row_scale[m] in fp32 before the bias.
 *   tensor_scale NULL, or fp32 [1]: Y is multiplied by tensor_scale[0] likewise.
 *   W      [N, K] bf16, row stride ldw (>= K), 16-byte aligned base, ldw % 8 == 0.
 *   bias   NULL or bf16 [N].
 *   Y      [M, N] bf16, row stride ldy (>= N). 2-byte aligned is enough.
 *   workspace  rtl_packed_linear_workspace(M, N, K) bytes (never 0 for a non-empty problem),
 *          256-byte aligned: receives the k-major copy of the compressed operand that the tile
 *          loop streams (a small re-layout kernel runs first; rtl_sparse_linear has its pack
 *          sweep write that layout directly and skips this step).
 * ------------------------------------------------------------------------------------------- */
size_t rtl_packed_linear_workspace(int64_t M, int64_t N, int64_t K);
rtl_status rtl_packed_linear(const void* vals, const void* meta,
                             const float* row_scale, const float* tensor_scale,
                             const void* W, const void* bias, void* Y,
                             int64_t M, int64_t N, int64_t K, int64_t ldw, int64_t ldy,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * rtl_sparse_linear - the whole of Alg. 1 without its LoRA branch:
 *     Y = compensate(sparsify_2:4(X)) W^T (+ b).
 * Equivalent to rtl_sparsify_pack into the workspace followed by rtl_packed_linear.
 *
 *   X [M,K] bf16 (ldx), W [N,K] bf16 (ldw), bias NULL or bf16 [N], Y [M,N] bf16 (ldy).
 *   K % 64 == 0; X and W 16-byte aligned with ldx % 8 == 0 and ldw % 8 == 0.
 *   workspace  rtl_sparse_linear_workspace(M, N, K, comp) bytes, 256-byte aligned.
 * ------------------------------------------------------------------------------------------- */
size_t rtl_sparse_linear_workspace(int64_t M, int64_t N, int64_t K, rtl_comp comp);
rtl_status rtl_sparse_linear(const void* X, const void* W, const void* bias, void* Y,
                             int64_t M, int64_t N, int64_t K,
                             int64_t ldx, int64_t ldw, int64_t ldy,
                             rtl_comp comp, float eps,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * rtl_sparse_linear_static - rtl_sparse_linear for callers that cannot allocate device memory or
 * pass a workspace: code running under HIP-graph capture, tight serving loops, harnesses that
 * forbid hipMalloc. Same arguments, checks, kernels and results as rtl_sparse_linear, but the
 * scratch (compressed operand, factors) lives in a fixed device array inside the library of
 * RTL_STATIC_SCRATCH_BYTES bytes, which every GPU the library is used on holds until the process
 * ends. The call allocates and frees nothing.
 *   - Problems whose rtl_sparse_linear_workspace(M, N, K, comp) exceeds RTL_STATIC_SCRATCH_BYTES
 *     are refused with RTL_ERR_WORKSPACE (64 MiB covers every layer shape with M <= 4608 and
 *     K <= 12288, e.g. the [4096, 12288] x [3072, 12288] MLP-down layer).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race on it; serialise them, or use rtl_sparse_linear with separate
 *     workspaces. Nothing in the array needs to survive between calls.
 *   - The first call on a device (or rtl_init) looks up the array's device address; do that
 *     before a graph capture starts.
 * ------------------------------------------------------------------------------------------- */
#define RTL_STATIC_SCRATCH_BYTES (64u * 1024u * 1024u)
rtl_status rtl_sparse_linear_static(const void* X, const void* W, const void* bias, void* Y,
                                    int64_t M, int64_t N, int64_t K,
                                    int64_t ldx, int64_t ldw, int64_t ldy,
                                    rtl_comp comp, float eps, void* stream);

/* ---------------------------------------------------------------------------------------------
 * rtl_sparse_lora_linear - the whole of Alg. 1 including its LoRA residual (Eq. sparse+lora):
 *     Y = compensate(sparsify_2:4(X)) W^T + X (L_A L_B)^T (+ b).
 * The residual is evaluated as (X L_B^T) L_A^T: a skinny product T = X L_B^T ([M,R], kept in the
 * workspace as a bf16 hi/lo pair) and a rank-R update added to the sparse product's fp32 accumulators inside the
 * GEMM kernel, so Y_r is never materialised (method section, "CUDA Kernel Optimization", second item).
 *
 *   LA [N,R] bf16, row stride ldla (>= R); LB [R,K] bf16, row stride ldlb (>= K); both 16-byte
 *   aligned with ldla % 8 == 0 and ldlb % 8 == 0. R must be 64 (the paper's rank), else RTL_ERR_SHAPE.
 *   The compensation factors of ROW / TENSOR scope multiply the sparse product only.
 *   Everything else as for rtl_sparse_linear.
 *   workspace  rtl_sparse_lora_linear_workspace(M, N, K, R, comp) bytes, 256-byte aligned.
 * ------------------------------------------------------------------------------------------- */
size_t rtl_sparse_lora_linear_workspace(int64_t M, int64_t N, int64_t K, int64_t R, rtl_comp comp);
rtl_status rtl_sparse_lora_linear(const void* X, const void* W, const void* LA, const void* LB,
                                  const void* bias, void* Y,
                                  int64_t M, int64_t N, int64_t K, int64_t R,
                                  int64_t ldx, int64_t ldw, int64_t ldla, int64_t ldlb, int64_t ldy,
                                  rtl_comp comp, float eps,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * rtl_dense_linear - Eq. (linear_layer), Y = X W^T (+ b), on the dense matrix instructions.
 * The denominator of every speedup the paper reports ("GEMM" column of its kernel tables).
 * Same layouts and alignment rules as rtl_sparse_linear; K % 64 == 0.
 *   workspace  rtl_dense_linear_workspace(M, N, K) bytes, 256-byte aligned (may be 0).
 * ------------------------------------------------------------------------------------------- */
size_t rtl_dense_linear_workspace(int64_t M, int64_t N, int64_t K);
rtl_status rtl_dense_linear(const void* X, const void* W, const void* bias, void* Y,
                            int64_t M, int64_t N, int64_t K,
                            int64_t ldx, int64_t ldw, int64_t ldy,
                            void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * FP8 composition (implementation details, "orthogonal validation with FP8 quantization": symmetric
 * FP8 quantisation of the activations, weights cast directly to FP8; 2:4 FP8 is one of the formats
 * of the App. A table). FP8 is E4M3 without infinities (bias 7, largest finite 448, S.1111.111 =
 * NaN); every conversion is round-to-nearest-even and saturating (|v| >= 448 and +-inf give +-448,
 * NaN gives 0x7F).
 *
 * rtl_quantize_fp8 - the direct cast of the weights: Wq[r, c] = e4m3(W[r, c]).
 *   W [rows, cols] bf16 (ld), 16-byte aligned, ld % 8 == 0; Wq [rows, cols] bytes (ldq), 8-byte
 *   aligned, ldq % 8 == 0; cols % 8 == 0.
 *
 * rtl_sparsify_pack_fp8 - rtl_sparsify_pack with FP8 kept values. Selection, metadata, `scale`
 *   and the workspace are exactly those of rtl_sparsify_pack (they look at the bf16 input only).
 *   x_scale  fp32 [1] on the device, > 0: the symmetric activation scale (one per tensor, supplied
 *            by the caller, e.g. calibrated max|S(X)| / 448).
 *   vals     [M, K/2] bytes, 4-byte aligned: e4m3((s_g * x) * (1 / x_scale[0])) for GROUP (s_g as in
 *            rtl_sparsify_pack, both products in fp32, one rounding), e4m3(x * (1 / x_scale[0])) otherwise.
 *
 * rtl_sparse_linear_fp8 - W8A8 + 2:4 activation sparsity:
 *     Y = f * (Q Wq^T) (+ b),  Q = the quantised S(X) above,  f = x_scale[0] (times the ROW / TENSOR factor),
 *   on the FP8 structured-sparse matrix instruction, fp32 accumulation, bf16 output. (Inside one
 *   instruction the hardware aligns the 32 products to the largest exponent among them with about
 *   14 fractional bits, truncating; between instructions the accumulation is plain fp32.)
 *   X [M,K] bf16 (ldx) as for rtl_sparse_linear; Wq [N,K] E4M3 bytes (ldw >= K, ldw % 16 == 0,
 *   16-byte aligned); K % 128 == 0; bias NULL or bf16 [N]; Y [M,N] bf16 (ldy).
 *   workspace  rtl_sparse_linear_fp8_workspace(M, N, K, comp) bytes, 256-byte aligned.
 * ------------------------------------------------------------------------------------------- */
rtl_status rtl_quantize_fp8(const void* W, int64_t rows, int64_t cols, int64_t ld,
                            void* Wq, int64_t ldq, void* stream);
size_t rtl_sparsify_pack_fp8_workspace(int64_t M, int64_t K, rtl_comp comp);
rtl_status rtl_sparsify_pack_fp8(const void* X, int64_t M, int64_t K, int64_t ldx,
                                 rtl_comp comp, float eps, const float* x_scale,
                                 void* vals, void* meta, float* scale,
                                 void* workspace, size_t workspace_bytes, void* stream);
size_t rtl_sparse_linear_fp8_workspace(int64_t M, int64_t N, int64_t K, rtl_comp comp);
rtl_status rtl_sparse_linear_fp8(const void* X, const void* Wq, const float* x_scale,
                                 const void* bias, void* Y,
                                 int64_t M, int64_t N, int64_t K,
                                 int64_t ldx, int64_t ldw, int64_t ldy,
                                 rtl_comp comp, float eps,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* rtl_sparse_lora_linear_fp8 - the whole of Alg. 1 on FP8 operands (the "W8A8 + RT-Lynx" rows of the
 * orthogonality tables): Y = f * (Q Wq^T) + X (L_A L_B)^T (+ b), the sparse product as in
 * rtl_sparse_linear_fp8, the LoRA residual as in rtl_sparse_lora_linear: it looks at the bf16 input,
 * its factors stay bf16, and it is added in fp32 to the dequantised sparse product before the single
 * bf16 rounding of Y. One sweep over X writes the FP8 compressed operand and forms X L_B^T.
 *   Arguments as for rtl_sparse_linear_fp8 plus LA, LB, R, ldla, ldlb as for rtl_sparse_lora_linear.
 *   workspace  rtl_sparse_lora_linear_fp8_workspace(M, N, K, R, comp) bytes, 256-byte aligned. */
size_t rtl_sparse_lora_linear_fp8_workspace(int64_t M, int64_t N, int64_t K, int64_t R, rtl_comp comp);
rtl_status rtl_sparse_lora_linear_fp8(const void* X, const void* Wq, const float* x_scale,
                                      const void* LA, const void* LB, const void* bias, void* Y,
                                      int64_t M, int64_t N, int64_t K, int64_t R,
                                      int64_t ldx, int64_t ldw, int64_t ldla, int64_t ldlb, int64_t ldy,
                                      rtl_comp comp, float eps,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * rtl_diag_matrix_rate - diagnostic, not a step of the method: measures the issue rate of the matrix
 * instruction the linears are built on with nothing else running (operands in registers), so that a
 * benchmark can quote the tile loops against a ceiling measured on the device at hand.
 *   kind      0: dense 32x32x16 bf16 instruction (Eq. linear_layer path), 1: structured-sparse
 *             32x32x32 bf16 instruction (Alg. 1 "Y_s <- S(X) W^T" path).
 *   operands  device, 3072 bytes, 16-byte aligned: bf16 bit patterns fed to every wave (all equal
 *             values give the full-clock rate, random values the rate under real switching activity).
 *   iters     1 .. 2^24; every wave issues 4 * iters instructions. blocks: 1 .. 65536 workgroups of
 *             four waves (1024 = one wave per SIMD four times over on 256 compute units).
 *   clocks    device uint64[2], written by the first wave: [0] shader-clock cycles, [1] ticks of the
 *             constant 100 MHz counter between its first and last instruction.
 *   sink      device float[1]; practically never written (keeps the arithmetic alive).
 * Work per launch: blocks * 4 * 4 * iters instructions of 2*32*32*16 executed flops each.
 * ------------------------------------------------------------------------------------------- */
rtl_status rtl_diag_matrix_rate(int kind, const void* operands, int64_t iters, int blocks,
                                uint64_t* clocks, float* sink, void* stream);

/* rtl_diag_fill_rate - diagnostic, not a step of the method: measures how fast the compute units can
 * stream operands from the L2s into LDS with the direct-to-LDS loads the tile loops are built on, with
 * nothing else running; the stage rate of a tile loop cannot exceed it.
 *   region    device, region_bytes bytes (>= 1 MiB, a multiple of 8192, 16-byte aligned), only read.
 *             A few MiB stay resident in the L2s, up to ~200 MiB in the memory-side cache.
 *   iters     1 .. 2^24; blocks 1 .. 65536 workgroups of eight waves (256 = one per compute unit).
 *             Bytes moved per launch: blocks * 8 * iters * 8192.
 *   clocks    device uint64[2] as for rtl_diag_matrix_rate; sink device float[1], never written. */
rtl_status rtl_diag_fill_rate(const void* region, size_t region_bytes, int64_t iters, int blocks,
                              uint64_t* clocks, float* sink, void* stream);

/* rtl_diag_pack_sweep - diagnostic: the online sparsification sweep (Alg. 1 "X~ <- TopK(X)",
 * "S(X) <- s X~", App. A operand format) exactly as rtl_sparse_linear launches it - same kernel, same
 * compressed operand into the head of the same workspace layout - without the tile loop that follows,
 * so that the two halves of a call can be timed separately (the benchmark's "Sparse-Cost" share).
 *   X, M, K, ldx, comp, eps   as for rtl_sparse_linear (K % 64 == 0).
 *   workspace   device, 256-byte aligned, at least rtl_sparse_linear_workspace(M, 1, K, comp) bytes. */
rtl_status rtl_diag_pack_sweep(const void* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp, float eps,
                               void* workspace, size_t workspace_bytes, void* stream);

/* rtl_diag_tile_plan - diagnostic (host arithmetic only, nothing is launched): how the linears cut an
 * [M, N] output into workgroup tiles. plan (HOST pointer, int64[4]) receives {body tile width (256 or
 * 192), rows covered by 256-row body tiles, number of body tiles, number of 256 x 128 tail tiles}.
 * dense != 0 asks for the plan of rtl_dense_linear, else of the sparse linears. */
rtl_status rtl_diag_tile_plan(int64_t M, int64_t N, int dense, int64_t* plan);

/* Human-readable name of a status code; never NULL. */
const char* rtl_status_str(rtl_status s);
/* Library version string, e.g. "rtlynx-gfx950 0.1". */
const char* rtl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RTLYNX_H */
