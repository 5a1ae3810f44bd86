// Internal declarations shared by the HIP translation units of librtlynx (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "rtlynx.h"

namespace rtl {

// ---- sparsify + pack (pack.hip) -------------------------------------------------------------
// Launches the select/compensate/compress sweep. `rowsums` ([M][2] fp32) is only touched for
// RTL_COMP_TENSOR. Returns the HIP launch status.
hipError_t launch_sparsify_pack(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                float eps, uint16_t* vals, uint8_t* meta, float* scale,
                                float* rowsums, hipStream_t stream);

// ---- GEMMs (gemm.hip) -----------------------------------------------------------------------
struct GemmArgs {
    const uint16_t* A;      // dense: X [M,K] (lda); sparse: vals [M,K/2] (lda = K/2)
    const uint8_t* meta;    // sparse only: [M,K/8]
    const uint16_t* W;      // [N,K] (ldw)
    const uint16_t* bias;   // nullable [N]
    const float* row_scale; // nullable [M]
    const float* tensor_scale; // nullable [1]
    uint16_t* Y;            // [M,N] (ldy)
    float* partials;        // workspace for split contraction (may be null when unused)
    int64_t M, N, K, lda, ldw, ldy;
};
size_t gemm_workspace_bytes(bool sparse, int64_t M, int64_t N, int64_t K);
hipError_t launch_gemm(bool sparse, const GemmArgs& a, hipStream_t stream);

}  // namespace rtl
