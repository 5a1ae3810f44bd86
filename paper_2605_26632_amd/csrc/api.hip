// C ABI of librtlynx: argument validation and dispatch. Every check precedes any launch, so the
// error paths can be exercised on a host without a GPU.
#include <cmath>
#include <cstring>
#include <mutex>
#include "rtl_internal.h"

namespace {

// Scratch of rtl_sparse_linear_static, the entry point for callers that cannot allocate: a
// fixed array in device memory that every GPU the library runs on holds until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; the device address it
// yields (one per device) is what kernels and launches receive.
static __device__ __align__(256) unsigned char scratch[RTL_STATIC_SCRATCH_BYTES];

// Per-device set-up state. A device is prepared once: its architecture is checked (the kernels
// exist for gfx950 only), the kernels are readied for launch (rtl::prepare_*_kernels) and the
// address of this device's copy of `scratch` is looked up.
constexpr int kMaxDevices = 64;
struct DeviceState {
    int state;            // 0 = not looked at yet, 1 = ready, -1 = not a gfx950 device
    void* scratch_ptr;    // device address of `scratch` on this device (valid when state == 1)
};
DeviceState g_dev[kMaxDevices];
std::mutex g_dev_mutex;

// Status of the current device: RTL_OK once prepared, RTL_ERR_ARCH for another architecture,
// RTL_ERR_HIP when the runtime has no usable device.
rtl_status device_ready(void** scratch_out = nullptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RTL_ERR_HIP;
    DeviceState& d = g_dev[dev];
    if (d.state == 0) {
        std::lock_guard<std::mutex> lock(g_dev_mutex);
        if (d.state == 0) {
            hipDeviceProp_t prop;
            if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return RTL_ERR_HIP;
            if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
                d.state = -1;
            } else {
                if (rtl::prepare_pack_kernels() != hipSuccess || rtl::prepare_gemm_kernels() != hipSuccess ||
                    rtl::prepare_pack_lora_kernels() != hipSuccess || rtl::prepare_diag_kernels() != hipSuccess)
                    return RTL_ERR_HIP;
                void* ptr = nullptr;
                if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return RTL_ERR_HIP;
                d.scratch_ptr = ptr;
                d.state = 1;
            }
        }
    }
    if (d.state == 1 && scratch_out) *scratch_out = d.scratch_ptr;
    return d.state == 1 ? RTL_OK : RTL_ERR_ARCH;
}
#define RTL_REQUIRE_DEVICE()                          \
    do {                                              \
        const rtl_status ready_ = device_ready();     \
        if (ready_ != RTL_OK) return ready_;          \
    } while (0)

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool comp_ok(rtl_comp c) { return c >= RTL_COMP_NONE && c <= RTL_COMP_TENSOR; }
inline bool eps_ok(float e) { return std::isfinite(e) && e >= 0.0f; }

// Layout of the rtl_sparse_linear workspace:
// [vals | k-major meta | scale | pack scratch | gemm scratch]
struct SparseWs {
    size_t vals, meta, scale, pack, gemm, total;
};
SparseWs sparse_ws(int64_t M, int64_t N, int64_t K, rtl_comp comp, size_t val_bytes = 2) {
    SparseWs w{};
    size_t off = 0;
    w.vals = off; off += round_up(rtl::kmajor_val_bytes(M, K, val_bytes), 256);
    w.meta = off; off += round_up(rtl::kmajor_bytes(M, K), 256);
    w.scale = off; off += round_up((size_t)((M > 0 ? M : 1) + 1) * sizeof(float), 256);   // + one fused scalar
    w.pack = off; off += round_up(rtl_sparsify_pack_workspace(M, K, comp), 256);
    w.gemm = off; off += round_up(rtl::gemm_workspace_bytes(true, M, N, K), 256);
    w.total = off;
    return w;
}

}  // namespace

extern "C" {

const char* rtl_status_str(rtl_status s) {
    switch (s) {
        case RTL_OK: return "RTL_OK";
        case RTL_ERR_NULL: return "RTL_ERR_NULL: a required pointer is NULL";
        case RTL_ERR_SHAPE: return "RTL_ERR_SHAPE: bad size, K granule or leading dimension";
        case RTL_ERR_ALIGN: return "RTL_ERR_ALIGN: pointer or stride alignment";
        case RTL_ERR_WORKSPACE: return "RTL_ERR_WORKSPACE: workspace missing or too small";
        case RTL_ERR_ARG: return "RTL_ERR_ARG: enum out of range or bad eps";
        case RTL_ERR_HIP: return "RTL_ERR_HIP: HIP runtime error (no device, set-up or launch)";
        case RTL_ERR_ARCH: return "RTL_ERR_ARCH: the current device is not a gfx950 (MI355X) GPU";
    }
    return "RTL_ERR_UNKNOWN";
}

const char* rtl_version(void) { return "rtlynx-gfx950 0.3"; }

rtl_status rtl_init(void) { return device_ready(); }

size_t rtl_sparsify_pack_workspace(int64_t M, int64_t K, rtl_comp comp) {
    (void)K;
    if (comp != RTL_COMP_TENSOR || M <= 0) return 0;
    return (size_t)M * 2 * sizeof(float);
}

rtl_status rtl_sparsify_pack(const void* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                             float eps, void* vals, void* meta, float* scale, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (!comp_ok(comp) || !eps_ok(eps)) return RTL_ERR_ARG;
    if (M < 0 || K < 0 || K % 8 != 0 || ldx < K || K > (int64_t)1 << 30) return RTL_ERR_SHAPE;
    if (M == 0 || K == 0) return RTL_OK;
    if (!X || !vals || !meta) return RTL_ERR_NULL;
    if ((comp == RTL_COMP_ROW || comp == RTL_COMP_TENSOR) && !scale) return RTL_ERR_NULL;
    if (ldx % 8 != 0 || !aligned(X, 16) || !aligned(vals, 16) || !aligned(meta, 4))
        return RTL_ERR_ALIGN;
    if (scale && !aligned(scale, 4)) return RTL_ERR_ALIGN;
    const size_t need = rtl_sparsify_pack_workspace(M, K, comp);
    if (need && (!workspace || workspace_bytes < need)) return RTL_ERR_WORKSPACE;
    if (need && !aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    hipError_t e = rtl::launch_sparsify_pack(
        static_cast<const uint16_t*>(X), M, K, ldx, comp, eps, static_cast<uint16_t*>(vals),
        static_cast<uint8_t*>(meta), nullptr, nullptr, scale, static_cast<float*>(workspace),
        static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

static rtl_status check_linear(const void* A, const void* W, const void* Y, int64_t M, int64_t N,
                               int64_t K, int64_t lda, int64_t ldw, int64_t ldy, int64_t a_extent,
                               int64_t k_granule = 64, int64_t ldw_granule = 8) {
    if (M < 0 || N < 0 || K <= 0 || K % k_granule != 0 || lda < a_extent || ldw < K || ldy < N)
        return RTL_ERR_SHAPE;
    if (M > ((int64_t)1 << 30) || N > ((int64_t)1 << 30) || K > ((int64_t)1 << 30))
        return RTL_ERR_SHAPE;
    // the tile loop addresses the 256 rows of a tile with 32-bit byte offsets from the tile's base
    if (lda > ((int64_t)1 << 22) || ldw > ((int64_t)1 << 22)) return RTL_ERR_SHAPE;
    // one workgroup per output tile, numbered with 32-bit integers (far beyond what fits in memory)
    if (((M + 255) / 256) * ((N + 127) / 128) >= ((int64_t)1 << 31)) return RTL_ERR_SHAPE;
    if (M == 0 || N == 0) return RTL_OK;
    if (!A || !W || !Y) return RTL_ERR_NULL;
    if (lda % 8 != 0 || ldw % ldw_granule != 0 || !aligned(A, 16) || !aligned(W, 16) || !aligned(Y, 2))
        return RTL_ERR_ALIGN;
    return RTL_OK;
}

// rtl_packed_linear workspace: [k-major copy of the values | k-major copy of the metadata | gemm scratch]
size_t rtl_packed_linear_workspace(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return round_up(rtl::kmajor_val_bytes(M, K, 2), 256) + round_up(rtl::kmajor_bytes(M, K), 256) +
           rtl::gemm_workspace_bytes(true, M, N, K);
}

rtl_status rtl_packed_linear(const void* vals, const void* meta, const float* row_scale,
                             const float* tensor_scale, const void* W, const void* bias, void* Y,
                             int64_t M, int64_t N, int64_t K, int64_t ldw, int64_t ldy,
                             void* workspace, size_t workspace_bytes, void* stream) {
    rtl_status st = check_linear(vals, W, Y, M, N, K, K / 2, ldw, ldy, K / 2);
    if (st != RTL_OK || M == 0 || N == 0) return st;
    if (!meta) return RTL_ERR_NULL;
    if (!aligned(meta, 8) || (bias && !aligned(bias, 2))) return RTL_ERR_ALIGN;
    const size_t need = rtl_packed_linear_workspace(M, N, K);
    if (need && (!workspace || workspace_bytes < need)) return RTL_ERR_WORKSPACE;
    if (need && !aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    rtl::GemmArgs g{};
    uint8_t* vkm = static_cast<uint8_t*>(workspace);
    uint8_t* km = vkm + round_up(rtl::kmajor_val_bytes(M, K, 2), 256);
    hipError_t e = rtl::launch_operand_to_kmajor(static_cast<const uint16_t*>(vals),
                                                 static_cast<const uint8_t*>(meta), M, K, vkm, km,
                                                 static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return RTL_ERR_HIP;
    g.A = vkm;
    g.meta = km;
    g.W = W;
    g.bias = static_cast<const uint16_t*>(bias);
    g.row_scale = row_scale;
    g.tensor_scale = tensor_scale;
    g.Y = static_cast<uint16_t*>(Y);
    g.M = M; g.N = N; g.K = K; g.lda = 0; g.ldw = ldw; g.ldy = ldy;
    e = rtl::launch_gemm(true, g, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

size_t rtl_sparse_linear_workspace(int64_t M, int64_t N, int64_t K, rtl_comp comp) {
    if (M <= 0 || N <= 0 || K <= 0 || !comp_ok(comp)) return 0;
    return sparse_ws(M, N, K, comp).total;
}

// Pack sweep + tile loop of rtl_sparse_linear on an already validated problem, with `base` the
// 256-byte aligned scratch of sparse_ws(M, N, K, comp).total bytes (caller's workspace, or the
// static array of rtl_sparse_linear_static).
static rtl_status sparse_linear_on(uint8_t* base, const SparseWs& ws, const void* X, const void* W,
                                   const void* bias, void* Y, int64_t M, int64_t N, int64_t K, int64_t ldx,
                                   int64_t ldw, int64_t ldy, rtl_comp comp, float eps, hipStream_t s) {
    float* scale = reinterpret_cast<float*>(base + ws.scale);
    hipError_t e = rtl::launch_sparsify_pack(
        static_cast<const uint16_t*>(X), M, K, ldx, comp, eps, nullptr, nullptr, base + ws.vals,
        base + ws.meta, scale, reinterpret_cast<float*>(base + ws.pack), s);
    if (e != hipSuccess) return RTL_ERR_HIP;
    rtl::GemmArgs g{};
    g.A = base + ws.vals;
    g.meta = base + ws.meta;
    g.W = W;
    g.bias = static_cast<const uint16_t*>(bias);
    g.row_scale = comp == RTL_COMP_ROW ? scale : nullptr;
    g.tensor_scale = comp == RTL_COMP_TENSOR ? scale : nullptr;
    g.Y = static_cast<uint16_t*>(Y);
    g.M = M; g.N = N; g.K = K; g.lda = 0; g.ldw = ldw; g.ldy = ldy;
    e = rtl::launch_gemm(true, g, s);
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

rtl_status rtl_sparse_linear(const void* X, const void* W, const void* bias, void* Y, int64_t M,
                             int64_t N, int64_t K, int64_t ldx, int64_t ldw, int64_t ldy,
                             rtl_comp comp, float eps, void* workspace, size_t workspace_bytes,
                             void* stream) {
    if (!comp_ok(comp) || !eps_ok(eps)) return RTL_ERR_ARG;
    rtl_status st = check_linear(X, W, Y, M, N, K, ldx, ldw, ldy, K);
    if (st != RTL_OK || M == 0 || N == 0) return st;
    if (bias && !aligned(bias, 2)) return RTL_ERR_ALIGN;
    const SparseWs ws = sparse_ws(M, N, K, comp);
    if (!workspace || workspace_bytes < ws.total) return RTL_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    return sparse_linear_on(static_cast<uint8_t*>(workspace), ws, X, W, bias, Y, M, N, K, ldx, ldw, ldy, comp,
                            eps, static_cast<hipStream_t>(stream));
}

rtl_status rtl_sparse_linear_static(const void* X, const void* W, const void* bias, void* Y, int64_t M,
                                    int64_t N, int64_t K, int64_t ldx, int64_t ldw, int64_t ldy,
                                    rtl_comp comp, float eps, void* stream) {
    if (!comp_ok(comp) || !eps_ok(eps)) return RTL_ERR_ARG;
    rtl_status st = check_linear(X, W, Y, M, N, K, ldx, ldw, ldy, K);
    if (st != RTL_OK || M == 0 || N == 0) return st;
    if (bias && !aligned(bias, 2)) return RTL_ERR_ALIGN;
    const SparseWs ws = sparse_ws(M, N, K, comp);
    if (ws.total > (size_t)RTL_STATIC_SCRATCH_BYTES) return RTL_ERR_WORKSPACE;   // problem too large for the fixed scratch
    void* base = nullptr;
    const rtl_status ready = device_ready(&base);    // first call on a device: looks up this device's array
    if (ready != RTL_OK) return ready;
    return sparse_linear_on(static_cast<uint8_t*>(base), ws, X, W, bias, Y, M, N, K, ldx, ldw, ldy, comp, eps,
                            static_cast<hipStream_t>(stream));
}

// rtl_sparse_lora_linear workspace: [rtl_sparse_linear workspace | T as two bf16 planes [2][M,64] |
// per-K-range partial planes and row sums of the one-pass sweep]
size_t rtl_sparse_lora_linear_workspace(int64_t M, int64_t N, int64_t K, int64_t R, rtl_comp comp) {
    if (M <= 0 || N <= 0 || K <= 0 || R != rtl::kLoraRank || !comp_ok(comp)) return 0;
    return sparse_ws(M, N, K, comp).total + round_up((size_t)M * rtl::kLoraRank * 4, 256) +
           round_up(rtl::pack_down_scratch_bytes(M, K), 256);
}

rtl_status rtl_sparse_lora_linear(const void* X, const void* W, const void* LA, const void* LB,
                                  const void* bias, void* Y, int64_t M, int64_t N, int64_t K,
                                  int64_t R, int64_t ldx, int64_t ldw, int64_t ldla, int64_t ldlb,
                                  int64_t ldy, rtl_comp comp, float eps, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    if (!comp_ok(comp) || !eps_ok(eps)) return RTL_ERR_ARG;
    if (R != rtl::kLoraRank || ldla < R || ldlb < K) return RTL_ERR_SHAPE;
    rtl_status st = check_linear(X, W, Y, M, N, K, ldx, ldw, ldy, K);
    if (st != RTL_OK || M == 0 || N == 0) return st;
    if (!LA || !LB) return RTL_ERR_NULL;
    if (ldla % 8 != 0 || ldlb % 8 != 0 || !aligned(LA, 16) || !aligned(LB, 16) ||
        (bias && !aligned(bias, 2)))
        return RTL_ERR_ALIGN;
    const SparseWs ws = sparse_ws(M, N, K, comp);
    const size_t t_off = ws.total, p_off = t_off + round_up((size_t)M * rtl::kLoraRank * 4, 256);
    const size_t need = p_off + round_up(rtl::pack_down_scratch_bytes(M, K), 256);
    if (!workspace || workspace_bytes < need) return RTL_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    uint8_t* base = static_cast<uint8_t*>(workspace);
    float* scale = reinterpret_cast<float*>(base + ws.scale);
    uint16_t* T = reinterpret_cast<uint16_t*>(base + t_off);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // one pass over X: the sweep that compresses the activation also forms T = X L_B^T
    hipError_t e = rtl::launch_pack_down(static_cast<const uint16_t*>(X), M, K, ldx, comp, eps,
                                         static_cast<const uint16_t*>(LB), ldlb, base + ws.vals, base + ws.meta,
                                         reinterpret_cast<float*>(base + p_off), T, scale,
                                         reinterpret_cast<float*>(base + ws.pack), s);
    if (e != hipSuccess) return RTL_ERR_HIP;
    rtl::GemmArgs g{};
    g.A = base + ws.vals;
    g.meta = base + ws.meta;
    g.W = W;
    g.bias = static_cast<const uint16_t*>(bias);
    g.row_scale = comp == RTL_COMP_ROW ? scale : nullptr;
    g.tensor_scale = comp == RTL_COMP_TENSOR ? scale : nullptr;
    g.Y = static_cast<uint16_t*>(Y);
    g.M = M; g.N = N; g.K = K; g.lda = 0; g.ldw = ldw; g.ldy = ldy;
    g.T = T;
    g.LA = static_cast<const uint16_t*>(LA);
    g.ldla = ldla;
    e = rtl::launch_gemm(true, g, s);
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

// ---- FP8 (E4M3) composition -------------------------------------------------------------------

rtl_status rtl_quantize_fp8(const void* W, int64_t rows, int64_t cols, int64_t ld, void* Wq,
                            int64_t ldq, void* stream) {
    if (rows < 0 || cols < 0 || cols % 8 != 0 || ld < cols || ldq < cols) return RTL_ERR_SHAPE;
    if (rows > ((int64_t)1 << 30) || cols > ((int64_t)1 << 30)) return RTL_ERR_SHAPE;
    if (rows == 0 || cols == 0) return RTL_OK;
    if (!W || !Wq) return RTL_ERR_NULL;
    if (ld % 8 != 0 || ldq % 8 != 0 || !aligned(W, 16) || !aligned(Wq, 8)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    hipError_t e = rtl::launch_quantize_fp8(static_cast<const uint16_t*>(W), rows, cols, ld,
                                            static_cast<uint8_t*>(Wq), ldq,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

size_t rtl_sparsify_pack_fp8_workspace(int64_t M, int64_t K, rtl_comp comp) {
    return rtl_sparsify_pack_workspace(M, K, comp);
}

rtl_status rtl_sparsify_pack_fp8(const void* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp,
                                 float eps, const float* x_scale, void* vals, void* meta,
                                 float* scale, void* workspace, size_t workspace_bytes, void* stream) {
    if (!comp_ok(comp) || !eps_ok(eps)) return RTL_ERR_ARG;
    if (M < 0 || K < 0 || K % 8 != 0 || ldx < K || K > (int64_t)1 << 30) return RTL_ERR_SHAPE;
    if (M == 0 || K == 0) return RTL_OK;
    if (!X || !vals || !meta || !x_scale) return RTL_ERR_NULL;
    if ((comp == RTL_COMP_ROW || comp == RTL_COMP_TENSOR) && !scale) return RTL_ERR_NULL;
    if (ldx % 8 != 0 || !aligned(X, 16) || !aligned(vals, 4) || !aligned(meta, 4) || !aligned(x_scale, 4))
        return RTL_ERR_ALIGN;
    if (scale && !aligned(scale, 4)) return RTL_ERR_ALIGN;
    const size_t need = rtl_sparsify_pack_fp8_workspace(M, K, comp);
    if (need && (!workspace || workspace_bytes < need)) return RTL_ERR_WORKSPACE;
    if (need && !aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    hipError_t e = rtl::launch_sparsify_pack_fp8(
        static_cast<const uint16_t*>(X), M, K, ldx, comp, eps, x_scale, static_cast<uint8_t*>(vals),
        static_cast<uint8_t*>(meta), nullptr, nullptr, scale, static_cast<float*>(workspace), nullptr,
        static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

size_t rtl_sparse_linear_fp8_workspace(int64_t M, int64_t N, int64_t K, rtl_comp comp) {
    if (M <= 0 || N <= 0 || K <= 0 || !comp_ok(comp)) return 0;
    return sparse_ws(M, N, K, comp, 1).total;
}

rtl_status rtl_sparse_linear_fp8(const void* X, const void* Wq, const float* x_scale, const void* bias,
                                 void* Y, int64_t M, int64_t N, int64_t K, int64_t ldx, int64_t ldw,
                                 int64_t ldy, rtl_comp comp, float eps, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    if (!comp_ok(comp) || !eps_ok(eps)) return RTL_ERR_ARG;
    rtl_status st = check_linear(X, Wq, Y, M, N, K, ldx, ldw, ldy, K, 128, 16);
    if (st != RTL_OK || M == 0 || N == 0) return st;
    if (!x_scale) return RTL_ERR_NULL;
    if ((bias && !aligned(bias, 2)) || !aligned(x_scale, 4)) return RTL_ERR_ALIGN;
    const SparseWs ws = sparse_ws(M, N, K, comp, 1);
    if (!workspace || workspace_bytes < ws.total) return RTL_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    uint8_t* base = static_cast<uint8_t*>(workspace);
    float* scale = reinterpret_cast<float*>(base + ws.scale);
    float* fused = scale + (comp == RTL_COMP_ROW ? M : 1);   // x_scale times the TENSOR factor
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = rtl::launch_sparsify_pack_fp8(
        static_cast<const uint16_t*>(X), M, K, ldx, comp, eps, x_scale, nullptr, nullptr, base + ws.vals,
        base + ws.meta, scale, reinterpret_cast<float*>(base + ws.pack), fused, s);
    if (e != hipSuccess) return RTL_ERR_HIP;
    rtl::GemmArgs g{};
    g.fp8 = true;
    g.A = base + ws.vals;
    g.meta = base + ws.meta;
    g.W = Wq;
    g.bias = static_cast<const uint16_t*>(bias);
    g.row_scale = comp == RTL_COMP_ROW ? scale : nullptr;
    g.tensor_scale = comp == RTL_COMP_TENSOR ? fused : x_scale;   // dequantisation rides on the epilogue
    g.Y = static_cast<uint16_t*>(Y);
    g.M = M; g.N = N; g.K = K; g.lda = 0; g.ldw = ldw; g.ldy = ldy;
    e = rtl::launch_gemm(true, g, s);
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

// rtl_sparse_lora_linear_fp8 workspace: [rtl_sparse_linear_fp8 workspace | T as two bf16 planes | sweep scratch]
size_t rtl_sparse_lora_linear_fp8_workspace(int64_t M, int64_t N, int64_t K, int64_t R, rtl_comp comp) {
    if (M <= 0 || N <= 0 || K <= 0 || R != rtl::kLoraRank || !comp_ok(comp)) return 0;
    return sparse_ws(M, N, K, comp, 1).total + round_up((size_t)M * rtl::kLoraRank * 4, 256) +
           round_up(rtl::pack_down_scratch_bytes(M, K), 256);
}

rtl_status rtl_sparse_lora_linear_fp8(const void* X, const void* Wq, const float* x_scale, const void* LA,
                                      const void* LB, const void* bias, void* Y, int64_t M, int64_t N, int64_t K,
                                      int64_t R, int64_t ldx, int64_t ldw, int64_t ldla, int64_t ldlb, int64_t ldy,
                                      rtl_comp comp, float eps, void* workspace, size_t workspace_bytes,
                                      void* stream) {
    if (!comp_ok(comp) || !eps_ok(eps)) return RTL_ERR_ARG;
    if (R != rtl::kLoraRank || ldla < R || ldlb < K) return RTL_ERR_SHAPE;
    rtl_status st = check_linear(X, Wq, Y, M, N, K, ldx, ldw, ldy, K, 128, 16);
    if (st != RTL_OK || M == 0 || N == 0) return st;
    if (!x_scale || !LA || !LB) return RTL_ERR_NULL;
    if (ldla % 8 != 0 || ldlb % 8 != 0 || !aligned(LA, 16) || !aligned(LB, 16) || (bias && !aligned(bias, 2)) ||
        !aligned(x_scale, 4))
        return RTL_ERR_ALIGN;
    const SparseWs ws = sparse_ws(M, N, K, comp, 1);
    const size_t t_off = ws.total, p_off = t_off + round_up((size_t)M * rtl::kLoraRank * 4, 256);
    const size_t need = p_off + round_up(rtl::pack_down_scratch_bytes(M, K), 256);
    if (!workspace || workspace_bytes < need) return RTL_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    uint8_t* base = static_cast<uint8_t*>(workspace);
    float* scale = reinterpret_cast<float*>(base + ws.scale);
    float* fused = scale + (comp == RTL_COMP_ROW ? M : 1);   // x_scale times the TENSOR factor
    uint16_t* T = reinterpret_cast<uint16_t*>(base + t_off);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = rtl::launch_pack_down(static_cast<const uint16_t*>(X), M, K, ldx, comp, eps,
                                         static_cast<const uint16_t*>(LB), ldlb, base + ws.vals, base + ws.meta,
                                         reinterpret_cast<float*>(base + p_off), T, scale,
                                         reinterpret_cast<float*>(base + ws.pack), s, x_scale, fused);
    if (e != hipSuccess) return RTL_ERR_HIP;
    rtl::GemmArgs g{};
    g.fp8 = true;
    g.A = base + ws.vals;
    g.meta = base + ws.meta;
    g.W = Wq;
    g.bias = static_cast<const uint16_t*>(bias);
    g.row_scale = comp == RTL_COMP_ROW ? scale : nullptr;
    g.tensor_scale = comp == RTL_COMP_TENSOR ? fused : x_scale;   // dequantisation of the sparse product only
    g.Y = static_cast<uint16_t*>(Y);
    g.M = M; g.N = N; g.K = K; g.lda = 0; g.ldw = ldw; g.ldy = ldy;
    g.T = T;
    g.LA = static_cast<const uint16_t*>(LA);
    g.ldla = ldla;
    e = rtl::launch_gemm(true, g, s);
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

rtl_status rtl_diag_matrix_rate(int kind, const void* operands, int64_t iters, int blocks,
                                uint64_t* clocks, float* sink, void* stream) {
    if (kind < 0 || kind > 1) return RTL_ERR_ARG;
    if (iters <= 0 || iters > ((int64_t)1 << 24) || blocks <= 0 || blocks > 65536) return RTL_ERR_SHAPE;
    if (!operands || !clocks || !sink) return RTL_ERR_NULL;
    if (!aligned(operands, 16) || !aligned(clocks, 8) || !aligned(sink, 4)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    hipError_t e = rtl::launch_matrix_rate(kind, operands, iters, blocks,
                                           reinterpret_cast<unsigned long long*>(clocks), sink,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

rtl_status rtl_diag_fill_rate(const void* region, size_t region_bytes, int64_t iters, int blocks,
                              uint64_t* clocks, float* sink, void* stream) {
    if (iters <= 0 || iters > ((int64_t)1 << 24) || blocks <= 0 || blocks > 65536) return RTL_ERR_SHAPE;
    if (region_bytes < ((size_t)1 << 20) || region_bytes % 8192 != 0) return RTL_ERR_SHAPE;
    if (!region || !clocks || !sink) return RTL_ERR_NULL;
    if (!aligned(region, 16) || !aligned(clocks, 8) || !aligned(sink, 4)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    hipError_t e = rtl::launch_fill_rate(region, region_bytes, iters, blocks,
                                         reinterpret_cast<unsigned long long*>(clocks), sink,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

rtl_status rtl_diag_pack_sweep(const void* X, int64_t M, int64_t K, int64_t ldx, rtl_comp comp, float eps,
                               void* workspace, size_t workspace_bytes, void* stream) {
    if (!comp_ok(comp) || !eps_ok(eps)) return RTL_ERR_ARG;
    if (M < 0 || K <= 0 || K % 64 != 0 || ldx < K || M > ((int64_t)1 << 30) || K > ((int64_t)1 << 30) ||
        ldx > ((int64_t)1 << 22))
        return RTL_ERR_SHAPE;
    if (M == 0) return RTL_OK;
    if (!X) return RTL_ERR_NULL;
    if (ldx % 8 != 0 || !aligned(X, 16)) return RTL_ERR_ALIGN;
    const SparseWs ws = sparse_ws(M, 1, K, comp);
    if (!workspace || workspace_bytes < ws.total) return RTL_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    uint8_t* base = static_cast<uint8_t*>(workspace);
    hipError_t e = rtl::launch_sparsify_pack(static_cast<const uint16_t*>(X), M, K, ldx, comp, eps, nullptr, nullptr,
                                             base + ws.vals, base + ws.meta, reinterpret_cast<float*>(base + ws.scale),
                                             reinterpret_cast<float*>(base + ws.pack), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

rtl_status rtl_diag_tile_plan(int64_t M, int64_t N, int dense, int64_t* plan) {
    if (M <= 0 || N <= 0 || M > ((int64_t)1 << 30) || N > ((int64_t)1 << 30)) return RTL_ERR_SHAPE;
    if (!plan) return RTL_ERR_NULL;
    rtl::tile_plan(M, N, dense != 0, plan);
    return RTL_OK;
}

size_t rtl_dense_linear_workspace(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return rtl::gemm_workspace_bytes(false, M, N, K);
}

rtl_status rtl_dense_linear(const void* X, const void* W, const void* bias, void* Y, int64_t M,
                            int64_t N, int64_t K, int64_t ldx, int64_t ldw, int64_t ldy,
                            void* workspace, size_t workspace_bytes, void* stream) {
    rtl_status st = check_linear(X, W, Y, M, N, K, ldx, ldw, ldy, K);
    if (st != RTL_OK || M == 0 || N == 0) return st;
    if (bias && !aligned(bias, 2)) return RTL_ERR_ALIGN;
    const size_t need = rtl_dense_linear_workspace(M, N, K);
    if (need && (!workspace || workspace_bytes < need)) return RTL_ERR_WORKSPACE;
    if (need && !aligned(workspace, 256)) return RTL_ERR_ALIGN;
    RTL_REQUIRE_DEVICE();
    rtl::GemmArgs g{};
    g.A = X;
    g.W = W;
    g.bias = static_cast<const uint16_t*>(bias);
    g.Y = static_cast<uint16_t*>(Y);
    g.M = M; g.N = N; g.K = K; g.lda = ldx; g.ldw = ldw; g.ldy = ldy;
    hipError_t e = rtl::launch_gemm(false, g, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTL_OK : RTL_ERR_HIP;
}

}  // extern "C"
