"""Thin ctypes binding of librtlynx.so: argument marshalling only.

Same entry points as include/rtlynx.h. Tensors are torch CUDA tensors (used for device memory
and the current stream); every step of the path runs inside the library's HIP kernels. There is
no fallback: a missing library or a non-zero status raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librtlynx.so")

COMP_NONE, COMP_GROUP, COMP_ROW, COMP_TENSOR = 0, 1, 2, 3
COMP = {"none": COMP_NONE, "group": COMP_GROUP, "row": COMP_ROW, "tensor": COMP_TENSOR}

SYMBOLS = ["rtl_sparsify_pack_workspace", "rtl_sparsify_pack", "rtl_packed_linear_workspace",
           "rtl_packed_linear", "rtl_sparse_linear_workspace", "rtl_sparse_linear", "rtl_sparse_linear_static",
           "rtl_sparse_lora_linear_workspace", "rtl_sparse_lora_linear",
           "rtl_dense_linear_workspace", "rtl_dense_linear",
           "rtl_quantize_fp8", "rtl_sparsify_pack_fp8_workspace", "rtl_sparsify_pack_fp8",
           "rtl_sparse_linear_fp8_workspace", "rtl_sparse_linear_fp8",
           "rtl_sparse_lora_linear_fp8_workspace", "rtl_sparse_lora_linear_fp8",
           "rtl_diag_matrix_rate", "rtl_diag_fill_rate", "rtl_diag_pack_sweep", "rtl_diag_tile_plan", "rtl_init", "rtl_status_str", "rtl_version"]

_lib = None


class RtlError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s failed: %s" % (where, status_str(status)))


def lib():
    """Load librtlynx.so (built in-tree by paper_2605_26632_amd/build.py). Raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("librtlynx.so is not built: run `python -m paper_2605_26632_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        i64, vp, sz, fl, ci = C.c_int64, C.c_void_p, C.c_size_t, C.c_float, C.c_int
        L.rtl_sparsify_pack_workspace.argtypes = [i64, i64, ci]
        L.rtl_sparsify_pack_workspace.restype = sz
        L.rtl_sparsify_pack.argtypes = [vp, i64, i64, i64, ci, fl, vp, vp, vp, vp, sz, vp]
        L.rtl_sparsify_pack.restype = ci
        L.rtl_packed_linear_workspace.argtypes = [i64, i64, i64]
        L.rtl_packed_linear_workspace.restype = sz
        L.rtl_packed_linear.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, vp, sz, vp]
        L.rtl_packed_linear.restype = ci
        L.rtl_sparse_linear_workspace.argtypes = [i64, i64, i64, ci]
        L.rtl_sparse_linear_workspace.restype = sz
        L.rtl_sparse_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, fl, vp, sz, vp]
        L.rtl_sparse_linear.restype = ci
        L.rtl_sparse_linear_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, fl, vp]
        L.rtl_sparse_linear_static.restype = ci
        L.rtl_sparse_lora_linear_workspace.argtypes = [i64, i64, i64, i64, ci]
        L.rtl_sparse_lora_linear_workspace.restype = sz
        L.rtl_sparse_lora_linear.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64,
                                             i64, i64, ci, fl, vp, sz, vp]
        L.rtl_sparse_lora_linear.restype = ci
        L.rtl_dense_linear_workspace.argtypes = [i64, i64, i64]
        L.rtl_dense_linear_workspace.restype = sz
        L.rtl_dense_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, vp, sz, vp]
        L.rtl_dense_linear.restype = ci
        L.rtl_quantize_fp8.argtypes = [vp, i64, i64, i64, vp, i64, vp]
        L.rtl_quantize_fp8.restype = ci
        L.rtl_sparsify_pack_fp8_workspace.argtypes = [i64, i64, ci]
        L.rtl_sparsify_pack_fp8_workspace.restype = sz
        L.rtl_sparsify_pack_fp8.argtypes = [vp, i64, i64, i64, ci, fl, vp, vp, vp, vp, vp, sz, vp]
        L.rtl_sparsify_pack_fp8.restype = ci
        L.rtl_sparse_linear_fp8_workspace.argtypes = [i64, i64, i64, ci]
        L.rtl_sparse_linear_fp8_workspace.restype = sz
        L.rtl_sparse_linear_fp8.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, ci, fl, vp, sz, vp]
        L.rtl_sparse_linear_fp8.restype = ci
        L.rtl_diag_matrix_rate.argtypes = [ci, vp, i64, ci, vp, vp, vp]
        L.rtl_diag_matrix_rate.restype = ci
        L.rtl_diag_fill_rate.argtypes = [vp, sz, i64, ci, vp, vp, vp]
        L.rtl_diag_fill_rate.restype = ci
        L.rtl_sparse_lora_linear_fp8_workspace.argtypes = [i64, i64, i64, i64, ci]
        L.rtl_sparse_lora_linear_fp8_workspace.restype = sz
        L.rtl_sparse_lora_linear_fp8.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, i64,
                                                 i64, ci, fl, vp, sz, vp]
        L.rtl_sparse_lora_linear_fp8.restype = ci
        L.rtl_diag_pack_sweep.argtypes = [vp, i64, i64, i64, ci, fl, vp, sz, vp]
        L.rtl_diag_pack_sweep.restype = ci
        L.rtl_diag_tile_plan.argtypes = [i64, i64, ci, C.POINTER(C.c_int64)]
        L.rtl_diag_tile_plan.restype = ci
        L.rtl_init.argtypes = []
        L.rtl_init.restype = ci
        L.rtl_status_str.argtypes = [ci]
        L.rtl_status_str.restype = C.c_char_p
        L.rtl_version.restype = C.c_char_p
        _lib = L
    return _lib


def status_str(status):
    return lib().rtl_status_str(int(status)).decode()


def version():
    return lib().rtl_version().decode()


def init():
    """rtl_init: one-time set-up of the current device (required only before HIP-graph capture)."""
    _check(lib().rtl_init(), "rtl_init")


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != 0:
        raise RtlError(status, where)


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("librtlynx takes device tensors only")


def _ws(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def sparsify_pack(X, comp=COMP_GROUP, eps=1e-8, out=None):
    """rtl_sparsify_pack: X bf16 [M,K] -> (vals bf16 [M,K/2], meta u8 [M,K/8], scale fp32 or None)."""
    _need_cuda(X)
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    dev = X.device
    if out is None:
        vals = torch.empty((M, K // 2), dtype=torch.bfloat16, device=dev)
        meta = torch.empty((M, K // 8), dtype=torch.uint8, device=dev)
    else:
        vals, meta = out
    scale = None
    if comp == COMP_ROW:
        scale = torch.empty((M,), dtype=torch.float32, device=dev)
    elif comp == COMP_TENSOR:
        scale = torch.empty((1,), dtype=torch.float32, device=dev)
    L = lib()
    nws = L.rtl_sparsify_pack_workspace(M, K, comp)
    ws = _ws(nws, dev)
    st = L.rtl_sparsify_pack(_p(X), M, K, X.stride(0), comp, eps, _p(vals), _p(meta), _p(scale),
                             _p(ws), ws.numel(), _stream())
    _check(st, "rtl_sparsify_pack")
    return vals, meta, scale


def packed_linear(vals, meta, W, bias=None, row_scale=None, tensor_scale=None, out=None, ws=None):
    """rtl_packed_linear: Y = decode(vals, meta) W^T (* scales) (+ bias), bf16 [M,N]."""
    _need_cuda(vals, meta, W)
    M, K = vals.shape[0], vals.shape[1] * 2
    N = W.shape[0]
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=W.device) if out is None else out
    L = lib()
    if ws is None:
        ws = _ws(L.rtl_packed_linear_workspace(M, N, K), W.device)
    st = L.rtl_packed_linear(_p(vals), _p(meta), _p(row_scale), _p(tensor_scale), _p(W), _p(bias),
                             _p(Y), M, N, K, W.stride(0), Y.stride(0), _p(ws), ws.numel(), _stream())
    _check(st, "rtl_packed_linear")
    return Y


def sparse_linear_workspace(M, N, K, comp=COMP_GROUP):
    return int(lib().rtl_sparse_linear_workspace(M, N, K, comp))


def sparse_linear(X, W, bias=None, comp=COMP_GROUP, eps=1e-8, out=None, ws=None):
    """rtl_sparse_linear: Y = compensate(sparsify_2:4(X)) W^T (+ bias), bf16 [M,N]."""
    _need_cuda(X, W)
    M, K = X.shape
    N = W.shape[0]
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if out is None else out
    L = lib()
    if ws is None:
        ws = _ws(L.rtl_sparse_linear_workspace(M, N, K, comp), X.device)
    st = L.rtl_sparse_linear(_p(X), _p(W), _p(bias), _p(Y), M, N, K, X.stride(0), W.stride(0),
                             Y.stride(0), comp, eps, _p(ws), ws.numel(), _stream())
    _check(st, "rtl_sparse_linear")
    return Y


STATIC_SCRATCH_BYTES = 64 * 1024 * 1024     # RTL_STATIC_SCRATCH_BYTES of the header


def sparse_linear_static(X, W, Y, bias=None, comp=COMP_GROUP, eps=1e-8):
    """rtl_sparse_linear_static: rtl_sparse_linear on the library's fixed scratch; the caller passes
    inputs and the output, nothing is allocated (not by the library, not here)."""
    _need_cuda(X, W, Y)
    M, K = X.shape
    N = W.shape[0]
    st = lib().rtl_sparse_linear_static(_p(X), _p(W), _p(bias), _p(Y), M, N, K, X.stride(0), W.stride(0),
                                        Y.stride(0), comp, eps, _stream())
    _check(st, "rtl_sparse_linear_static")
    return Y


def sparse_lora_linear_workspace(M, N, K, R=64, comp=COMP_GROUP):
    return int(lib().rtl_sparse_lora_linear_workspace(M, N, K, R, comp))


def sparse_lora_linear(X, W, LA, LB, bias=None, comp=COMP_GROUP, eps=1e-8, out=None, ws=None):
    """rtl_sparse_lora_linear: Y = compensate(sparsify_2:4(X)) W^T + X (L_A L_B)^T (+ bias)."""
    _need_cuda(X, W, LA, LB)
    M, K = X.shape
    N, R = LA.shape
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if out is None else out
    L = lib()
    if ws is None:
        ws = _ws(L.rtl_sparse_lora_linear_workspace(M, N, K, R, comp), X.device)
    st = L.rtl_sparse_lora_linear(_p(X), _p(W), _p(LA), _p(LB), _p(bias), _p(Y), M, N, K, R,
                                  X.stride(0), W.stride(0), LA.stride(0), LB.stride(0), Y.stride(0),
                                  comp, eps, _p(ws), ws.numel(), _stream())
    _check(st, "rtl_sparse_lora_linear")
    return Y


def dense_linear(X, W, bias=None, out=None, ws=None):
    """rtl_dense_linear: Y = X W^T (+ bias), bf16 [M,N]."""
    _need_cuda(X, W)
    M, K = X.shape
    N = W.shape[0]
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if out is None else out
    L = lib()
    if ws is None:
        ws = _ws(L.rtl_dense_linear_workspace(M, N, K), X.device)
    st = L.rtl_dense_linear(_p(X), _p(W), _p(bias), _p(Y), M, N, K, X.stride(0), W.stride(0),
                            Y.stride(0), _p(ws), ws.numel(), _stream())
    _check(st, "rtl_dense_linear")
    return Y


# ---- FP8 (E4M3) composition; codes travel as uint8 tensors ----------------------------------

def quantize_fp8(W, out=None):
    """rtl_quantize_fp8: bf16 [rows, cols] -> E4M3 codes (uint8), direct cast."""
    _need_cuda(W)
    assert W.dtype == torch.bfloat16 and W.dim() == 2 and W.stride(1) == 1
    rows, cols = W.shape
    Wq = torch.empty((rows, cols), dtype=torch.uint8, device=W.device) if out is None else out
    st = lib().rtl_quantize_fp8(_p(W), rows, cols, W.stride(0), _p(Wq), Wq.stride(0), _stream())
    _check(st, "rtl_quantize_fp8")
    return Wq


def sparsify_pack_fp8(X, x_scale, comp=COMP_GROUP, eps=1e-8, out=None):
    """rtl_sparsify_pack_fp8: X bf16 [M,K], x_scale fp32 [1] -> (vals u8 [M,K/2], meta u8 [M,K/8], scale)."""
    _need_cuda(X, x_scale)
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.stride(1) == 1
    assert x_scale.dtype == torch.float32
    M, K = X.shape
    dev = X.device
    if out is None:
        vals = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
        meta = torch.empty((M, K // 8), dtype=torch.uint8, device=dev)
    else:
        vals, meta = out
    scale = None
    if comp == COMP_ROW:
        scale = torch.empty((M,), dtype=torch.float32, device=dev)
    elif comp == COMP_TENSOR:
        scale = torch.empty((1,), dtype=torch.float32, device=dev)
    L = lib()
    ws = _ws(L.rtl_sparsify_pack_fp8_workspace(M, K, comp), dev)
    st = L.rtl_sparsify_pack_fp8(_p(X), M, K, X.stride(0), comp, eps, _p(x_scale), _p(vals), _p(meta),
                                 _p(scale), _p(ws), ws.numel(), _stream())
    _check(st, "rtl_sparsify_pack_fp8")
    return vals, meta, scale


def sparse_linear_fp8_workspace(M, N, K, comp=COMP_GROUP):
    return int(lib().rtl_sparse_linear_fp8_workspace(M, N, K, comp))


def sparse_linear_fp8(X, Wq, x_scale, bias=None, comp=COMP_GROUP, eps=1e-8, out=None, ws=None):
    """rtl_sparse_linear_fp8: Y = x_scale * (e4m3(S(X) / x_scale) Wq^T) (+ bias), bf16 [M,N]."""
    _need_cuda(X, Wq, x_scale)
    assert Wq.dtype == torch.uint8 and x_scale.dtype == torch.float32
    M, K = X.shape
    N = Wq.shape[0]
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if out is None else out
    L = lib()
    if ws is None:
        ws = _ws(L.rtl_sparse_linear_fp8_workspace(M, N, K, comp), X.device)
    st = L.rtl_sparse_linear_fp8(_p(X), _p(Wq), _p(x_scale), _p(bias), _p(Y), M, N, K, X.stride(0),
                                 Wq.stride(0), Y.stride(0), comp, eps, _p(ws), ws.numel(), _stream())
    _check(st, "rtl_sparse_linear_fp8")
    return Y


def sparse_lora_linear_fp8_workspace(M, N, K, R=64, comp=COMP_GROUP):
    return int(lib().rtl_sparse_lora_linear_fp8_workspace(M, N, K, R, comp))


def sparse_lora_linear_fp8(X, Wq, x_scale, LA, LB, bias=None, comp=COMP_GROUP, eps=1e-8, out=None, ws=None):
    """rtl_sparse_lora_linear_fp8: Y = x_scale * (e4m3(S(X) / x_scale) Wq^T) + X (L_A L_B)^T (+ bias), bf16 [M,N]."""
    _need_cuda(X, Wq, x_scale, LA, LB)
    assert Wq.dtype == torch.uint8 and x_scale.dtype == torch.float32
    assert LA.dtype == torch.bfloat16 and LB.dtype == torch.bfloat16
    M, K = X.shape
    N, R = LA.shape
    assert Wq.shape == (N, K) and LB.shape == (R, K)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if out is None else out
    L = lib()
    if ws is None:
        ws = _ws(L.rtl_sparse_lora_linear_fp8_workspace(M, N, K, R, comp), X.device)
    st = L.rtl_sparse_lora_linear_fp8(_p(X), _p(Wq), _p(x_scale), _p(LA), _p(LB), _p(bias), _p(Y), M, N, K, R,
                                      X.stride(0), Wq.stride(0), LA.stride(0), LB.stride(0), Y.stride(0), comp, eps,
                                      _p(ws), ws.numel(), _stream())
    _check(st, "rtl_sparse_lora_linear_fp8")
    return Y


# ---- diagnostics ------------------------------------------------------------------------------

def diag_matrix_rate(kind, operands, iters, blocks=1024):
    """rtl_diag_matrix_rate: enqueue the issue-rate probe; returns (clocks uint64[2] as an int64 tensor,
    executed flops of the launch). Timing is the caller's (events around the call)."""
    _need_cuda(operands)
    assert operands.numel() * operands.element_size() >= 3072
    clocks = torch.zeros(2, dtype=torch.int64, device=operands.device)
    sink = torch.zeros(1, dtype=torch.float32, device=operands.device)
    st = lib().rtl_diag_matrix_rate(int(kind), _p(operands), int(iters), int(blocks), _p(clocks), _p(sink), _stream())
    _check(st, "rtl_diag_matrix_rate")
    return clocks, float(blocks) * 4 * 4 * iters * 2 * 32 * 32 * 16


def diag_pack_sweep(X, comp=COMP_GROUP, eps=1e-8, ws=None):
    """rtl_diag_pack_sweep: the sparsification sweep as rtl_sparse_linear launches it, alone (for timing);
    the compressed operand lands in the head of `ws` (an rtl_sparse_linear workspace)."""
    _need_cuda(X)
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    L = lib()
    if ws is None:
        ws = _ws(L.rtl_sparse_linear_workspace(M, 1, K, comp), X.device)
    _check(L.rtl_diag_pack_sweep(_p(X), M, K, X.stride(0), comp, eps, _p(ws), ws.numel(), _stream()),
           "rtl_diag_pack_sweep")
    return ws


def diag_tile_plan(M, N, dense=False):
    """rtl_diag_tile_plan: dict(body_width, body_rows, body_tiles, tail_tiles) for an [M, N] output."""
    out = (C.c_int64 * 4)()
    _check(lib().rtl_diag_tile_plan(int(M), int(N), int(bool(dense)), out), "rtl_diag_tile_plan")
    return dict(body_width=int(out[0]), body_rows=int(out[1]), body_tiles=int(out[2]), tail_tiles=int(out[3]))


def diag_fill_rate(region, iters, blocks=256):
    """rtl_diag_fill_rate: enqueue the L2 -> LDS streaming probe on `region` (a uint8 device tensor);
    returns (clocks int64[2] tensor, bytes moved by the launch)."""
    _need_cuda(region)
    nbytes = region.numel() * region.element_size()
    clocks = torch.zeros(2, dtype=torch.int64, device=region.device)
    sink = torch.zeros(1, dtype=torch.float32, device=region.device)
    st = lib().rtl_diag_fill_rate(_p(region), nbytes, int(iters), int(blocks), _p(clocks), _p(sink), _stream())
    _check(st, "rtl_diag_fill_rate")
    return clocks, float(blocks) * 8 * iters * 8192
