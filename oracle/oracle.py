"""ctypes front end of the C oracle: numpy in, numpy out, bf16 carried as uint16 bit patterns.

Each function names the passage of the paper it follows; the arithmetic itself lives in
rtlynx_oracle.c. `sparse_linear_oracle` strings the steps together in the order of Alg. 1.
"""
import ctypes as C
import numpy as np

from .build import build as _build

NONE, GROUP, ROW, TENSOR = 0, 1, 2, 3
SCOPES = {"none": NONE, "group": GROUP, "row": ROW, "tensor": TENSOR}

# RTL_ORACLE_LIB: load another build of the oracle instead (used only by the mutation test, which
# plants mistakes in a copy of rtlynx_oracle.c and checks that the pins notice them).
import os as _os
_lib = C.CDLL(_os.environ.get("RTL_ORACLE_LIB") or _build())
_i64 = C.c_int64
_p = C.c_void_p


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 tensors travel as uint16 bit patterns"
    return a


_lib.orc_topk24.argtypes = [_p, _i64, _i64, _i64, _p]
_lib.orc_scales.argtypes = [_p, _p, _i64, _i64, _i64, C.c_int, C.c_float, _p]
_lib.orc_apply.argtypes = [_p, _p, _p, _i64, _i64, _i64, C.c_int, C.c_int, _p, _p]
_lib.orc_pack.argtypes = [_p, _i64, _p, _i64, _i64, _p, _p]
_lib.orc_unpack.argtypes = [_p, _p, _i64, _i64, _p]
_lib.orc_linear.argtypes = [_p, _p, _p, _i64, _i64, _i64, _i64, _i64, _i64, _p]
_lib.orc_lora_delta.argtypes = [_p, _p, _i64, _i64, _i64, _p]
_lib.orc_linear_f32w.argtypes = [_p, _p, _i64, _i64, _i64, _i64, _i64, _p]
_lib.orc_add.argtypes = [_p, _p, _i64, _p]
_lib.orc_widen.argtypes = [_p, _i64, _i64, _i64, _p]
_lib.orc_round_bf16.argtypes = [_p, _i64, _p]
_lib.orc_rfe.argtypes = [_p, _p, _i64]
_lib.orc_rfe.restype = C.c_double
_lib.orc_bf16_to_f32.argtypes = [C.c_uint16]
_lib.orc_bf16_to_f32.restype = C.c_float
_lib.orc_f32_to_bf16.argtypes = [C.c_float]
_lib.orc_f32_to_bf16.restype = C.c_uint16
_lib.orc_num_threads.restype = C.c_int
_lib.orc_e4m3_encode.argtypes = [_p, _i64, _p]
_lib.orc_e4m3_decode.argtypes = [_p, _i64, _p]
_lib.orc_apply_fp8.argtypes = [_p, _p, _p, _i64, _i64, _i64, C.c_int, C.c_float, _p]
_lib.orc_pack8.argtypes = [_p, _p, _i64, _i64, _p, _p]


def num_threads() -> int:
    return int(_lib.orc_num_threads())


def bf16_to_f32(bits):
    """Widen bf16 bit patterns (uint16 array) to float32."""
    bits = _u16(bits)
    out = np.empty(bits.shape, dtype=np.float32)
    flat = bits.reshape(1, -1)
    _lib.orc_widen(_ptr(flat), 1, flat.shape[1], flat.shape[1], _ptr(out))
    return out


def f32_to_bf16(x):
    """Round float32 to bf16 bit patterns, round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    _lib.orc_round_bf16(_ptr(x), x.size, _ptr(out))
    return out


def topk24(X):
    """TopK(.) of Alg. 1: keep mask [M,K] (uint8 0/1), two per aligned group of 4 along K."""
    X = _u16(X)
    M, K = X.shape
    keep = np.empty((M, K), dtype=np.uint8)
    rc = _lib.orc_topk24(_ptr(X), M, K, K, _ptr(keep))
    if rc:
        raise ValueError("K must be a multiple of 4")
    return keep


def scales(X, keep, scope=GROUP, eps=1e-8):
    """s of Alg. 1 / the norm-compensation equation: [M,K/4] (GROUP), [M] (ROW), [1] (TENSOR)."""
    X = _u16(X)
    M, K = X.shape
    if scope == NONE:
        return np.zeros((0,), dtype=np.float32)
    shape = {GROUP: (M, K // 4), ROW: (M,), TENSOR: (1,)}[scope]
    s = np.empty(shape, dtype=np.float32)
    rc = _lib.orc_scales(_ptr(X), _ptr(keep), M, K, K, scope, eps, _ptr(s))
    assert rc == 0
    return s


def apply_scales(X, keep, s, scope=GROUP, operand_round=True):
    """S(X) = s * X~ as dense masked fp32 [M,K]; also the bf16 bits of every product."""
    X = _u16(X)
    M, K = X.shape
    S = np.empty((M, K), dtype=np.float32)
    Sb = np.empty((M, K), dtype=np.uint16)
    _lib.orc_apply(_ptr(X), _ptr(keep), _ptr(s), M, K, K, scope, int(operand_round), _ptr(S),
                   _ptr(Sb))
    return S, Sb


def pack(D, keep):
    """Compressed operand of App. A: vals [M,K/2] (uint16 bf16 bits), meta [M,K/8] (uint8)."""
    D = _u16(D)
    M, K = D.shape
    vals = np.empty((M, K // 2), dtype=np.uint16)
    meta = np.empty((M, K // 8), dtype=np.uint8)
    rc = _lib.orc_pack(_ptr(D), K, _ptr(np.ascontiguousarray(keep)), M, K, _ptr(vals), _ptr(meta))
    if rc:
        raise ValueError("orc_pack failed (%d): K %% 8 != 0 or a group without exactly 2 kept" % rc)
    return vals, meta


def unpack(vals, meta):
    """Inverse of pack: dense bf16 bits [M,K] with zeros at the dropped positions."""
    vals = _u16(vals)
    meta = np.ascontiguousarray(meta, dtype=np.uint8)
    M, K = vals.shape[0], vals.shape[1] * 2
    D = np.empty((M, K), dtype=np.uint16)
    rc = _lib.orc_unpack(_ptr(vals), _ptr(meta), M, K, _ptr(D))
    assert rc == 0
    return D


def linear(S, W, bias=None, rows=None):
    """Y = S W^T (+ b): fp32 triple loop, k ascending. S fp32 [M,K]; W, bias bf16 bits.

    rows=(m0, m1) restricts the computation to those rows (the others stay zero)."""
    S = np.ascontiguousarray(S, dtype=np.float32)
    W = _u16(W)
    M, K = S.shape
    N = W.shape[0]
    assert W.shape[1] == K
    m0, m1 = (0, M) if rows is None else rows
    Y = np.zeros((M, N), dtype=np.float32)
    b = None if bias is None else _u16(bias)
    rc = _lib.orc_linear(_ptr(S), _ptr(W), _ptr(b), M, N, K, K, m0, m1, _ptr(Y))
    assert rc == 0
    return Y


def rfe(A, B):
    """Relative Frobenius error ||A-B||_F / ||A||_F (appendix RFE metric)."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    return float(_lib.orc_rfe(_ptr(A), _ptr(B), A.size))


def sparsify_pack_oracle(X, scope=GROUP, eps=1e-8):
    """Alg. 1 up to the compressed operand. Returns dict(keep, s, S, vals, meta).

    vals hold the re-rounded s*x for GROUP scope and the untouched kept inputs otherwise
    (ROW/TENSOR scales are constant along the contraction and are applied to Y in fp32)."""
    X = _u16(X)
    keep = topk24(X)
    s = scales(X, keep, scope, eps)
    rounded = scope in (NONE, GROUP)
    S, Sb = apply_scales(X, keep, s, scope, operand_round=rounded)
    vals, meta = pack(Sb if scope == GROUP else X, keep)
    return dict(keep=keep, s=s, S=S, vals=vals, meta=meta)


def sparse_linear_oracle(X, W, bias=None, scope=GROUP, eps=1e-8, rows=None):
    """Alg. 1 without the LoRA branch: Y = S(X) W^T (+ b), fp32 [M,N]."""
    r = sparsify_pack_oracle(X, scope, eps)
    r["Y"] = linear(r["S"], W, bias, rows)
    return r


def dense_linear_oracle(X, W, bias=None, rows=None):
    """Eq. (linear_layer): Y = X W^T (+ b), fp32 [M,N]."""
    return linear(bf16_to_f32(_u16(X)), W, bias, rows)


def lora_delta(LA, LB):
    """Eq. (sparse+lora): the LoRA product L_A L_B as fp32 [N,K]. L_A [N,R], L_B [R,K] bf16 bits."""
    LA, LB = _u16(LA), _u16(LB)
    N, R = LA.shape
    K = LB.shape[1]
    assert LB.shape[0] == R
    D = np.empty((N, K), dtype=np.float32)
    _lib.orc_lora_delta(_ptr(LA), _ptr(LB), N, K, R, _ptr(D))
    return D


def linear_f32w(A, Wf, rows=None):
    """Y = A Wf^T with fp32 operands (fp32 triple loop, k ascending)."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    Wf = np.ascontiguousarray(Wf, dtype=np.float32)
    M, K = A.shape
    N = Wf.shape[0]
    m0, m1 = (0, M) if rows is None else rows
    Y = np.zeros((M, N), dtype=np.float32)
    rc = _lib.orc_linear_f32w(_ptr(A), _ptr(Wf), M, N, K, m0, m1, _ptr(Y))
    assert rc == 0
    return Y


def sparse_lora_linear_oracle(X, W, LA, LB, bias=None, scope=GROUP, eps=1e-8, delta=None):
    """The whole of Alg. 1: Y = S(X) W^T (+ b) + X (L_A L_B)^T, fp32 [M,N].

    `delta` lets a caller reuse the LoRA product L_A L_B across calls (it does not depend on X)."""
    r = sparse_linear_oracle(X, W, bias, scope, eps)
    D = lora_delta(LA, LB) if delta is None else delta
    Yr = linear_f32w(bf16_to_f32(_u16(X)), D)
    Y = np.empty_like(Yr)
    _lib.orc_add(_ptr(r["Y"]), _ptr(Yr), Yr.size, _ptr(Y))
    r["Y_s"], r["Y_r"], r["Y"] = r["Y"], Yr, Y
    return r


# ---- FP8 (E4M3) composition: implementation details, "orthogonal validation with FP8 quantization" ----

def e4m3_encode(x):
    """fp32 -> E4M3 codes (uint8), round-to-nearest-even, saturating at +-448, NaN -> 0x7F."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    _lib.orc_e4m3_encode(_ptr(x), x.size, _ptr(out))
    return out


def e4m3_decode(c):
    """E4M3 codes (uint8) -> fp32."""
    c = np.ascontiguousarray(c, dtype=np.uint8)
    out = np.empty(c.shape, dtype=np.float32)
    _lib.orc_e4m3_decode(_ptr(c), c.size, _ptr(out))
    return out


def quantize_weights_fp8(W):
    """Weights "directly quantized to FP8": the E4M3 code of every bf16 weight, no scale."""
    return e4m3_encode(bf16_to_f32(_u16(W)))


def sparsify_pack_fp8_oracle(X, x_scale, scope=GROUP, eps=1e-8):
    """Alg. 1 up to the compressed operand with FP8 kept values.

    Selection and the compensation factor are those of the bf16 path (they look at the bf16
    input); the kept value is then (s * x) / x_scale quantised once to E4M3.
    Returns dict(keep, s, Q (dense masked codes), vals (codes [M,K/2]), meta)."""
    X = _u16(X)
    M, K = X.shape
    keep = topk24(X)
    s = scales(X, keep, scope, eps)
    Q = np.empty((M, K), dtype=np.uint8)
    _lib.orc_apply_fp8(_ptr(X), _ptr(keep), _ptr(s), M, K, K, scope, float(np.float32(x_scale)), _ptr(Q))
    vals = np.empty((M, K // 2), dtype=np.uint8)
    meta = np.empty((M, K // 8), dtype=np.uint8)
    rc = _lib.orc_pack8(_ptr(Q), _ptr(keep), M, K, _ptr(vals), _ptr(meta))
    assert rc == 0
    return dict(keep=keep, s=s, Q=Q, vals=vals, meta=meta)


def sparse_linear_fp8_oracle(X, Wq, x_scale, bias=None, scope=GROUP, eps=1e-8, rows=None):
    """W8A8 + 2:4 activation sparsity: Y = f * (Q Wq^T) (+ b), fp32 [M,N], with Q the quantised S(X),
    Wq the E4M3 weight codes and f = x_scale (times the ROW / TENSOR compensation factor)."""
    r = sparsify_pack_fp8_oracle(X, x_scale, scope, eps)
    acc = linear_f32w(e4m3_decode(r["Q"]), e4m3_decode(Wq), rows)
    f = np.float32(x_scale)
    if scope == ROW:
        f = (f * r["s"].astype(np.float32))[:, None]
    elif scope == TENSOR:
        f = f * np.float32(r["s"][0])
    Y = (np.float32(1) * f * acc).astype(np.float32)
    if bias is not None:
        Y = Y + bf16_to_f32(_u16(bias))[None, :]
        if rows is not None:
            Y[: rows[0]] = 0
            Y[rows[1]:] = 0
    r["Y"] = Y.astype(np.float32)
    return r


def sparse_lora_linear_fp8_oracle(X, Wq, x_scale, LA, LB, bias=None, scope=GROUP, eps=1e-8, delta=None):
    """The whole of Alg. 1 on FP8 operands: the W8A8 sparse product of sparse_linear_fp8_oracle plus the
    LoRA residual X (L_A L_B)^T of sparse_lora_linear_oracle (bf16 input, bf16 factors, fp32), fp32 [M,N].
    Returns the FP8 oracle's dict with Y_s (sparse product, bias included), Y_r and Y = Y_s + Y_r."""
    r = sparse_linear_fp8_oracle(X, Wq, x_scale, bias, scope, eps)
    D = lora_delta(LA, LB) if delta is None else delta
    Yr = linear_f32w(bf16_to_f32(_u16(X)), D)
    Y = np.empty_like(Yr)
    _lib.orc_add(_ptr(r["Y"]), _ptr(Yr), Yr.size, _ptr(Y))
    r["Y_s"], r["Y_r"], r["Y"] = r["Y"], Yr, Y
    return r

