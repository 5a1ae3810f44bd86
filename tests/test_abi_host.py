"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before touching any memory."""
import ctypes as C
import os
import re

import pytest

from paper_2605_26632_amd import binding as rtl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "rtlynx.h")).read()
    declared = set(re.findall(r"\b(rtl_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(rtl.SYMBOLS), declared ^ set(rtl.SYMBOLS)
    L = rtl.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert rtl.version().startswith("rtlynx-gfx950")


def test_status_strings():
    for s in range(8):
        assert rtl.status_str(s).startswith("RTL_")
    assert rtl.status_str(7).startswith("RTL_ERR_ARCH") and rtl.status_str(99) == "RTL_ERR_UNKNOWN"


def test_init_reports_a_status_without_a_gpu():
    """rtl_init never aborts: without a usable device it reports RTL_ERR_HIP, on another AMD GPU
    RTL_ERR_ARCH, on a gfx950 device RTL_OK."""
    assert rtl.lib().rtl_init() in (0, 6, 7)


FAKE = 0x10000  # non-null, 256-byte aligned, never dereferenced: validation precedes any launch


def test_sparsify_pack_rejects_bad_arguments():
    L = rtl.lib()
    f = L.rtl_sparsify_pack
    ok_args = dict(X=FAKE, M=4, K=64, ldx=64, comp=1, eps=1e-8, vals=FAKE, meta=FAKE, scale=None,
                   ws=None, wsb=0, stream=None)

    def call(**kw):
        a = dict(ok_args, **kw)
        return f(a["X"], a["M"], a["K"], a["ldx"], a["comp"], a["eps"], a["vals"], a["meta"],
                 a["scale"], a["ws"], a["wsb"], a["stream"])

    assert call(K=12) == 2 and call(K=60) == 2          # K % 8
    assert call(ldx=32) == 2 and call(M=-1) == 2
    assert call(X=None) == 1 and call(vals=None) == 1 and call(meta=None) == 1
    assert call(comp=2) == 1 and call(comp=3) == 1       # ROW / TENSOR need `scale`
    assert call(X=FAKE + 2) == 3 and call(ldx=68) == 3
    assert call(comp=7) == 5 and call(eps=-1.0) == 5 and call(eps=float("nan")) == 5
    assert call(comp=3, scale=FAKE) == 4                 # TENSOR needs workspace
    assert call(comp=3, scale=FAKE, ws=FAKE, wsb=8) == 4
    assert call(M=0) == 0                                # empty input: OK, nothing launched
    assert L.rtl_sparsify_pack_workspace(100, 64, 3) == 800
    assert L.rtl_sparsify_pack_workspace(100, 64, 1) == 0


def test_linear_entry_points_reject_bad_arguments():
    L = rtl.lib()

    def dense(X=FAKE, W=FAKE, bias=None, Y=FAKE, M=4, N=4, K=64, ldx=64, ldw=64, ldy=4, ws=FAKE, wsb=1 << 30):
        return L.rtl_dense_linear(X, W, bias, Y, M, N, K, ldx, ldw, ldy, ws, wsb, None)

    def sparse(X=FAKE, W=FAKE, bias=None, Y=FAKE, M=4, N=4, K=64, ldx=64, ldw=64, ldy=4, comp=1,
               eps=1e-8, ws=FAKE, wsb=1 << 30):
        return L.rtl_sparse_linear(X, W, bias, Y, M, N, K, ldx, ldw, ldy, comp, eps, ws, wsb, None)

    for f in (dense, sparse):
        assert f(K=32) == 2 and f(K=0) == 2 and f(ldy=2) == 2 and f(ldw=32) == 2 and f(N=-3) == 2
        assert f(X=None) == 1 and f(W=None) == 1 and f(Y=None) == 1
        assert f(W=FAKE + 8) == 3 and f(ldx=68) == 3 and f(Y=FAKE + 1) == 3
        assert f(M=0) == 0 and f(N=0) == 0
    for f in (dense, sparse):        # more output tiles than a 32-bit grid index can number
        assert f(M=1 << 30, N=1 << 30, ldy=1 << 30) == 2
    for f in (dense, sparse):        # strides beyond the 32-bit tile-offset range are refused
        assert f(ldx=(1 << 22) + 8) == 2 and f(ldw=(1 << 22) + 8) == 2
    assert sparse(comp=9) == 5 and sparse(eps=float("inf")) == 5
    assert sparse(ws=None) == 4 and sparse(wsb=16) == 4 and sparse(ws=FAKE + 64) == 3
    need = L.rtl_sparse_linear_workspace(4096, 3072, 12288, 1)
    assert need >= 4096 * 12288 + 4096 * 12288 // 8

    def packed(vals=FAKE, meta=FAKE, W=FAKE, Y=FAKE, M=4, N=4, K=64, ldw=64, ldy=4):
        return L.rtl_packed_linear(vals, meta, None, None, W, None, Y, M, N, K, ldw, ldy, FAKE, 1 << 30, None)

    def lora(LA=FAKE, LB=FAKE, R=64, ldla=64, ldlb=64, ws=FAKE, wsb=1 << 30, K=64):
        return L.rtl_sparse_lora_linear(FAKE, FAKE, LA, LB, None, FAKE, 4, 4, K, R, K, K, ldla, ldlb, 4, 1, 1e-8,
                                        ws, wsb, None)

    assert lora(R=32) == 2 and lora(R=128) == 2 and lora(ldla=32) == 2 and lora(ldlb=32) == 2
    assert lora(LA=None) == 1 and lora(LB=None) == 1 and lora(LA=FAKE + 8) == 3 and lora(wsb=64) == 4
    assert L.rtl_sparse_lora_linear_workspace(4096, 3072, 12288, 64, 1) > L.rtl_sparse_linear_workspace(4096, 3072, 12288, 1)
    assert L.rtl_sparse_lora_linear_workspace(4096, 3072, 12288, 32, 1) == 0

    assert packed(meta=None) == 1 and packed(vals=None) == 1 and packed(K=96) == 2
    assert packed(meta=FAKE + 4) == 3 and packed(M=0) == 0


def test_fp8_entry_points_reject_bad_arguments():
    L = rtl.lib()

    def quant(W=FAKE, rows=4, cols=64, ld=64, Wq=FAKE, ldq=64):
        return L.rtl_quantize_fp8(W, rows, cols, ld, Wq, ldq, None)

    assert quant(cols=12) == 2 and quant(ld=32) == 2 and quant(ldq=32) == 2 and quant(rows=-1) == 2
    assert quant(W=None) == 1 and quant(Wq=None) == 1
    assert quant(W=FAKE + 2) == 3 and quant(Wq=FAKE + 4) == 3 and quant(ld=68) == 3
    assert quant(rows=0) == 0

    def pack(X=FAKE, M=4, K=64, ldx=64, comp=1, eps=1e-8, xs=FAKE, vals=FAKE, meta=FAKE, scale=None,
             ws=None, wsb=0):
        return L.rtl_sparsify_pack_fp8(X, M, K, ldx, comp, eps, xs, vals, meta, scale, ws, wsb, None)

    assert pack(K=12) == 2 and pack(ldx=32) == 2
    assert pack(xs=None) == 1 and pack(vals=None) == 1 and pack(comp=2) == 1
    assert pack(vals=FAKE + 2) == 3 and pack(xs=FAKE + 2) == 3
    assert pack(comp=5) == 5 and pack(eps=-1.0) == 5
    assert pack(comp=3, scale=FAKE) == 4
    assert pack(M=0) == 0

    def lin(X=FAKE, Wq=FAKE, xs=FAKE, Y=FAKE, M=4, N=4, K=128, ldx=128, ldw=128, ldy=4, comp=1, eps=1e-8,
            ws=FAKE, wsb=1 << 30):
        return L.rtl_sparse_linear_fp8(X, Wq, xs, None, Y, M, N, K, ldx, ldw, ldy, comp, eps, ws, wsb, None)

    assert lin(K=64, ldx=64, ldw=64) == 2 and lin(ldw=64) == 2 and lin(ldy=2) == 2
    assert lin(X=None) == 1 and lin(Wq=None) == 1 and lin(xs=None) == 1
    assert lin(ldw=136) == 3 and lin(Wq=FAKE + 8) == 3
    assert lin(comp=4) == 5
    assert lin(ws=None) == 4 and lin(wsb=8) == 4
    assert lin(M=0) == 0
    # half the value bytes of the bf16 workspace, same metadata
    assert L.rtl_sparse_linear_fp8_workspace(4096, 3072, 12288, 1) < L.rtl_sparse_linear_workspace(4096, 3072, 12288, 1)

    def lora(X=FAKE, Wq=FAKE, xs=FAKE, LA=FAKE, LB=FAKE, Y=FAKE, M=4, N=8, K=128, R=64, ldx=128, ldw=128, ldla=64,
             ldlb=128, ldy=8, comp=1, eps=1e-8, ws=FAKE, wsb=1 << 30):
        return L.rtl_sparse_lora_linear_fp8(X, Wq, xs, LA, LB, None, Y, M, N, K, R, ldx, ldw, ldla, ldlb, ldy, comp,
                                            eps, ws, wsb, None)

    assert lora(R=32) == 2 and lora(ldla=32) == 2 and lora(ldlb=64) == 2 and lora(K=64, ldx=64, ldw=64, ldlb=64) == 2
    assert lora(X=None) == 1 and lora(xs=None) == 1 and lora(LA=None) == 1 and lora(LB=None) == 1
    assert lora(LA=FAKE + 8) == 3 and lora(ldla=68) == 3 and lora(ldw=136) == 3 and lora(xs=FAKE + 2) == 3
    assert lora(comp=7) == 5 and lora(eps=float("nan")) == 5
    assert lora(ws=None) == 4 and lora(wsb=64) == 4
    assert lora(M=0) == 0 and lora(N=0) == 0
    need = L.rtl_sparse_lora_linear_fp8_workspace(4096, 3072, 12288, 64, 1)
    assert need > L.rtl_sparse_linear_fp8_workspace(4096, 3072, 12288, 1)       # + T planes + sweep scratch
    assert L.rtl_sparse_lora_linear_fp8_workspace(4096, 3072, 12288, 32, 1) == 0  # rank other than 64


def test_tile_plan_covers_the_output_exactly():
    """Host arithmetic of the launch plan: body tiles (256 x 256 or 256 x 192) on the first rows, 256 x 128
    tail tiles on the rest; together they cover every output element once, for any shape."""
    import random
    rnd = random.Random(5)
    shapes = [(4096, 3072), (4608, 12288), (16896, 3072), (1, 1), (255, 129), (257, 193), (100003, 40), (40, 70001)]
    shapes += [(rnd.randint(1, 20000), rnd.randint(1, 20000)) for _ in range(200)]
    for M, N in shapes:
        for dense in (False, True):
            p = rtl.diag_tile_plan(M, N, dense)
            assert p["body_width"] in (192, 256)
            tm = (M + 255) // 256
            rows = p["body_rows"]
            assert 0 <= rows <= M and (rows % 256 == 0 or rows == M)
            body_panels = (rows + 255) // 256
            assert p["body_tiles"] == body_panels * ((N + p["body_width"] - 1) // p["body_width"])
            assert p["tail_tiles"] == (tm - body_panels) * ((N + 127) // 128)
            assert p["body_tiles"] + p["tail_tiles"] >= 1
            if p["tail_tiles"] == 0:
                assert rows == M
    assert rtl.lib().rtl_diag_tile_plan(0, 5, 0, None) == 2 and rtl.lib().rtl_diag_tile_plan(5, 5, 0, None) == 1
    # the headline shape keeps its one-round plan: 256 tiles of 256 x 192, no tail
    assert rtl.diag_tile_plan(4096, 3072) == dict(body_width=192, body_rows=4096, body_tiles=256, tail_tiles=0)
