"""Pins for the CPU oracle: closed forms, hand cases, invariants, brute force, library routines.

Every check here compares the oracle with something that is not the oracle: a second formulation
of the selection rule, values worked by hand from the paper's definitions (tests/golden), exact
closed forms, numpy's fp64 matmul. No GPU involved.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_2605_26632_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
VALID_NIBBLES = {0x4, 0x8, 0x9, 0xC, 0xD, 0xE}


def bf(x):
    return oracle.f32_to_bf16(np.asarray(x, dtype=np.float32))


def second_opinion_keep(Xf):
    """Independent formulation: stable sort of each group by descending |x|, first two win."""
    M, K = Xf.shape
    g = np.abs(Xf.astype(np.float64)).reshape(M, K // 4, 4)
    order = np.argsort(-g, axis=2, kind="stable")
    keep = np.zeros_like(g, dtype=np.uint8)
    np.put_along_axis(keep, order[:, :, :2], 1, axis=2)
    return keep.reshape(M, K)


# ---------------------------------------------------------------- bf16 helpers
def test_bf16_round_trip_and_rne():
    # every finite bf16 pattern survives widen -> round
    allbits = np.arange(0, 0x10000, dtype=np.uint32).astype(np.uint16)
    finite = allbits[(allbits & 0x7F80) != 0x7F80]
    assert np.array_equal(oracle.f32_to_bf16(oracle.bf16_to_f32(finite)), finite)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.bf16_to_f32(bf([1 + 2.0 ** -8]))[0] == 1.0
    assert oracle.bf16_to_f32(bf([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6
    assert oracle.bf16_to_f32(bf([1 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1 + 2.0 ** -7
    # matches torch's conversion on random data
    import torch
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    t = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(synth.bits(t), bf(x))


# ---------------------------------------------------------------- selection
def test_selection_brute_force_all_tuples():
    vals = np.array([-2.0, -1.0, -0.0, 0.0, 0.5, 1.0, 2.0], dtype=np.float32)
    groups = np.array(list(itertools.product(vals, repeat=4)), dtype=np.float32)  # 2401 x 4
    keep = oracle.topk24(bf(groups))
    assert np.array_equal(keep, second_opinion_keep(groups))
    assert np.all(keep.sum(axis=1) == 2)


def test_selection_hand_cases_and_golden_file():
    rows = []
    with open(os.path.join(GOLDEN, "topk24_hand_cases.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            x, pos, nib, s, kept = [p.split() for p in line.split("|")]
            rows.append(([float(v) for v in x], [int(p) for p in pos], int(nib[0], 16),
                         float(s[0]), [float(v) for v in kept]))
    assert len(rows) == 10
    # the byte-wide metadata needs K % 8 == 0: a zero group is appended to every case
    X = bf([r[0] + [0.0] * 4 for r in rows])
    out = oracle.sparsify_pack_oracle(X, scope=oracle.GROUP)
    for i, (x, pos, nib, s, kept) in enumerate(rows):
        assert list(np.flatnonzero(out["keep"][i, :4])) == pos, x
        assert out["meta"][i, 0] & 0xF == nib, x
        assert out["s"][i, 0] == pytest.approx(s, rel=3e-7, abs=1e-12), x
        assert list(oracle.bf16_to_f32(out["vals"][i, :2])) == kept, x
        assert out["meta"][i, 0] >> 4 == 0x4 and not out["vals"][i, 2:].any()


def test_selection_special_values():
    inf, nan = np.inf, np.nan
    X = bf([[1.0, inf, -inf, 2.0], [nan, 1.0, inf, 0.0], [-0.0, 0.0, -0.0, 0.0],
            [1e-40, -1e-40, 0.0, 0.0]])
    keep = oracle.topk24(X)
    assert keep.tolist() == [[0, 1, 1, 0], [1, 0, 1, 0], [1, 1, 0, 0], [1, 1, 0, 0]]


@pytest.mark.parametrize("kind", ["laplace_outlier", "gelu", "normal"])
def test_selection_invariants_random(kind):
    X = synth.bits(synth.activations(kind, 64, 1024, seed=3))
    keep = oracle.topk24(X).reshape(64, 256, 4).astype(bool)
    key = (X & 0x7FFF).reshape(64, 256, 4).astype(np.int32)
    assert np.all(keep.sum(axis=2) == 2)
    kmin = np.where(keep, key, 1 << 20).min(axis=2)
    dmax = np.where(~keep, key, -1).max(axis=2)
    assert np.all(kmin >= dmax)
    # on a tie between a kept and a dropped element the dropped one sits at the larger index
    idx = np.arange(4)[None, None, :]
    tie = kmin == dmax
    last_kept_tied = np.where(keep & (key == kmin[..., None]), idx, -1).max(axis=2)
    first_drop_tied = np.where(~keep & (key == dmax[..., None]), idx, 9).min(axis=2)
    assert np.all(first_drop_tied[tie] > last_kept_tied[tie])
    assert np.array_equal(keep.reshape(64, 1024), second_opinion_keep(oracle.bf16_to_f32(X)) > 0)


# ---------------------------------------------------------------- pack / unpack
def test_pack_layout_and_round_trip():
    X = synth.bits(synth.activations("laplace", 32, 256, seed=5))
    r = oracle.sparsify_pack_oracle(X, scope=oracle.NONE)
    vals, meta, keep = r["vals"], r["meta"], r["keep"]
    assert vals.shape == (32, 128) and meta.shape == (32, 32)
    nibs = np.stack([meta & 0xF, meta >> 4], axis=-1).reshape(32, 64)
    assert set(np.unique(nibs)) <= VALID_NIBBLES
    p0, p1 = nibs & 3, nibs >> 2
    assert np.all(p0 < p1)
    # positions named by the metadata are the kept ones, and values equal the originals
    g = np.arange(64)[None, :] * 4
    rows = np.arange(32)[:, None]
    assert np.all(keep[rows, g + p0] == 1) and np.all(keep[rows, g + p1] == 1)
    assert np.array_equal(vals[:, 0::2], X[rows, g + p0])
    assert np.array_equal(vals[:, 1::2], X[rows, g + p1])
    # round trip: unpack(pack(X)) == mask * X, bit for bit
    assert np.array_equal(oracle.unpack(vals, meta), np.where(keep > 0, X, 0).astype(np.uint16))


# ---------------------------------------------------------------- compensation
def test_compensation_closed_forms():
    X = bf([[1, 1, 1, 1], [0, 0, 0, 0], [0, 6, 0, -2], [3, -4, 1, 0]])
    keep = oracle.topk24(X)
    s = oracle.scales(X, keep, oracle.GROUP)[:, 0]
    assert s[0] == np.float32(np.sqrt(np.float32(4) / (np.float32(2) + np.float32(1e-8))))
    assert s[0] == pytest.approx(np.sqrt(2.0), rel=1e-7)
    assert s[1] == 0.0                       # all-zero group: 0 / eps -> 0, no NaN
    assert s[2] == pytest.approx(1.0, rel=1e-7)   # already 2-sparse: nothing to restore
    assert s[3] == pytest.approx(np.sqrt(26.0 / 25.0), rel=1e-7)
    # eps matters for tiny magnitudes: |x| = 1e-4 -> kept norm 2e-8, s = sqrt(4e-8/(2e-8+1e-8))
    t = bf([[1e-4, 1e-4, 1e-4, 1e-4]])
    tv = float(oracle.bf16_to_f32(t)[0, 0])
    st = oracle.scales(t, oracle.topk24(t), oracle.GROUP)[0, 0]
    assert st == pytest.approx(np.sqrt(4 * tv * tv / (2 * tv * tv + 1e-8)), rel=1e-6)


@pytest.mark.parametrize("scope", [oracle.GROUP, oracle.ROW, oracle.TENSOR])
def test_compensation_restores_norm(scope):
    X = synth.bits(synth.activations("laplace_outlier", 48, 512, seed=7))
    Xf = oracle.bf16_to_f32(X).astype(np.float64)
    keep = oracle.topk24(X)
    s = oracle.scales(X, keep, scope)
    S, _ = oracle.apply_scales(X, keep, s, scope, operand_round=False)
    S = S.astype(np.float64)
    kept2 = np.where(keep > 0, Xf, 0.0) ** 2
    shape = {oracle.GROUP: (48, 128, 4), oracle.ROW: (48, 1, 512), oracle.TENSOR: (1, 1, 48 * 512)}[scope]
    full = (Xf ** 2).reshape(shape).sum(axis=2)
    kn = kept2.reshape(shape).sum(axis=2)
    got = (S ** 2).reshape(shape).sum(axis=2)
    want = full * kn / (kn + 1e-8)           # the identity implied by the definition of s
    assert np.allclose(got, want, rtol=5e-6, atol=1e-12)
    # eps is negligible at these magnitudes, so the norm of every scope is restored
    big = kn > 1e-3
    assert np.allclose(got[big], full[big], rtol=1e-4)
    # finer scopes imply the coarser ones: whole-tensor norm is restored as well
    assert np.isclose((S ** 2).sum(), (Xf ** 2).sum(), rtol=1e-4)
    # independent fp64 evaluation of s itself
    s64 = np.sqrt(full / (kn + 1e-8)).reshape(s.shape)
    assert np.allclose(s, s64, rtol=3e-7, atol=1e-12)


def test_compensation_never_changes_the_mask_and_none_is_identity():
    X = synth.bits(synth.activations("gelu", 16, 256, seed=9))
    a = oracle.sparsify_pack_oracle(X, scope=oracle.NONE)
    b = oracle.sparsify_pack_oracle(X, scope=oracle.GROUP)
    assert np.array_equal(a["meta"], b["meta"]) and np.array_equal(a["keep"], b["keep"])
    assert np.array_equal(oracle.unpack(a["vals"], a["meta"]), np.where(a["keep"] > 0, X, 0))
    # GROUP values are the re-rounded products s * x
    sg = np.repeat(b["s"], 2, axis=1)
    assert np.array_equal(b["vals"], bf(sg * oracle.bf16_to_f32(a["vals"])))
    # s lies in [0, sqrt(2)]: the two kept entries carry at least half of the group's energy
    assert b["s"].min() >= 0 and b["s"].max() <= np.float32(np.sqrt(2.0)) * (1 + 1e-6)


# ---------------------------------------------------------------- GEMM
def test_linear_matches_fp64_matmul_and_is_not_transposed():
    X, W = synth.activations("normal", 24, 96, 1), synth.weights(40, 96, 2, std=1.0)
    Xb, Wb = synth.bits(X), synth.bits(W)
    Y = oracle.dense_linear_oracle(Xb, Wb)
    ref = oracle.bf16_to_f32(Xb).astype(np.float64) @ oracle.bf16_to_f32(Wb).astype(np.float64).T
    assert Y.shape == (24, 40)
    assert np.allclose(Y, ref, rtol=0, atol=2e-5 * np.abs(ref).max())
    b = synth.bits(synth.bias(40, 3, std=1.0))
    Yb = oracle.dense_linear_oracle(Xb, Wb, bias=b)
    assert np.allclose(Yb, ref + oracle.bf16_to_f32(b)[None, :], atol=2e-5 * np.abs(ref).max())
    part = oracle.dense_linear_oracle(Xb, Wb, rows=(5, 9))
    assert np.array_equal(part[5:9], Y[5:9]) and not part[:5].any() and not part[9:].any()


def test_linear_one_hot_rows_read_back_weight_rows():
    K, N = 64, 48
    Wb = synth.bits(synth.weights(N, K, 4, std=1.0))
    X = np.zeros((K, K), dtype=np.float32)
    X[np.arange(K), np.arange(K)] = 1.0
    Y = oracle.sparse_linear_oracle(bf(X), Wb, scope=oracle.NONE)["Y"]
    assert np.array_equal(Y, oracle.bf16_to_f32(Wb).T)     # row k of Y is column k of W


def test_sparse_linear_equals_dense_gemm_of_masked_input():
    X, W = synth.workload("tiny", seed=0, M=32)
    Xb, Wb = synth.bits(X), synth.bits(W)
    for scope in (oracle.NONE, oracle.GROUP, oracle.ROW, oracle.TENSOR):
        r = oracle.sparse_linear_oracle(Xb, Wb, scope=scope)
        ref = r["S"].astype(np.float64) @ oracle.bf16_to_f32(Wb).astype(np.float64).T
        assert np.allclose(r["Y"], ref, rtol=0, atol=3e-5 * np.abs(ref).max())
        # the compressed operand decodes to the same matrix the GEMM consumed
        dec = oracle.bf16_to_f32(oracle.unpack(r["vals"], r["meta"])).astype(np.float64)
        if scope == oracle.ROW:
            dec = dec * r["s"][:, None]
        elif scope == oracle.TENSOR:
            dec = dec * r["s"][0]
        assert np.allclose(dec, r["S"], rtol=1e-6, atol=0)


def test_already_sparse_input_reduces_to_plain_gemm():
    X, W = synth.workload("tiny", seed=1, M=16)
    Xb, Wb = synth.bits(X), synth.bits(W)
    keep = oracle.topk24(Xb)
    Xs = np.where(keep > 0, Xb, 0).astype(np.uint16)      # exactly 2:4 sparse already
    Y = oracle.sparse_linear_oracle(Xs, Wb, scope=oracle.NONE)["Y"]
    ref = oracle.bf16_to_f32(Xs).astype(np.float64) @ oracle.bf16_to_f32(Wb).astype(np.float64).T
    assert np.allclose(Y, ref, rtol=0, atol=3e-5 * np.abs(ref).max())
    assert np.array_equal(Y, oracle.dense_linear_oracle(Xs, Wb))


def test_rfe_definition_and_sanity_on_config_inputs():
    a = np.array([3.0, 4.0], dtype=np.float32)
    assert oracle.rfe(a, np.array([3.0, 0.0], dtype=np.float32)) == pytest.approx(0.8)
    X, W = synth.workload("mlp_down", seed=0, M=8)
    Xb, Wb = synth.bits(X), synth.bits(W)
    dense = oracle.dense_linear_oracle(Xb, Wb)
    e_none = oracle.rfe(dense, oracle.sparse_linear_oracle(Xb, Wb, scope=oracle.NONE)["Y"])
    e_grp = oracle.rfe(dense, oracle.sparse_linear_oracle(Xb, Wb, scope=oracle.GROUP)["Y"])
    assert 0 < e_none < 0.6 and 0 < e_grp < 0.6   # an approximation, but not garbage


# ---------------------------------------------------------------- LoRA branch (Eq. sparse+lora)
def test_lora_branch_matches_fp64_and_is_low_rank():
    X, W = synth.workload("tiny", seed=5, M=40)
    LA, LB = synth.lora(W.shape[0], W.shape[1], 16, seed=6, std_a=1.0, std_b=1.0)
    Xb, Wb, LAb, LBb = (synth.bits(t) for t in (X, W, LA, LB))
    r = oracle.sparse_lora_linear_oracle(Xb, Wb, LAb, LBb, scope=oracle.GROUP)
    Xf = oracle.bf16_to_f32(Xb).astype(np.float64)
    A64 = oracle.bf16_to_f32(LAb).astype(np.float64)
    B64 = oracle.bf16_to_f32(LBb).astype(np.float64)
    ref_r = Xf @ (A64 @ B64).T
    assert np.allclose(r["Y_r"], ref_r, rtol=0, atol=3e-5 * np.abs(ref_r).max())
    # (X L_B^T) L_A^T is the same map: the order of the two small products does not matter
    assert np.allclose((Xf @ B64.T) @ A64.T, ref_r, rtol=1e-9, atol=1e-9 * np.abs(ref_r).max())
    assert np.linalg.matrix_rank(r["Y_r"].astype(np.float64), tol=1e-3 * np.abs(ref_r).max()) <= 16
    # the sum is the sparse output plus the residual, nothing else
    base = oracle.sparse_linear_oracle(Xb, Wb, scope=oracle.GROUP)["Y"]
    assert np.array_equal(r["Y_s"], base)
    assert np.allclose(r["Y"], base.astype(np.float64) + ref_r, rtol=0, atol=3e-5 * np.abs(ref_r).max())


def test_lora_special_cases():
    X, W = synth.workload("tiny", seed=7, M=24)
    Xb, Wb = synth.bits(X), synth.bits(W)
    N, K = W.shape
    # zero L_A: the branch vanishes and Alg. 1 is the sparse linear alone
    LA0 = np.zeros((N, 8), dtype=np.uint16)
    LB = synth.bits(synth.lora(N, K, 8, seed=8)[1])
    r0 = oracle.sparse_lora_linear_oracle(Xb, Wb, LA0, LB, scope=oracle.NONE)
    assert np.array_equal(r0["Y"], oracle.sparse_linear_oracle(Xb, Wb, scope=oracle.NONE)["Y"])
    # full-rank "LoRA" with L_B = I and L_A = W: the residual is the dense layer itself
    eye = bf(np.eye(K, dtype=np.float32))
    r1 = oracle.sparse_lora_linear_oracle(Xb, Wb, Wb, eye, scope=oracle.NONE)
    dense = oracle.dense_linear_oracle(Xb, Wb)
    assert np.allclose(r1["Y_r"], dense, rtol=0, atol=3e-5 * np.abs(dense).max())
    # the residual uses the un-sparsified X: it differs from feeding the masked activation
    keep = oracle.topk24(Xb)
    Xs = np.where(keep > 0, Xb, 0).astype(np.uint16)
    assert not np.allclose(oracle.linear_f32w(oracle.bf16_to_f32(Xs), oracle.lora_delta(Wb, eye)), dense,
                           atol=1e-3 * np.abs(dense).max())


# ---------------------------------------------------------------- FP8 (E4M3) composition
def test_e4m3_decode_closed_forms_and_library():
    """Code values from the format definition (bias 7, 3 mantissa bits, subnormals, no inf) and
    torch's own E4M3 view as a second implementation."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    dec = oracle.e4m3_decode(codes)
    hand = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125,
            0x40: 2.0, 0x64: 48.0, 0x68: 64.0, 0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0}
    for c, v in hand.items():
        assert dec[c] == np.float32(v), hex(c)
    assert np.isnan(dec[0x7F]) and np.isnan(dec[0xFF])
    assert np.signbit(dec[0x80]) and dec[0x80] == 0.0
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    ok = ~np.isnan(lib)
    assert np.array_equal(np.isnan(dec), np.isnan(lib))
    assert np.array_equal(dec[ok], lib[ok])
    # positive codes are strictly increasing in value
    assert np.all(np.diff(dec[:0x7F]) > 0)


def test_e4m3_encode_rounding_saturation_and_library():
    import torch
    # round trip: every non-NaN code is a fixed point
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    assert np.array_equal(oracle.e4m3_encode(oracle.e4m3_decode(codes)), codes)
    # ties go to the even mantissa; just off a tie goes to the nearer neighbour
    hand = [(1.0625, 0x38), (1.1875, 0x3A), (np.nextafter(np.float32(1.0625), np.float32(2)), 0x39),
            (np.nextafter(np.float32(1.1875), np.float32(0)), 0x39),
            (2.0 ** -10, 0x00), (3 * 2.0 ** -10, 0x02), (np.nextafter(np.float32(2.0 ** -10), np.float32(1)), 0x01),
            (15.5 * 2.0 ** -9 / 2, 0x08),              # 7.75 quanta -> 8 quanta = smallest normal
            (0.9999, 0x38), (-3.0594, 0xC4), (48.95, 0x64), (-65.27, 0xE8),
            (448.0, 0x7E), (449.0, 0x7E), (463.9, 0x7E), (464.0, 0x7E), (1e9, 0x7E), (np.inf, 0x7E),
            (-np.inf, 0xFE), (-1e30, 0xFE), (np.nan, 0x7F), (-0.0, 0x80), (1e-12, 0x00)]
    got = oracle.e4m3_encode(np.array([h[0] for h in hand], dtype=np.float32))
    for (v, want), g in zip(hand, got):
        assert g == want, (v, hex(g), hex(want))
    # second implementation: torch's conversion on everything it can represent (it has no saturation)
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(200000) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)]).astype(np.float32)
    x = x[np.abs(x) < 448.0]
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.e4m3_encode(x), lib)
    # every midpoint between neighbouring codes and its two fp32 neighbours
    v = oracle.e4m3_decode(np.arange(0x7F, dtype=np.uint8)).astype(np.float64)
    mids = ((v[:-1] + v[1:]) / 2).astype(np.float32)
    pts = np.concatenate([mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9))])
    pts = np.concatenate([pts, -pts])
    lib = torch.from_numpy(pts).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.e4m3_encode(pts), lib)
    # monotone
    xs = np.sort(x)
    assert np.all(np.diff(oracle.e4m3_decode(oracle.e4m3_encode(xs))) >= 0)


def test_fp8_sparsify_hand_case_and_invariants():
    # (3,-4,1,0): keeps 3 and -4, s = sqrt(26/(25+1e-8)) = 1.0198039; with x_scale 1/16 the scaled
    # values are 48.95 and -65.27 -> 48 (0x64) and -64 (0xE8). (1,1,1,1): s = sqrt(2), 16*1.41421 = 22.63 -> 22 (0x5B)
    Xf = np.array([[3, -4, 1, 0, 1, 1, 1, 1]], dtype=np.float32)
    r = oracle.sparsify_pack_fp8_oracle(bf(Xf), 1.0 / 16.0, scope=oracle.GROUP)
    assert r["keep"].tolist() == [[1, 1, 0, 0, 1, 1, 0, 0]]
    assert r["vals"].tolist() == [[0x64, 0xE8, 0x5B, 0x5B]]
    assert r["meta"].tolist() == [[0x44]]
    assert r["Q"].tolist() == [[0x64, 0xE8, 0, 0, 0x5B, 0x5B, 0, 0]]
    # without compensation the codes are those of x / x_scale: 48 and -64 exactly
    r0 = oracle.sparsify_pack_fp8_oracle(bf(Xf), 1.0 / 16.0, scope=oracle.NONE)
    assert r0["vals"].tolist() == [[0x64, 0xE8, 0x58, 0x58]]
    # random input: same mask and metadata as the bf16 path, dropped entries are code 0, kept entries
    # decode to within half a quantum (2^-4 relative) of the fp32 value they quantise
    X, _ = synth.workload("tiny", seed=4, M=64)
    Xb = synth.bits(X)
    amax = np.abs(oracle.bf16_to_f32(Xb)).max()
    x_scale = np.float32(amax * np.sqrt(2.0) / 448.0)
    for scope in (oracle.NONE, oracle.GROUP, oracle.ROW, oracle.TENSOR):
        r8 = oracle.sparsify_pack_fp8_oracle(Xb, x_scale, scope=scope)
        r16 = oracle.sparsify_pack_oracle(Xb, scope=scope)
        assert np.array_equal(r8["keep"], r16["keep"]) and np.array_equal(r8["meta"], r16["meta"])
        assert np.all(r8["Q"][r8["keep"] == 0] == 0)
        target = oracle.bf16_to_f32(Xb).astype(np.float64)
        if scope == oracle.GROUP:
            target = target * np.repeat(r8["s"].astype(np.float64), 4, axis=1)
        target = np.where(r8["keep"] > 0, target, 0.0) / np.float64(x_scale)
        assert np.abs(target).max() <= 448.0 * (1 + 1e-6)          # sqrt(2) * amax bounds s * x
        dec = oracle.e4m3_decode(r8["Q"]).astype(np.float64)
        quantum = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(target), 2.0 ** -6))) - 3), 2.0 ** -9)
        assert np.all(np.abs(dec - target) <= 0.5 * quantum * (1 + 1e-5))
    # saturation instead of overflow when the scale is too small
    rs = oracle.sparsify_pack_fp8_oracle(bf(np.array([[1000, -2000, 1, 0, 0, 0, 0, 0]], dtype=np.float32)), 1.0, scope=oracle.NONE)
    assert rs["vals"].tolist() == [[0x7E, 0xFE, 0, 0]]


def test_fp8_sparse_linear_reduces_to_integer_matmul_and_fp64():
    rng = np.random.default_rng(5)
    # already 2:4 sparse small integers, integer weights, scale 1, no compensation: everything is exact
    M, K, N = 8, 64, 16
    Xi = rng.integers(-8, 9, size=(M, K))
    Xi.reshape(M, K // 4, 4)[:, :, 2:] = 0
    Xi[Xi == 0] = 1
    Xi.reshape(M, K // 4, 4)[:, :, 2:] = 0
    Wi = rng.integers(-8, 9, size=(N, K))
    Wq = oracle.quantize_weights_fp8(bf(Wi.astype(np.float32)))
    assert np.array_equal(oracle.e4m3_decode(Wq), Wi.astype(np.float32))
    Y = oracle.sparse_linear_fp8_oracle(bf(Xi.astype(np.float32)), Wq, 1.0, scope=oracle.NONE)["Y"]
    assert np.array_equal(Y, (Xi @ Wi.T).astype(np.float32))
    # general input: equals the fp64 product of the decoded operands times the factors, and is
    # not transposed; bias is added last
    X, W = synth.workload("tiny", seed=6, M=16)
    Xb, Wb = synth.bits(X), synth.bits(W)
    Wq = oracle.quantize_weights_fp8(Wb)
    bias = bf(rng.standard_normal(W.shape[0]).astype(np.float32))
    x_scale = np.float32(np.abs(oracle.bf16_to_f32(Xb)).max() * np.sqrt(2.0) / 448.0)
    for scope in (oracle.NONE, oracle.GROUP, oracle.ROW, oracle.TENSOR):
        r = oracle.sparse_linear_fp8_oracle(Xb, Wq, x_scale, bias=bias, scope=scope)
        f = np.float64(x_scale)
        if scope == oracle.ROW:
            f = f * r["s"].astype(np.float64)[:, None]
        elif scope == oracle.TENSOR:
            f = f * np.float64(r["s"][0])
        ref = f * (oracle.e4m3_decode(r["Q"]).astype(np.float64) @ oracle.e4m3_decode(Wq).astype(np.float64).T)
        ref = ref + oracle.bf16_to_f32(bias).astype(np.float64)[None, :]
        assert np.allclose(r["Y"], ref, rtol=0, atol=3e-5 * np.abs(ref).max())
    # the quantised path approximates the bf16 sparse path (sanity, not a gate of the paper)
    y16 = oracle.sparse_linear_oracle(Xb, Wb, scope=oracle.GROUP)["Y"]
    y8 = oracle.sparse_linear_fp8_oracle(Xb, Wq, x_scale, scope=oracle.GROUP)["Y"]
    assert oracle.rfe(y16, y8) < 0.1


def test_fp8_lora_composition_is_the_sum_of_its_two_pinned_parts():
    """sparse_lora_linear_fp8_oracle: the W8A8 sparse product (pinned above) plus the LoRA residual of the
    bf16 input (pinned above), nothing else: checked against both parts, against an fp64 evaluation of the
    residual, and with a zero factor."""
    X, W = synth.workload("tiny", seed=15, M=48)
    LA, LB = synth.lora(W.shape[0], W.shape[1], 16, seed=16, std_a=0.5, std_b=0.5)
    Xb, Wb, LAb, LBb = (synth.bits(t) for t in (X, W, LA, LB))
    Wq = oracle.quantize_weights_fp8(Wb)
    xs = float(np.abs(oracle.bf16_to_f32(Xb)).max() * 2 ** 0.5 / 448.0)
    b = synth.bits(synth.bias(W.shape[0], seed=17))
    for scope in (oracle.NONE, oracle.GROUP, oracle.ROW, oracle.TENSOR):
        r = oracle.sparse_lora_linear_fp8_oracle(Xb, Wq, xs, LAb, LBb, bias=b, scope=scope)
        base = oracle.sparse_linear_fp8_oracle(Xb, Wq, xs, bias=b, scope=scope)["Y"]
        assert np.array_equal(r["Y_s"], base)
        Xf = oracle.bf16_to_f32(Xb).astype(np.float64)
        ref_r = Xf @ (oracle.bf16_to_f32(LAb).astype(np.float64) @ oracle.bf16_to_f32(LBb).astype(np.float64)).T
        assert np.allclose(r["Y_r"], ref_r, rtol=0, atol=3e-5 * np.abs(ref_r).max())
        assert np.allclose(r["Y"], base.astype(np.float64) + ref_r, rtol=0, atol=3e-5 * np.abs(ref_r).max() + 1e-6 * np.abs(base).max())
        r0 = oracle.sparse_lora_linear_fp8_oracle(Xb, Wq, xs, np.zeros_like(LAb), LBb, bias=b, scope=scope)
        assert np.array_equal(r0["Y"], base)

