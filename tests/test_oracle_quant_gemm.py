"""Pins for the oracle's quantizers, the dual INT8 GEMM and the dequant epilogue.

Brute force on tiny matrices (numpy int64 / exact rationals), the fp64 fake-quant
definition computed WITHOUT any permutation, the paper's rounding-error closed form,
and the two reduction invariants (no outliers / all outliers == single-scale W8A8).
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import workloads as wl


# ----------------------------------------------------------------- helpers

def frac_to_f32(fr: Fraction) -> np.float32:
    """Round an exact rational to fp32, round-half-even (normal range only)."""
    if fr == 0:
        return np.float32(0.0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = 0
    while a >= 2 ** 24:
        a /= 2
        e += 1
    while a < 2 ** 23:
        a *= 2
        e -= 1
    n = a.numerator // a.denominator
    rem = a - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    assert e > -140
    return np.float32(sign * float(n) * 2.0 ** e)


def bf16_bits_torch(y_f32: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(y_f32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


# --------------------------------------------------------------- quantizer

def test_round_half_to_even_and_clip():
    # amax = 127 -> s = 1 exactly, so x/s = x and ties are visible
    X = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, -126.5, 126.5]], np.float32)
    Xq, sx = oracle.quant_act(X)
    assert sx[0] == 1.0
    assert Xq[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 3, -126, 126]


def test_quant_act_matches_numpy_recomputation_and_bounds():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((64, 384)).astype(np.float32)
    X[:, 5] *= 20
    X[3] = 0.0                                    # zero token: scale 0 -> all zeros
    perm = rng.permutation(384).astype(np.int32)
    Xq, sx = oracle.quant_act(X, perm)
    amax = np.abs(X).max(axis=1)
    assert np.array_equal(sx, amax / np.float32(127.0))
    with np.errstate(invalid="ignore", divide="ignore"):
        ref = np.rint(X / sx[:, None])            # fp32 division, rint = half-to-even
    ref[3] = 0
    assert np.array_equal(Xq, ref.astype(np.int8)[:, perm])
    assert Xq.min() >= -127 and Xq.max() <= 127
    nz = np.flatnonzero(amax > 0)
    assert np.all(np.abs(Xq[nz]).max(axis=1) == 127)      # absmax element maps to +-127
    assert np.all(Xq[3] == 0) and sx[3] == 0.0
    # element bound |q*s - x| <= s/2 and the closed form E|err| = s/4 under uniform rounding error
    inv = np.argsort(perm)
    err = np.abs(Xq[:, inv].astype(np.float64) * sx[:, None].astype(np.float64) - X)
    assert np.all(err <= 0.5 * sx[:, None] * (1 + 1e-6))


def test_rounding_error_closed_form_quarter_scale():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((256, 4096)).astype(np.float32) * 5.0
    Xq, sx = oracle.quant_act(X)
    err = np.abs(Xq.astype(np.float64) * sx[:, None] - X)
    ratio = (err.mean(axis=1) / sx).mean()
    assert abs(ratio - 0.25) < 0.01


def test_quant_act_perm_is_a_gather():
    X = np.arange(1, 9, dtype=np.float32)[None, :] * 127.0 / 8.0   # s = 1: values k*15.875
    perm = np.array([7, 0, 3, 1, 2, 4, 5, 6], np.int32)
    Xq, _ = oracle.quant_act(X, perm)
    Xq_id, _ = oracle.quant_act(X)
    assert Xq[0].tolist() == [Xq_id[0, k] for k in perm]
    assert Xq[0, 0] == 127                                         # position 0 holds channel 7


def test_static_activation_scale_variant():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((8, 32)).astype(np.float32) * 3
    s = np.float32(0.02)
    perm = rng.permutation(32).astype(np.int32)
    Xq = oracle.quant_act_static(X, s, perm)
    ref = np.clip(np.rint(X / s), -127, 127).astype(np.int8)[:, perm]
    assert np.array_equal(Xq, ref)
    assert np.abs(Xq).max() == 127                 # clip fires: 3-sigma values exceed 127*0.02
    # a zero scale gives the code 0, not the clipped infinity x / 0 would round to
    assert not oracle.quant_act_static(X, np.float32(0.0), perm).any()


def test_weight_scales_and_blocks():
    L = wl.small_random_case(7, 8, 48, 160, 5)
    q = oracle.quantize_weight(L["W"])
    W, perm, K_o = L["W"], q["perm"], q["K_o"]
    assert K_o == 32
    Wp = W[:, perm]
    a_o = np.abs(Wp[:, :K_o]).max(axis=1)
    a_n = np.abs(Wp[:, K_o:]).max(axis=1)
    assert np.array_equal(q["s_outlier"], a_o / np.float32(127))
    assert np.array_equal(q["s_normal"], a_n / np.float32(127))
    s_single = np.abs(W).max(axis=1) / np.float32(127)
    assert np.array_equal(np.maximum(q["s_normal"], q["s_outlier"]), s_single)
    assert np.all(q["s_normal"] <= s_single)
    assert np.all(q["s_normal"] < 0.5 * s_single)          # planted x10+: normal scale drops a lot
    ref = np.concatenate([np.rint(Wp[:, :K_o] / q["s_outlier"][:, None]),
                          np.rint(Wp[:, K_o:] / q["s_normal"][:, None])], axis=1).astype(np.int8)
    assert np.array_equal(q["Wq"], ref)
    assert np.all(np.abs(q["Wq"][:, :K_o]).max(axis=1) == 127)
    assert np.all(np.abs(q["Wq"][:, K_o:]).max(axis=1) == 127)
    # dual-scale lowers the mean dequant error of the normal block relative to single scale
    deq = q["Wq"][:, K_o:] * q["s_normal"][:, None].astype(np.float64)
    e_dual = np.abs(deq - Wp[:, K_o:]).mean()
    e_single = np.abs(np.rint(Wp[:, K_o:] / s_single[:, None]) * s_single[:, None] - Wp[:, K_o:]).mean()
    assert e_dual < 0.5 * e_single


def test_zero_weight_row_and_zero_block():
    W = np.zeros((3, 8), np.float32)
    W[1] = [1, -2, 0, 0, 0, 0, 0, 4]
    mask = np.array([0, 0, 1, 1, 0, 0, 0, 0], np.uint8)    # outlier block is all-zero in every row
    q = oracle.quantize_weight(W, forced_mask=mask)
    assert q["s_outlier"].tolist() == [0, 0, 0] and q["s_normal"][0] == 0 and q["s_normal"][2] == 0
    assert np.all(q["Wq"][0] == 0) and np.all(q["Wq"][:, :2] == 0)
    assert q["Wq"][1].tolist() == [0, 0, 32, -64, 0, 0, 0, 127]


# -------------------------------------------------------------------- GEMM

@pytest.mark.parametrize("seed", range(8))
def test_accumulators_brute_force_int64(seed):
    rng = np.random.default_rng(200 + seed)
    M, N, K = (int(rng.integers(1, 40)) for _ in range(3))
    K = max(K, 2)
    Xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    Wq = rng.integers(-127, 128, (N, K)).astype(np.int8)
    sx = rng.uniform(0.01, 0.1, M).astype(np.float32)
    sn = rng.uniform(0.001, 0.01, N).astype(np.float32)
    so = rng.uniform(0.01, 0.1, N).astype(np.float32)
    for K_o in sorted({0, 1, K // 2, K - 1, K}):
        out = oracle.dual_gemm(Xq, sx, Wq, sn, so, None, K_o)
        X64, W64 = Xq.astype(np.int64), Wq.astype(np.int64)
        assert np.array_equal(out["acc_o"], X64[:, :K_o] @ W64[:, :K_o].T)
        assert np.array_equal(out["acc_n"], X64[:, K_o:] @ W64[:, K_o:].T)   # a transposed operand fails (M != N)


def test_accumulator_extreme_values_do_not_overflow():
    K = 4096
    Xq = np.full((2, K), 127, np.int8)
    Wq = np.full((3, K), -127, np.int8)
    one = np.ones(3, np.float32)
    out = oracle.dual_gemm(Xq, np.ones(2, np.float32), Wq, one, one, None, 1024)
    assert np.all(out["acc_o"] == -16129 * 1024) and np.all(out["acc_n"] == -16129 * 3072)


def test_epilogue_exact_rational_check():
    rng = np.random.default_rng(9)
    M, N, K, K_o = 5, 7, 96, 32
    Xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    Wq = rng.integers(-127, 128, (N, K)).astype(np.int8)
    sx = rng.uniform(0.01, 0.1, M).astype(np.float32)
    sn = rng.uniform(0.001, 0.01, N).astype(np.float32)
    so = rng.uniform(0.01, 0.1, N).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32)
    out = oracle.dual_gemm(Xq, sx, Wq, sn, so, b, K_o)
    for m in range(M):
        for j in range(N):
            ao, an = int(out["acc_o"][m, j]), int(out["acc_n"][m, j])
            r = frac_to_f32(Fraction(ao) * Fraction(float(so[j])))                 # one rounding
            r = frac_to_f32(Fraction(an) * Fraction(float(sn[j])) + Fraction(float(r)))   # fused: one rounding
            r = frac_to_f32(Fraction(float(r)) * Fraction(float(sx[m])) + Fraction(float(b[j])))
            assert out["Y_f32"][m, j] == r
    assert np.array_equal(out["Y_bf16"], bf16_bits_torch(out["Y_f32"]))
    # absent bias is +0
    out0 = oracle.dual_gemm(Xq, sx, Wq, sn, so, None, K_o)
    outz = oracle.dual_gemm(Xq, sx, Wq, sn, so, np.zeros(N, np.float32), K_o)
    assert np.array_equal(out0["Y_f32"].view(np.uint32), outz["Y_f32"].view(np.uint32))


def test_bf16_rounding_ties_to_even():
    vals = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e-5, 65504.0, 1.0039062], np.float32)
    one = np.ones(1, np.float32)
    # feed values through the epilogue as bias with zero accumulators
    out = oracle.dual_gemm(np.zeros((1, 4), np.int8), one, np.zeros((len(vals), 4), np.int8),
                           np.ones(len(vals), np.float32), np.ones(len(vals), np.float32), vals, 0)
    assert np.array_equal(out["Y_f32"][0], vals)
    assert np.array_equal(out["Y_bf16"][0], bf16_bits_torch(vals))
    assert out["Y_bf16"][0, 1] == 0x3F80 and out["Y_bf16"][0, 2] == 0x3F82   # ties go to the even mantissa


@pytest.mark.parametrize("seed,M,N,K,c", [(0, 24, 40, 192, 3), (1, 9, 33, 96, 0), (2, 31, 17, 256, 20)])
def test_whole_linear_vs_unpermuted_fake_quant_fp64(seed, M, N, K, c):
    L = wl.small_random_case(300 + seed, M, N, K, c)
    X, W, b = L["X"], L["W"], L["bias"]
    r = oracle.linear(X, W, b)
    perm, K_o = r["perm"], r["K_o"]
    inv = np.argsort(perm)
    # de-quantized operands in ORIGINAL channel order (quantize-then-dequantize, Eq. recon)
    scale_cols = np.where(np.arange(K)[None, :] < K_o, r["s_outlier"][:, None], r["s_normal"][:, None])
    W_hat = (r["Wq"].astype(np.float64) * scale_cols.astype(np.float64))[:, inv]
    X_hat = (r["Xq"].astype(np.float64) * r["s_x"][:, None].astype(np.float64))[:, inv]
    Y = X_hat @ W_hat.T + b.astype(np.float64)
    mag = np.abs(X_hat) @ np.abs(W_hat).T + np.abs(b)
    assert np.all(np.abs(r["Y_f32"] - Y) <= 4 * 2.0 ** -24 * mag)
    # and the fake-quant output is a sane approximation of the fp64 linear
    Y_fp = X.astype(np.float64) @ W.astype(np.float64).T + b
    assert np.abs(Y - Y_fp).mean() < 0.05 * np.abs(Y_fp).mean()
    # permutation invariance: any other order of the same split gives the same accumulators
    rng = np.random.default_rng(seed)
    p2 = np.concatenate([rng.permutation(perm[:K_o]), rng.permutation(perm[K_o:])]).astype(np.int32)
    Wq2, sn2, so2 = oracle.quantize_rows(W, p2, K_o)
    Xq2, sx2 = oracle.quant_act(X, p2)
    o2 = oracle.dual_gemm(Xq2, sx2, Wq2, sn2, so2, b, K_o)
    assert np.array_equal(o2["acc_n"], r["acc_n"]) and np.array_equal(o2["acc_o"], r["acc_o"])
    assert np.array_equal(o2["Y_f32"].view(np.uint32), r["Y_f32"].view(np.uint32))


@pytest.mark.parametrize("seed", range(3))
def test_invariant_no_outliers_equals_single_scale(seed):
    L = wl.small_random_case(400 + seed, 12, 320, 128, 0)   # N large enough that no column norm strays past 1.2x the median
    r = oracle.linear(L["X"], L["W"], L["bias"])
    s = oracle.single_scale_linear(L["X"], L["W"], L["bias"])
    assert r["K_o"] == 0 and np.all(r["acc_o"] == 0)
    assert np.array_equal(r["perm"], np.arange(128))
    assert np.array_equal(r["acc_n"], s["acc"])
    assert np.array_equal(r["s_normal"], s["s_w"]) and np.all(r["s_outlier"] == 0)
    assert np.array_equal(r["Y_f32"].view(np.uint32), s["Y_f32"].view(np.uint32))
    assert np.array_equal(r["Y_bf16"], s["Y_bf16"])


@pytest.mark.parametrize("seed", range(3))
def test_invariant_all_outliers_equals_single_scale(seed):
    L = wl.small_random_case(500 + seed, 20, 28, 128, 6)
    r = oracle.linear(L["X"], L["W"], L["bias"], forced_mask=np.ones(128, np.uint8))
    s = oracle.single_scale_linear(L["X"], L["W"], L["bias"])
    assert r["K_o"] == 128 and np.all(r["acc_n"] == 0)
    assert np.array_equal(r["s_outlier"], s["s_w"]) and np.all(r["s_normal"] == 0)
    assert np.array_equal(r["acc_o"], s["acc"])
    assert np.array_equal(r["Y_f32"].view(np.uint32), s["Y_f32"].view(np.uint32))
    assert np.array_equal(r["Y_bf16"], s["Y_bf16"])


def test_dual_scale_beats_single_scale_on_planted_outliers():
    # Sec. 3.2: a separate quantizer lowers the normal scale and with it the error (Eq. round_error)
    L = wl.small_random_case(600, 64, 96, 512, 8)
    X, W, b = L["X"], L["W"], L["bias"]
    Y_fp = X.astype(np.float64) @ W.astype(np.float64).T + b
    r = oracle.linear(X, W, b)
    s = oracle.single_scale_linear(X, W, b)
    e_dual = np.abs(r["Y_f32"] - Y_fp).mean()
    e_single = np.abs(s["Y_f32"] - Y_fp).mean()
    assert r["K_o"] == 32 and e_dual < e_single
