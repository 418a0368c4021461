"""Pins for the 4-bit weight setting of the oracle (W4A8, Sec. 4.2: same Eq. (quantization), b = 4).

The codes are checked against a numpy re-computation, the symmetric range and the error bounds
that follow from the equation, the exact scale relation to the 8-bit setting, and the fp64
fake-quant definition of the whole layer computed without any permutation.
"""
import numpy as np
import pytest

import oracle
import workloads as wl


def test_w4_codes_scales_and_range():
    L = wl.small_random_case(11, 8, 48, 160, 5)
    q = oracle.quantize_weight(L["W"], bits=4)
    q8 = oracle.quantize_weight(L["W"], bits=8)
    W, perm, K_o = L["W"], q["perm"], q["K_o"]
    # the detector, alignment and permutation do not depend on the bit-width
    assert K_o == q8["K_o"] == 32 and np.array_equal(perm, q8["perm"])
    Wp = W[:, perm]
    a_o = np.abs(Wp[:, :K_o]).max(axis=1)
    a_n = np.abs(Wp[:, K_o:]).max(axis=1)
    assert np.array_equal(q["s_outlier"], a_o / np.float32(7))      # q_max = 2^(4-1) - 1
    assert np.array_equal(q["s_normal"], a_n / np.float32(7))
    ref = np.concatenate([np.rint(Wp[:, :K_o] / q["s_outlier"][:, None]),
                          np.rint(Wp[:, K_o:] / q["s_normal"][:, None])], axis=1).astype(np.int8)
    assert np.array_equal(q["Wq"], ref)
    assert q["Wq"].min() == -7 and q["Wq"].max() == 7
    assert np.all(np.abs(q["Wq"][:, :K_o]).max(axis=1) == 7)        # every block holds its absmax
    assert np.all(np.abs(q["Wq"][:, K_o:]).max(axis=1) == 7)
    # element bound |q*s - w| <= s/2 and the s/4 mean of a uniform rounding error (Eq. round_error)
    sc = np.where(np.arange(W.shape[1])[None, :] < K_o, q["s_outlier"][:, None], q["s_normal"][:, None]).astype(np.float64)
    err = np.abs(q["Wq"] * sc - Wp)
    assert np.all(err <= 0.5 * sc * (1 + 1e-6))
    ratio = (err[:, K_o:] / sc[:, K_o:]).mean()
    assert 0.2 < ratio < 0.3
    # a 4-bit step is 127/7 times the 8-bit step of the same block
    assert np.allclose(q["s_normal"] / q8["s_normal"], 127.0 / 7.0, rtol=1e-6)


def test_w4_half_way_cases_round_to_even_and_clip_is_symmetric():
    W = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -6.5, -7.0]], np.float32)   # scale = 1 exactly
    q = oracle.quantize_weight(W, forced_mask=np.zeros(8, np.uint8), bits=4)
    assert q["s_normal"][0] == np.float32(1.0)
    assert q["Wq"][0].tolist() == [7, 0, 2, 2, 0, -2, -6, -7]


@pytest.mark.parametrize("seed,M,N,K,c", [(0, 24, 40, 192, 3), (1, 9, 33, 96, 0)])
def test_w4a8_linear_vs_unpermuted_fake_quant_fp64(seed, M, N, K, c):
    L = wl.small_random_case(900 + seed, M, N, K, c)
    X, W, b = L["X"], L["W"], L["bias"]
    q = oracle.quantize_weight(W, bits=4)
    Xq, sx = oracle.quant_act(X, q["perm"])
    r = oracle.dual_gemm(Xq, sx, q["Wq"], q["s_normal"], q["s_outlier"], b, q["K_o"])
    # brute-force INT32 sums
    K_o = q["K_o"]
    assert np.array_equal(r["acc_o"], Xq[:, :K_o].astype(np.int64) @ q["Wq"][:, :K_o].astype(np.int64).T)
    assert np.array_equal(r["acc_n"], Xq[:, K_o:].astype(np.int64) @ q["Wq"][:, K_o:].astype(np.int64).T)
    inv = np.argsort(q["perm"])
    scale_cols = np.where(np.arange(K)[None, :] < K_o, q["s_outlier"][:, None], q["s_normal"][:, None])
    W_hat = (q["Wq"].astype(np.float64) * scale_cols.astype(np.float64))[:, inv]
    X_hat = (Xq.astype(np.float64) * sx[:, None].astype(np.float64))[:, inv]
    Y = X_hat @ W_hat.T + b.astype(np.float64)
    mag = np.abs(X_hat) @ np.abs(W_hat).T + np.abs(b)
    assert np.all(np.abs(r["Y_f32"] - Y) <= 4 * 2.0 ** -24 * mag)
    # coarser than W8A8, but still the same layer
    Y_fp = X.astype(np.float64) @ W.astype(np.float64).T + b
    q8 = oracle.quantize_weight(W, bits=8)
    r8 = oracle.dual_gemm(Xq, sx, q8["Wq"], q8["s_normal"], q8["s_outlier"], b, K_o)
    e4, e8 = np.abs(r["Y_f32"] - Y_fp).mean(), np.abs(r8["Y_f32"] - Y_fp).mean()
    assert e8 < e4 < 0.35 * np.abs(Y_fp).mean()


def test_w4_dual_scale_gain_is_larger_than_at_8_bits():
    """Sec. 4.3 (ablation): the dual scale matters most at low weight bit-width."""
    L = wl.small_random_case(77, 64, 96, 512, 12)
    X, W = L["X"], L["W"]
    Y_fp = X.astype(np.float64) @ W.astype(np.float64).T
    gain = {}
    for bits in (8, 4):
        d = oracle.quantize_weight(W, bits=bits)
        s = oracle.quantize_weight(W, forced_mask=np.zeros(W.shape[1], np.uint8), bits=bits)
        err = {}
        for name, q in (("dual", d), ("single", s)):
            Xq, sx = oracle.quant_act(X, q["perm"])
            r = oracle.dual_gemm(Xq, sx, q["Wq"], q["s_normal"], q["s_outlier"], None, q["K_o"])
            err[name] = np.abs(r["Y_f32"] - Y_fp).mean()
        assert err["dual"] < err["single"]
        gain[bits] = err["single"] - err["dual"]
    assert gain[4] > gain[8]
