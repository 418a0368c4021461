"""Pins for the chained-layer epilogue of the oracle: the fp32 GELU and the quantize-for-the-next-layer
GEMM (static per-tensor activation scale, Sec. 4.1; Eq. (quantization))."""
import math

import numpy as np
import pytest

import oracle
import workloads as wl


def gelu64(x):
    x = np.asarray(x, np.float64)
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def test_gelu_matches_the_tanh_definition_in_double():
    """The oracle's GELU is the tanh form evaluated in double and rounded once.  Pinned to torch's own
    tanh-approximate GELU in float64 (a library routine, not a retyped formula), to two values worked
    by hand, and to properties of the function."""
    import torch
    x = np.concatenate([np.linspace(-12, 12, 4801), np.array([0.0, 1e-6, -1e-6, 1e-3, 30.0, -30.0, 100.0, -100.0])]).astype(np.float32)
    g = oracle.gelu_tanh(x)
    lib = torch.nn.functional.gelu(torch.from_numpy(x.astype(np.float64)), approximate="tanh").numpy()
    assert np.all(np.abs(g - lib) <= 6.1e-8 * np.abs(lib) + 4e-15)       # half an fp32 ulp of the double result (+ the
    #                                  cancellation of 1 + tanh(u) in double, deep in the negative tail)
    assert np.all(np.abs(lib - gelu64(x)) <= 1e-14 * np.maximum(1.0, np.abs(lib)))
    # tanh(sqrt(2/pi) * 1.044715) = tanh(0.83354...) = 0.682419...: gelu(1) = 0.841192, gelu(-1) = gelu(1) - 1
    assert abs(float(oracle.gelu_tanh(np.float32([1.0]))[0]) - 0.8411919906) < 5e-8
    assert abs(float(oracle.gelu_tanh(np.float32([-1.0]))[0]) + 0.1588080094) < 2e-8
    assert oracle.gelu_tanh(np.float32([0.0]))[0] == 0.0
    big = np.float32([9.0, 20.0, 100.0])
    assert np.array_equal(oracle.gelu_tanh(big), big)                  # saturates to the identity exactly
    assert np.all(np.abs(oracle.gelu_tanh(-big)) < 1e-9)               # and to zero on the other side
    # x * Phi(x) - (-x) * Phi(-x) ... = x : gelu(x) - gelu(-x) == x
    xs = np.linspace(0, 6, 601).astype(np.float32)
    assert np.all(np.abs(oracle.gelu_tanh(xs) - oracle.gelu_tanh(-xs) - xs) <= 1e-6 * np.maximum(1, xs))
    # minimum of GELU (tanh form) is about -0.17 near x = -0.75
    xm = np.linspace(-1.5, 0, 1501).astype(np.float32)
    gm = oracle.gelu_tanh(xm)
    assert -0.1702 < gm.min() < -0.1698 and abs(xm[gm.argmin()] + 0.752) < 0.01


@pytest.mark.parametrize("act", [0, 1])
def test_q8_epilogue_codes(act):
    L = wl.small_random_case(500 + act, 37, 48, 160, 5)
    r = oracle.linear(L["X"], L["W"], L["bias"])
    y = r["Y_f32"]
    a = oracle.gelu_tanh(y) if act else y
    s_out = np.float32(np.abs(a).max() / 127 * 0.8)                    # a static scale that clips a little
    Y8 = oracle.dual_gemm_q8(r["Xq"], r["s_x"], r["Wq"], r["s_normal"], r["s_outlier"], L["bias"], r["K_o"], s_out, act)
    ref = np.clip(np.rint(a / s_out), -127, 127).astype(np.int8)       # numpy's fp32 division and rint
    assert np.array_equal(Y8, ref)
    assert Y8.max() == 127 and (act == 1 or Y8.min() == -127)
    # against the definition in double: same code except where a/s sits on a rounding boundary
    a64 = gelu64(y.astype(np.float64)) if act else y.astype(np.float64)
    ref64 = np.clip(np.rint(a64 / np.float64(s_out)), -127, 127)
    assert np.abs(Y8 - ref64).max() <= 1 and np.mean(Y8 != ref64) < 2e-3


def test_chained_ffn_tracks_the_float_computation():
    """FFN up -> GELU -> down with the intermediate kept in INT8 (static scale) stays close to fp64."""
    rng = np.random.default_rng(3)
    M, H, F = 48, 96, 256
    X = rng.standard_normal((M, H)).astype(np.float32)
    W1 = (rng.standard_normal((F, H)) * 0.1).astype(np.float32)
    W2 = (rng.standard_normal((H, F)) * 0.1).astype(np.float32)
    b1 = (rng.standard_normal(F) * 0.1).astype(np.float32)
    Y_ref = gelu64(X.astype(np.float64) @ W1.T.astype(np.float64) + b1) @ W2.T.astype(np.float64)
    q2 = oracle.quantize_weight(W2)
    q1 = oracle.quantize_weight(W1[q2["perm"]])          # rows of the first layer in the second layer's packed order
    Xq, sx = oracle.quant_act(X, q1["perm"])
    hidden = oracle.dual_gemm(Xq, sx, q1["Wq"], q1["s_normal"], q1["s_outlier"], b1[q2["perm"]], q1["K_o"])["Y_f32"]
    s_out = np.float32(np.abs(oracle.gelu_tanh(hidden)).max() / 127)
    H8 = oracle.dual_gemm_q8(Xq, sx, q1["Wq"], q1["s_normal"], q1["s_outlier"], b1[q2["perm"]], q1["K_o"], s_out, 1)
    out = oracle.dual_gemm(H8, np.full(M, s_out, np.float32), q2["Wq"], q2["s_normal"], q2["s_outlier"], None, q2["K_o"])
    err = np.abs(out["Y_f32"] - Y_ref).mean() / np.abs(Y_ref).mean()
    assert err < 0.03
