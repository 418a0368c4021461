"""Pins for the oracle's percentile-clip scale search (Sec. 4.1 "Quantization Implementation": the clipping
percentile is searched over {0.999, 0.9999, 0.99999}).  The percentile is checked against numpy's linear
interpolation, the errors against a float64 recomputation, the decision against the argmin of those, and the
three outcomes are each forced by a construction whose winner follows from a short argument."""
import numpy as np
import pytest

import oracle

P = [0.999, 0.9999, 0.99999]


def sse64(w, s, qmax):
    w = w.astype(np.float64)
    if s == 0:
        return float(np.sum(w * w))
    q = np.clip(np.rint(w.astype(np.float32) / np.float32(s)), -qmax, qmax).astype(np.float64)
    return float(np.sum((w - np.float64(s) * q) ** 2))


@pytest.mark.parametrize("n", [1, 2, 3, 5, 32, 33, 1000, 1536, 8896])
@pytest.mark.parametrize("qmax", [127.0, 7.0])
def test_clip_values_errors_and_choice(n, qmax):
    rng = np.random.default_rng(n * 3 + int(qmax))
    w = (rng.standard_t(3, n) * 0.02).astype(np.float32)               # heavy-tailed
    r = oracle.clip_search(w, qmax)
    a = np.abs(w).astype(np.float64)
    ref_clip = np.percentile(a, [100 * p for p in P])                  # numpy's default linear interpolation
    assert np.allclose(r["clip"], ref_clip, rtol=3e-7, atol=0)
    assert np.all(r["clip"] <= a.max() * (1 + 1e-7)) and np.all(np.diff(r["clip"]) >= 0)
    ref_sse = np.array([sse64(w, np.float32(c) / np.float32(qmax), qmax) for c in r["clip"]])
    assert np.allclose(r["sse"], ref_sse, rtol=1e-5, atol=1e-18)
    # decision: smallest error, the larger percentile on ties
    best = 2
    for c in (1, 0):
        if r["sse"][c] < r["sse"][best]:
            best = c
    assert r["choice"] == best
    assert r["s"] == np.float32(r["clip"][best]) / np.float32(qmax)
    gap = np.sort(ref_sse)
    if gap[1] - gap[0] > 1e-6 * gap[1]:                                 # a clear winner: the float64 recomputation agrees
        assert r["choice"] == int(np.argmin(ref_sse))


def test_small_example_by_hand():
    # |w| sorted: 1, 2, 3, 100 -> h = 3 p; p = 0.999: 2.997 -> 3 + 0.997 * 97
    w = np.float32([2.0, -100.0, 1.0, 3.0])
    r = oracle.clip_search(w, 127.0)
    assert np.allclose(r["clip"], [3 + 0.997 * 97, 3 + 0.9997 * 97, 3 + 0.99997 * 97], rtol=2e-7)
    # an empty block (no outlier channel) has scale 0 and reports the least-clipping percentile
    e = oracle.clip_search(np.zeros(0, np.float32), 127.0)
    assert float(e["s"]) == 0.0 and e["choice"] == 2


def test_each_percentile_can_win():
    rng = np.random.default_rng(5)
    n = 8896
    g = rng.standard_normal(n).astype(np.float32)
    # Gaussian, 8 bits: rounding noise n s^2 / 12 shrinks by ~0.2 sigma^2 when clipping at 3.3 sigma instead of the
    # maximum, the nine clipped values cost more -> 0.999 loses
    r = oracle.clip_search(g, 127.0)
    assert r["choice"] != 0 and r["sse"][0] > r["sse"][2]
    # five equal large values over small noise: 0.999 (rank n - 9.9) falls into the noise and destroys them
    # (error ~ 5 * 10^2), the other two both land on the plateau (ranks n-1.9 and n-1.09) -> tie -> 0.99999
    t = (g * 0.01).astype(np.float32)
    t[[3, 500, 501, 4000, 8000]] = [10, -10, 10, -10, 10]
    r = oracle.clip_search(t, 127.0)
    assert r["choice"] == 2 and r["clip"][1] == r["clip"][2] == 10 and r["sse"][0] > 400 > 10 > r["sse"][2]
    # Gaussian, 4 bits: the step is 18 times larger, the rounding term dominates -> clip hardest (0.999)
    assert oracle.clip_search(g, 7.0)["choice"] == 0
    # the middle candidate: for this Gaussian draw at 8 bits shaving the single largest value wins by a clear margin
    # in the float64 recomputation too
    r = oracle.clip_search(g, 127.0)
    ref = [sse64(g, np.float32(c) / np.float32(127.0), 127.0) for c in r["clip"]]
    assert r["choice"] == 1 == int(np.argmin(ref)) and min(ref[0], ref[2]) > ref[1] * 1.001
    # all magnitudes equal: the three candidates coincide, the tie goes to the largest percentile
    e = np.full(100, -0.5, np.float32)
    r = oracle.clip_search(e, 127.0)
    assert r["choice"] == 2 and np.all(r["clip"] == 0.5) and r["sse"].max() < 1e-12
    z = oracle.clip_search(np.zeros(10, np.float32), 127.0)
    assert z["s"] == 0 and z["choice"] == 2 and not z["sse"].any()
    assert oracle.clip_search(np.zeros(0, np.float32), 127.0)["s"] == 0


@pytest.mark.parametrize("bits", [8, 4])
def test_rows_with_clip_search(bits):
    rng = np.random.default_rng(bits)
    N, K, K_o = 24, 200, 32
    W = (rng.standard_t(4, (N, K)) * 0.02).astype(np.float32)
    W[3] = 0
    perm = rng.permutation(K).astype(np.int32)
    qmax = 127.0 if bits == 8 else 7.0
    Wq, sn, so, cn, co = oracle.quantize_rows_clip(W, perm, K_o, bits)
    Wq0, sn0, so0 = oracle.quantize_rows(W, perm, K_o) if bits == 8 else (None, None, None)
    for j in range(N):
        bo, bn = W[j, perm[:K_o]], W[j, perm[K_o:]]
        ro, rn = oracle.clip_search(bo, qmax), oracle.clip_search(bn, qmax)
        assert so[j] == ro["s"] and sn[j] == rn["s"] and co[j] == ro["choice"] and cn[j] == rn["choice"]
        ref = np.concatenate([np.clip(np.rint(bo / so[j]), -qmax, qmax) if so[j] else np.zeros(K_o),
                              np.clip(np.rint(bn / sn[j]), -qmax, qmax) if sn[j] else np.zeros(K - K_o)])
        assert np.array_equal(Wq[j], ref.astype(np.int8))
        if bits == 8:                                                   # never looser than the absmax scale
            assert so[j] <= so0[j] and sn[j] <= sn0[j]
    assert not Wq[3].any() and sn[3] == 0
    # the whole offline step with the flag: same split as without, these scales
    full = oracle.quantize_weight(W, bits=bits, clip_search=True)
    base = oracle.quantize_weight(W, bits=bits)
    assert np.array_equal(full["perm"], base["perm"]) and full["K_o"] == base["K_o"]
    Wq2, sn2, so2, _, _ = oracle.quantize_rows_clip(W, base["perm"], base["K_o"], bits)
    assert np.array_equal(full["Wq"], Wq2) and np.array_equal(full["s_normal"], sn2) and np.array_equal(full["s_outlier"], so2)
    # the dual GEMM on these codes and scales still approximates the float product, and at 4 bits better than absmax
    X = rng.standard_normal((16, K)).astype(np.float32)
    Y = X.astype(np.float64) @ W.T.astype(np.float64)
    def err(qw):
        Xq, sx = oracle.quant_act(X, qw["perm"])
        out = oracle.dual_gemm(Xq, sx, qw["Wq"], qw["s_normal"], qw["s_outlier"], None, qw["K_o"])["Y_f32"]
        return np.abs(out - Y).mean() / np.abs(Y).mean()
    assert err(full) < (0.02 if bits == 8 else 0.2)
    if bits == 4:
        assert err(full) < err(base)
