"""GPU parity of the chained-layer epilogue (qarvd_w8a8_dual_gemm_q8): the dual GEMM followed, in the same
kernel, by an optional fp32 GELU and the next layer's static-scale INT8 quantization (Sec. 4.1 static
per-tensor activation scales; Eq. (quantization)).  INT8 codes: bit-exact against the oracle without an
activation; with GELU (the oracle: the tanh form in double, rounded once; the kernel: its own fp32 sequence)
equal except next to a rounding boundary of a / s_out, where they may be one apart (gpu_util.assert_q8_codes).
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2605_21072_amd")
from gpu_util import assert_q8_codes, bf16_bits, bf16_ulp_distance, dev, gpu_quantize_weight, logical  # noqa: E402


def pack_int8(a, K, K_o):
    n_off, kp = q.packed_normal_offset(K_o), q.packed_k(K, K_o)
    out = np.zeros((a.shape[0], kp), np.int8)
    out[:, :K_o] = a[:, :K_o]
    out[:, n_off:n_off + K - K_o] = a[:, K_o:]
    return out


def random_codes_case(seed, M, N, K, K_o):
    rng = np.random.default_rng(seed)
    Xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    Wq = rng.integers(-127, 128, (N, K)).astype(np.int8)
    # scales that put the fp32 results at a few units, where GELU is neither the identity nor zero
    sx = rng.uniform(0.5, 1.5, M).astype(np.float32) * np.float32(1.0 / (127 * np.sqrt(K)))
    sn = rng.uniform(0.5, 1.5, N).astype(np.float32) * np.float32(2.0 / 127)
    so = rng.uniform(0.5, 1.5, N).astype(np.float32) * np.float32(4.0 / 127)
    b = (rng.standard_normal(N) * 0.3).astype(np.float32)
    return Xq, Wq, sx, sn, so, b


@pytest.mark.parametrize("act", [q.ACT_NONE, q.ACT_GELU_TANH])
@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("M,N,K,K_o", [(300, 208, 384, 32), (520, 384, 1536, 64), (257, 144, 640, 0),
                                       (64, 96, 130, 7), (33, 48, 96, 96), (700, 528, 512, 128), (1, 16, 32, 0)])
def test_q8_gemm_codes_match_oracle(act, variant, M, N, K, K_o):
    Xq, Wq, sx, sn, so, b = random_codes_case(act * 7 + variant * 31 + M + N + K + K_o, M, N, K, K_o)
    y = oracle.dual_gemm(Xq, sx, Wq, sn, so, b, K_o)["Y_f32"]
    a = oracle.gelu_tanh(y) if act else y
    s_out = float(np.float32(np.abs(a).max() / 127 * 0.7))              # clips the largest values
    ref, A = oracle.dual_gemm_q8(Xq, sx, Wq, sn, so, b, K_o, s_out, act, want_act=True)
    assert ref.max() == 127 and len(np.unique(ref)) > 100 or M * N < 4096
    w = q.DualScaleWeight(dev(pack_int8(Wq, K, K_o)), dev(sn), dev(so), None, K_o, N, K)
    ld = (N + 127) // 128 * 128 + 16                                       # wider than N: the rest must stay untouched
    Y8 = torch.full((M, ld), 0x55, dtype=torch.int8, device="cuda")
    q.w8a8_dual_gemm_q8(dev(pack_int8(Xq, K, K_o)), dev(sx), w, dev(b), M, s_out, act, Y8=Y8, variant=variant)
    torch.cuda.synchronize()
    got = Y8.cpu().numpy()
    assert_q8_codes(got[:, :N], ref, A, s_out, act)
    assert np.all(got[:, N:] == 0x55)


def test_q8_gemm_without_bias():
    M, N, K, K_o = 130, 160, 256, 32
    Xq, Wq, sx, sn, so, _ = random_codes_case(77, M, N, K, K_o)
    w = q.DualScaleWeight(dev(pack_int8(Wq, K, K_o)), dev(sn), dev(so), None, K_o, N, K)
    Xd = dev(pack_int8(Xq, K, K_o))
    for act in (0, 1):
        ref, A = oracle.dual_gemm_q8(Xq, sx, Wq, sn, so, None, K_o, 0.02, act, want_act=True)
        Y8 = q.w8a8_dual_gemm_q8(Xd, dev(sx), w, None, M, 0.02, act)
        torch.cuda.synchronize()
        assert_q8_codes(Y8.cpu().numpy(), ref, A, 0.02, act)
    with pytest.raises(ValueError):                                       # a static scale of 0 is an error on both sides
        oracle.dual_gemm_q8(Xq, sx, Wq, sn, so, None, K_o, 0.0, 1)
    with pytest.raises(q.QarvdError):
        q.w8a8_dual_gemm_q8(Xd, dev(sx), w, None, M, 0.0, 1)


ALL_ONES = float(np.array([0x3F7FFFFF], np.uint32).view(np.float32)[0])        # 1 - 2^-24: every mantissa bit set


@pytest.mark.parametrize("act,s_out", [(0, 0.0371), (0, 1.0), (0, ALL_ONES), (0, 3.3e-5), (0, 517.3), (0, 2.5e-30),
                                       (0, 7.0e29 / 130), (1, 0.0371), (1, 0.004)])
def test_q8_rounding_boundaries_and_dense_sweep(act, s_out):
    """Without an activation the kernel forms the quotient as a product with 1 / s corrected by two fused
    multiply-adds, which must equal the IEEE quotient: drive it with values ON and up to four ulps either side
    of every rounding boundary (k + 1/2) * s, for ordinary scales, a power of two, a mantissa of all ones and
    the ends of the accepted range.  With GELU: a dense sweep of the activation's input range.  Zero
    activations make y equal the bias."""
    s_out = float(np.float32(s_out))
    if act == 0:
        k = np.arange(-130, 130, dtype=np.float64) + 0.5
        centre = (k * np.float64(np.float32(s_out))).astype(np.float32)
        vals = [centre]
        for steps in range(1, 5):
            up, dn = centre.copy(), centre.copy()
            for _ in range(steps):
                up, dn = np.nextafter(up, np.float32(np.inf)), np.nextafter(dn, np.float32(-np.inf))
            vals += [up, dn]
        b = np.concatenate(vals + [np.float32([0.0, -0.0, 1e-38, -1e-38, 1e30, -1e30, 4.7, -4.7, 3e38, -3e38])])
        b = np.concatenate([b, np.zeros(-len(b) % 16, np.float32)]).astype(np.float32)
    else:
        b = np.concatenate([np.linspace(-9, 9, 49152), np.linspace(-0.9, 0.9, 16384)]).astype(np.float32)
    N, M, K = len(b), 33, 32
    Xq = np.zeros((M, K), np.int8)
    rng = np.random.default_rng(act)
    Wq = rng.integers(-127, 128, (N, K)).astype(np.int8)
    sx, sn = np.ones(M, np.float32), np.ones(N, np.float32)
    ref, A = oracle.dual_gemm_q8(Xq, sx, Wq, sn, sn, b, 0, s_out, act, want_act=True)
    w = q.DualScaleWeight(dev(pack_int8(Wq, K, 0)), dev(sn), dev(sn), None, 0, N, K)
    for variant in range(1, q.q8_gemm_num_variants() + 1):
        Y8 = q.w8a8_dual_gemm_q8(dev(pack_int8(Xq, K, 0)), dev(sx), w, dev(b), M, s_out, act, variant=variant)
        torch.cuda.synchronize()
        assert_q8_codes(Y8.cpu().numpy(), ref, A, s_out, act)
    if act == 0:                       # the crafted values do straddle the boundaries
        assert len(np.unique(ref[0, :260 * 9])) == 255 and np.any(ref[0, :260] != ref[0, 260:520])


def test_q8_gemm_rejects_what_it_cannot_run():
    M, N, K = 64, 72, 128                                                  # N not a multiple of 16
    Xq, Wq, sx, sn, so, b = random_codes_case(5, M, N, K, 0)
    w = q.DualScaleWeight(dev(pack_int8(Wq, K, 0)), dev(sn), dev(so), None, 0, N, K)
    Xd = dev(pack_int8(Xq, K, 0))
    Y8 = torch.empty((M, 80), dtype=torch.int8, device="cuda")
    with pytest.raises(q.QarvdError) as e:
        q.w8a8_dual_gemm_q8(Xd, dev(sx), w, dev(b), M, 0.1, 0, Y8=Y8)
    assert e.value.status == -2
    w.N = 64
    for bad in (dict(out_scale=float("nan")), dict(out_scale=0.0), dict(out_scale=-1.0), dict(out_scale=float("inf")),
                dict(out_scale=1e-38), dict(act=7),
                dict(variant=q.q8_gemm_num_variants() + 1)):
        kw = dict(out_scale=0.1, act=0, variant=0)
        kw.update(bad)
        with pytest.raises(q.QarvdError) as e:
            q.w8a8_dual_gemm_q8(Xd, dev(sx), w, dev(b), M, Y8=Y8, **kw)
        assert e.value.status == -1, bad
    w4 = q.DualScaleWeight(w.Wq.view(torch.uint8), w.s_normal, w.s_outlier, None, 0, 64, K, None, 4)
    with pytest.raises(ValueError):
        q.w8a8_dual_gemm_q8(Xd, dev(sx), w4, dev(b), M, 0.1)


def chain_weights(W1, b1, W2):
    """Second layer quantized first; first layer's rows and bias gathered into its packed channel order
    (zero rows at the pad positions), so that the first GEMM's INT8 output IS the second layer's Xq."""
    w2 = gpu_quantize_weight(W2)
    cmap = q.packed_channel_map(w2).cpu().numpy()
    W1p = np.zeros((cmap.shape[0], W1.shape[1]), np.float32)
    b1p = np.zeros(cmap.shape[0], np.float32)
    W1p[cmap >= 0] = W1[cmap[cmap >= 0]]
    b1p[cmap >= 0] = b1[cmap[cmap >= 0]]
    w1 = gpu_quantize_weight(W1p)
    return w1, dev(b1p), w2


def oracle_chain(X_rows, W1, b1, W2, b2, s_mid, act):
    """First layer (codes and the values they were rounded from) and the weights of the second."""
    o2 = oracle.quantize_weight(W2)
    o1 = oracle.quantize_weight(W1[o2["perm"]])
    Xq, sx = oracle.quant_act(X_rows, o1["perm"])
    H8, A = oracle.dual_gemm_q8(Xq, sx, o1["Wq"], o1["s_normal"], o1["s_outlier"], b1[o2["perm"]], o1["K_o"], s_mid, act,
                                want_act=True)
    return o2, H8, A


def oracle_second_layer(o2, H8, b2, s_mid):
    """The second layer on given hand-over codes (the kernel's own, once they have passed the code rule:
    next to a rounding boundary they may differ from the oracle's by one, and the second layer is
    checked on what it was actually fed)."""
    return oracle.dual_gemm(H8, np.full(H8.shape[0], s_mid, np.float32), o2["Wq"], o2["s_normal"], o2["s_outlier"],
                            b2, o2["K_o"])


def gpu_chain(X, w1, b1p, w2, b2, s_mid, act, out_dtype):
    M = X.shape[0]
    Xq, sx = q.quant_act(dev(X), w1.perm if w1.K_o else None, w1.K_o)
    H8 = q.w8a8_dual_gemm_q8(Xq, sx, w1, b1p, M, s_mid, act)               # [M, kp of layer 2]: that layer's Xq
    s_mid_rows = torch.full((M,), s_mid, dtype=torch.float32, device="cuda")
    Y = q.w8a8_dual_gemm(H8, s_mid_rows, w2, dev(b2), M, out_dtype)
    torch.cuda.synchronize()
    return H8, Y


@pytest.mark.parametrize("act", [0, 1])
def test_chained_ffn_small(act):
    rng = np.random.default_rng(11 + act)
    M, H, F = 300, 256, 640
    X = rng.standard_normal((M, H)).astype(np.float32)
    X[:, [5, 77]] *= 15
    W1 = (rng.standard_normal((F, H)) * 0.05).astype(np.float32)
    W1[:, [5, 77]] *= 20
    W2 = (rng.standard_normal((H, F)) * 0.05).astype(np.float32)
    W2[:, [9, 300, 511]] *= 25
    b1 = (rng.standard_normal(F) * 0.1).astype(np.float32)
    b2 = (rng.standard_normal(H) * 0.1).astype(np.float32)
    s_mid = 0.05
    o2, H8_ref, A_ref = oracle_chain(X, W1, b1, W2, b2, s_mid, act)
    assert o2["K_o"] > 0
    w1, b1p, w2 = chain_weights(W1, b1, W2)
    assert w2.K_o == o2["K_o"] and w1.N == w2.kp
    for out_dtype in (torch.float32, torch.bfloat16):
        H8, Y = gpu_chain(X, w1, b1p, w2, b2, s_mid, act, out_dtype)
        H8_l = logical(H8, w2.K, w2.K_o)                                   # also checks the pad columns are 0
        assert_q8_codes(H8_l, H8_ref, A_ref, s_mid, act)
        out = oracle_second_layer(o2, H8_l, b2, s_mid)
        if out_dtype == torch.float32:
            y, r = Y.cpu().numpy(), out["Y_f32"]
            assert np.all((np.abs(y - r) <= 1e-6 * np.abs(r)) | (y == r))
        else:
            assert bf16_ulp_distance(bf16_bits(Y), out["Y_bf16"]).max() <= 1


def test_chained_ffn_full_size_sampled_rows():
    """The DiT FFN pair at the benchmark's shapes (4680 tokens, 1536 -> 8960 -> 1536): GELU and INT8 hand-over
    in the up-projection's epilogue; 24 sampled token rows against the oracle, every variant."""
    up, down = wl.find_layer("cfg2.ffn_up.c16"), wl.find_layer("cfg2.ffn_down.c64")
    Lu, Ld = wl.make_layer(up), wl.make_layer(down)
    X, W1, b1, W2, b2 = Lu["X"], Lu["W"], Lu["bias"], Ld["W"], Ld["bias"]
    rng = np.random.default_rng(up.seed + 9)
    rows = np.unique(np.concatenate([[0, up.M - 1], rng.choice(up.M, 22, replace=False)]))
    w1, b1p, w2 = chain_weights(W1, b1, W2)
    # static scale "calibrated" on the sampled rows by the oracle
    o1 = oracle.quantize_weight(W1)
    hid = oracle.gelu_tanh(oracle.linear(X[rows], W1, b1)["Y_f32"])
    s_mid = float(np.float32(np.abs(hid).max() / 127))
    o2, H8_ref, A_ref = oracle_chain(X[rows], W1, b1, W2, b2, s_mid, 1)
    assert o1["K_o"] > 0 and o2["K_o"] > 0
    rt = torch.from_numpy(rows).cuda()
    Xq, sx = q.quant_act(dev(X), w1.perm, w1.K_o)
    for variant in range(0, q.q8_gemm_num_variants() + 1):
        H8 = q.w8a8_dual_gemm_q8(Xq, sx, w1, b1p, up.M, s_mid, q.ACT_GELU_TANH, variant=variant)
        torch.cuda.synchronize()
        assert_q8_codes(logical(H8[rt], w2.K, w2.K_o), H8_ref, A_ref, s_mid, 1)
    out = oracle_second_layer(o2, logical(H8[rt], w2.K, w2.K_o), b2, s_mid)
    s_rows = torch.full((up.M,), s_mid, dtype=torch.float32, device="cuda")
    Y = q.w8a8_dual_gemm(H8, s_rows, w2, dev(b2), up.M, torch.bfloat16)
    torch.cuda.synchronize()
    assert bf16_ulp_distance(bf16_bits(Y[rt]), out["Y_bf16"]).max() <= 1


def test_fused_qkv_as_one_layer_sampled_rows():
    """Three projections of one block as ONE layer (weight rows concatenated, N = 4608, one shared outlier
    set from the concatenated matrix): the ordinary entry points on a wider N; sampled rows against the oracle."""
    specs = [wl.find_layer(n) for n in ("cfg2.q.c16", "cfg2.k.c16", "cfg2.v.c16")]
    Ls = [wl.make_layer(s) for s in specs]
    W = np.concatenate([L["W"] for L in Ls], 0)
    b = np.concatenate([L["bias"] for L in Ls])
    X = Ls[0]["X"]
    M = specs[0].M
    o = oracle.quantize_weight(W)
    w = gpu_quantize_weight(W)
    assert w.K_o == o["K_o"] and w.N == 4608 and np.array_equal(w.perm.cpu().numpy(), o["perm"])
    rng = np.random.default_rng(77)
    rows = np.unique(np.concatenate([[0, M - 1], rng.choice(M, 30, replace=False)]))
    Xq_o, sx_o = oracle.quant_act(X[rows], o["perm"])
    ref = oracle.dual_gemm(Xq_o, sx_o, o["Wq"], o["s_normal"], o["s_outlier"], b, o["K_o"])
    Xq, sx = q.quant_act(dev(X), w.perm if w.K_o else None, w.K_o)
    Y = q.w8a8_dual_gemm(Xq, sx, w, dev(b), M, torch.bfloat16)
    torch.cuda.synchronize()
    rt = torch.from_numpy(rows).cuda()
    assert np.array_equal(logical(Xq[rt], w.K, w.K_o), Xq_o)
    assert np.array_equal(sx[rt].cpu().numpy().view(np.uint32), sx_o.view(np.uint32))
    assert bf16_ulp_distance(bf16_bits(Y[rt]), ref["Y_bf16"]).max() <= 1
