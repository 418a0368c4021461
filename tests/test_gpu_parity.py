"""GPU parity: the HIP library (through the C ABI) against the CPU oracle, element by element.

Bar: bit-exact INT8 activations and weights, scales, permutation, K_o and both INT32 accumulators;
fp32 outputs within 1e-6 relative and bf16 outputs within 1 bf16 ulp (both are expected to be
bit-equal because the epilogue's three operations are fixed).
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2605_21072_amd")
from gpu_util import (assert_weight_equal, bf16_bits, bf16_ulp_distance, dev, gpu_quantize_weight, logical,  # noqa: E402
                      weight_to_numpy)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a device"
    q.load_library()


def check_y(Y_gpu: torch.Tensor, ref: dict):
    if Y_gpu.dtype == torch.float32:
        y = Y_gpu.cpu().numpy()
        r = ref["Y_f32"]
        rel = np.abs(y - r) / np.maximum(np.abs(r), 1e-30)
        assert np.all((rel <= 1e-6) | (y == r)), "fp32 output beyond 1e-6 relative"
        return int(np.count_nonzero(y.view(np.uint32) != r.view(np.uint32)))
    d = bf16_ulp_distance(bf16_bits(Y_gpu), ref["Y_bf16"])
    assert d.max() <= 1, "bf16 output beyond 1 ulp"
    return int(np.count_nonzero(d))


# ------------------------------------------------------------------ quantize_weight

@pytest.mark.parametrize("seed,N,K,c", [(0, 64, 128, 3), (1, 300, 320, 20), (2, 257, 1000, 9), (3, 96, 37, 0),
                                        (4, 1536, 1536, 8), (5, 128, 4100, 50)])
def test_quantize_weight_detected(seed, N, K, c):
    L = wl.small_random_case(1000 + seed, 4, N, K, c)
    o = oracle.quantize_weight(L["W"])
    g = weight_to_numpy(gpu_quantize_weight(L["W"]))
    assert_weight_equal(g, o)


@pytest.mark.parametrize("align", [1, 8, 32, 64])
def test_quantize_weight_alignments(align):
    L = wl.small_random_case(1100 + align, 4, 200, 512, 11)
    o = oracle.quantize_weight(L["W"], align=align)
    g = weight_to_numpy(gpu_quantize_weight(L["W"], align=align))
    assert_weight_equal(g, o)
    assert o["K_o"] == (11 + align - 1) // align * align


@pytest.mark.parametrize("tau,alpha", [(3.5, 0.0), (2.5, 1.1), (4.5, 1.3), (0.5, 1.0)])
def test_quantize_weight_detector_parameters(tau, alpha):
    L = wl.small_random_case(1200, 4, 64, 2048, 6, mult=(1.5, 3.0))
    o = oracle.quantize_weight(L["W"], tau=tau, alpha=alpha)
    g = weight_to_numpy(gpu_quantize_weight(L["W"], tau=tau, alpha=alpha))
    assert_weight_equal(g, o)


@pytest.mark.parametrize("K_o", [0, 1, 31, 32, 33, 199, 200])
def test_quantize_weight_forced_masks(K_o):
    K = 200
    L = wl.small_random_case(1300 + K_o, 4, 50, K, 4)
    rng = np.random.default_rng(K_o)
    mask = np.zeros(K, np.uint8)
    mask[rng.choice(K, K_o, replace=False)] = 1
    o = oracle.quantize_weight(L["W"], forced_mask=mask)
    g = weight_to_numpy(gpu_quantize_weight(L["W"], forced_mask=mask))
    assert_weight_equal(g, o)


def test_quantize_weight_degenerate_rows_and_ties():
    W = np.zeros((6, 64), np.float32)
    W[1, :] = 1.0                      # all column norms tie
    W[2, 5] = -3.0
    W[4, ::2] = 0.25
    o = oracle.quantize_weight(W)
    g = weight_to_numpy(gpu_quantize_weight(W))
    assert_weight_equal(g, o)
    Wc = np.ones((8, 96), np.float32)   # constant norms: MAD = 0, no outliers
    assert_weight_equal(weight_to_numpy(gpu_quantize_weight(Wc)), oracle.quantize_weight(Wc))


# ------------------------------------------------------------------------ quant_act

@pytest.mark.parametrize("M,K,c,dtype", [(33, 1536, 8, "f32"), (17, 5120, 40, "f32"), (9, 8960, 64, "f32"),
                                         (5, 13824, 128, "f32"), (40, 1536, 8, "bf16"), (12, 8960, 30, "bf16"),
                                         (7, 250, 5, "f32"), (7, 37, 2, "f32"), (6, 1000, 0, "bf16"),
                                         (3, 20000, 10, "f32")])
def test_quant_act_parity(M, K, c, dtype):
    rng = np.random.default_rng(M * 100003 + K)
    X = rng.standard_normal((M, K)).astype(np.float32)
    if c:
        X[:, rng.choice(K, c, replace=False)] *= 15
    X[M // 2] = 0.0                                      # an all-zero token
    sel = np.zeros(K, np.uint8)
    if c:
        sel[rng.choice(K, c, replace=False)] = 1
    perm, K_o = oracle.build_perm(sel)
    Xd = dev(X)
    if dtype == "bf16":
        Xd = Xd.to(torch.bfloat16)
        X = Xd.float().cpu().numpy()                     # the oracle sees the exactly widened values
    Xq_o, sx_o = oracle.quant_act(X, perm)
    Xq_g, sx_g = q.quant_act(Xd, dev(perm) if c else None, K_o)
    torch.cuda.synchronize()
    assert np.array_equal(sx_g.cpu().numpy().view(np.uint32), sx_o.view(np.uint32))
    assert np.array_equal(logical(Xq_g, K, K_o), Xq_o)


@pytest.mark.parametrize("K", [1536, 8960])
def test_quant_act_perm_at_a_4_byte_aligned_address(K):
    """perm is fetched 16 bytes per lane when it is 16-byte aligned; a permutation that starts one element into
    a buffer takes the scalar path and must give the same bytes."""
    rng = np.random.default_rng(K)
    M, c = 21, 37
    X = rng.standard_normal((M, K)).astype(np.float32)
    sel = np.zeros(K, np.uint8)
    sel[rng.choice(K, c, replace=False)] = 1
    perm, K_o = oracle.build_perm(sel)
    Xq_o, sx_o = oracle.quant_act(X, perm)
    buf = torch.zeros(K + 1, dtype=torch.int32, device="cuda")
    buf[1:] = dev(perm)
    assert buf[1:].data_ptr() % 16 == 4
    Xq_g, sx_g = q.quant_act(dev(X), buf[1:], K_o)
    torch.cuda.synchronize()
    assert np.array_equal(sx_g.cpu().numpy().view(np.uint32), sx_o.view(np.uint32))
    assert np.array_equal(logical(Xq_g, K, K_o), Xq_o)


@pytest.mark.parametrize("K,amax", [(1536, 100.3), (8960, 3.7), (1000, 127.0), (250, 0.011)])
def test_quant_act_rounding_boundaries(K, amax):
    """Values sitting on and next to the half-integer rounding boundaries of x / s: the kernel's
    reciprocal shortcut must fall back to the exact division exactly where it matters."""
    rng = np.random.default_rng(K)
    M = 16
    s64 = np.float64(np.float32(np.float32(amax) / np.float32(127.0)))
    X = np.empty((M, K), np.float32)
    for m in range(M):
        k = rng.integers(-126, 127, K).astype(np.float64) + 0.5
        x = (k * s64).astype(np.float32)
        steps = rng.integers(-3, 4, K)
        for _ in range(3):
            x = np.where(steps > 0, np.nextafter(x, np.float32(np.inf)), np.where(steps < 0, np.nextafter(x, np.float32(-np.inf)), x))
            steps = steps - np.sign(steps)
        X[m] = x
        X[m, rng.integers(0, K)] = np.float32(amax)        # fixes the token's absmax
    sel = (rng.random(K) < 0.02).astype(np.uint8)
    perm, K_o = oracle.build_perm(sel)
    Xq_o, sx_o = oracle.quant_act(X, perm)
    Xq_g, sx_g = q.quant_act(dev(X), dev(perm) if K_o else None, K_o)
    torch.cuda.synchronize()
    assert np.array_equal(sx_g.cpu().numpy().view(np.uint32), sx_o.view(np.uint32))
    assert np.array_equal(logical(Xq_g, K, K_o), Xq_o)
    Xq_s = q.quant_act_static(dev(X), dev(perm) if K_o else None, K_o, float(s64) * 0.5)   # clip fires
    torch.cuda.synchronize()
    assert np.array_equal(logical(Xq_s, K, K_o), oracle.quant_act_static(X, np.float32(s64 * 0.5), perm))


def test_quant_act_strided_input_and_output():
    rng = np.random.default_rng(5)
    M, K = 21, 1536
    big = rng.standard_normal((M, K + 64)).astype(np.float32)
    Xd = dev(big)[:, :K]                                 # ldx = K + 64
    perm, K_o = oracle.build_perm((rng.random(K) < 0.02).astype(np.uint8))
    Xq = torch.full((M, q.packed_k(K, K_o) + 128), 77, dtype=torch.int8, device="cuda")
    sx = torch.empty(M, dtype=torch.float32, device="cuda")
    q.quant_act(Xd, dev(perm), K_o, Xq=Xq, s_x=sx)
    torch.cuda.synchronize()
    Xq_o, sx_o = oracle.quant_act(big[:, :K], perm)
    assert np.array_equal(logical(Xq, K, K_o), Xq_o) and np.array_equal(sx.cpu().numpy(), sx_o)
    assert torch.all(Xq[:, q.packed_k(K, K_o):] == 77)   # bytes past the packed extent are untouched


@pytest.mark.parametrize("K,dtype", [(1536, "f32"), (250, "f32"), (8960, "bf16")])
def test_quant_act_static_parity(K, dtype):
    rng = np.random.default_rng(K)
    M = 19
    X = (rng.standard_normal((M, K)) * 3).astype(np.float32)
    perm, K_o = oracle.build_perm((rng.random(K) < 0.03).astype(np.uint8))
    Xd = dev(X)
    if dtype == "bf16":
        Xd = Xd.to(torch.bfloat16)
        X = Xd.float().cpu().numpy()
    s = np.float32(0.05)
    Xq_g = q.quant_act_static(Xd, dev(perm), K_o, float(s))
    torch.cuda.synchronize()
    assert np.array_equal(logical(Xq_g, K, K_o), oracle.quant_act_static(X, s, perm))
    Xq_0 = q.quant_act_static(Xd, dev(perm), K_o, 0.0)          # a zero scale gives zero codes
    torch.cuda.synchronize()
    assert np.array_equal(logical(Xq_0, K, K_o), oracle.quant_act_static(X, np.float32(0.0), perm))
    assert not Xq_0[:, :q.packed_k(K, K_o)].any()              # (bytes between the packed extent and the row stride are not written)


# ----------------------------------------------------------------------------- GEMM

def _gemm_case(seed, M, N, K, K_o):
    rng = np.random.default_rng(seed)
    Xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    Wq = rng.integers(-127, 128, (N, K)).astype(np.int8)
    sx = rng.uniform(0.01, 0.1, M).astype(np.float32)
    sn = rng.uniform(0.001, 0.01, N).astype(np.float32)
    so = rng.uniform(0.01, 0.1, N).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32)
    return Xq, Wq, sx, sn, so, b


def _pack(a, K, K_o):
    n_off, kp = q.packed_normal_offset(K_o), q.packed_k(K, K_o)
    out = np.zeros((a.shape[0], kp), np.int8)
    out[:, :K_o] = a[:, :K_o]
    out[:, n_off:n_off + K - K_o] = a[:, K_o:]
    return out


def _variants():
    return list(range(0, 34))


@pytest.mark.parametrize("variant", _variants())
@pytest.mark.parametrize("M,N,K,K_o", [(300, 200, 384, 32), (520, 384, 1536, 64), (257, 129, 640, 0),
                                       (64, 96, 130, 7), (700, 513, 512, 160), (33, 40, 96, 96)])
def test_gemm_accumulators_and_outputs(variant, M, N, K, K_o):
    if variant > q.gemm_num_variants():
        pytest.skip("no such variant")
    Xq, Wq, sx, sn, so, b = _gemm_case(variant * 7919 + M + N + K + K_o, M, N, K, K_o)
    ref = oracle.dual_gemm(Xq, sx, Wq, sn, so, b, K_o)
    w = q.DualScaleWeight(dev(_pack(Wq, K, K_o)), dev(sn), dev(so), None, K_o, N, K)
    Xq_d = dev(_pack(Xq, K, K_o))
    for out_dtype in (torch.float32, torch.bfloat16):
        try:
            Y, an, ao = q.w8a8_dual_gemm(Xq_d, dev(sx), w, dev(b), M, out_dtype, debug_acc=True, variant=variant)
        except q.QarvdError as e:
            assert e.status == -2                        # a single-accumulator variant refusing K_o > 0
            pytest.skip("variant does not support this shape")
        torch.cuda.synchronize()
        assert np.array_equal(an.cpu().numpy(), ref["acc_n"])
        assert np.array_equal(ao.cpu().numpy(), ref["acc_o"])
        check_y(Y, ref)
    # no bias == +0 bias, and the output stride is honoured
    Ybig = torch.full((M, N + 24), -5.0, dtype=torch.float32, device="cuda")
    q.w8a8_dual_gemm(Xq_d, dev(sx), w, None, M, Y=Ybig[:, :N], variant=variant)
    torch.cuda.synchronize()
    ref0 = oracle.dual_gemm(Xq, sx, Wq, sn, so, None, K_o, want_acc=False)
    assert check_y(Ybig[:, :N], ref0) == 0
    assert torch.all(Ybig[:, N:] == -5.0)


def test_gemm_extreme_accumulator_values():
    M, N, K, K_o = 130, 140, 4096, 1024
    Xq = np.full((M, K), 127, np.int8)
    Wq = np.full((N, K), -127, np.int8)
    Wq[::2] = 127
    one_m, one_n = np.ones(M, np.float32), np.ones(N, np.float32)
    ref = oracle.dual_gemm(Xq, one_m, Wq, one_n, one_n, None, K_o)
    w = q.DualScaleWeight(dev(_pack(Wq, K, K_o)), dev(one_n), dev(one_n), None, K_o, N, K)
    Y, an, ao = q.w8a8_dual_gemm(dev(_pack(Xq, K, K_o)), dev(one_m), w, None, M, torch.float32, debug_acc=True)
    torch.cuda.synchronize()
    assert np.array_equal(an.cpu().numpy(), ref["acc_n"]) and np.array_equal(ao.cpu().numpy(), ref["acc_o"])
    assert abs(int(ref["acc_n"][0, 0])) == 16129 * 3072
    assert check_y(Y, ref) == 0


@pytest.mark.parametrize("variant", [0, 1, 9, 11, 17])
def test_gemm_longest_k_accumulators_at_the_int32_edge(variant):
    """K at the library's limit (K * 127^2 must stay below 2^31): every product +-16129, all of one sign per
    output, so the normal-range sum ends within 0.02 % of INT32_MAX / INT32_MIN."""
    K = 133120                                           # largest multiple of 128 not above the limit of 133143
    M, N, K_o = 40, 48, 32
    Xq = np.full((M, K), 127, np.int8)
    Wq = np.full((N, K), 127, np.int8)
    Wq[1::2] = -127
    one_m, one_n = np.ones(M, np.float32), np.ones(N, np.float32)
    ref = oracle.dual_gemm(Xq, one_m, Wq, one_n, one_n, None, K_o)
    assert int(ref["acc_n"][0, 0]) == 16129 * (K - K_o) > 2 ** 31 - 2 ** 20 and int(ref["acc_n"][0, 1]) == -16129 * (K - K_o)
    w = q.DualScaleWeight(dev(_pack(Wq, K, K_o)), dev(one_n), dev(one_n), None, K_o, N, K)
    Y, an, ao = q.w8a8_dual_gemm(dev(_pack(Xq, K, K_o)), dev(one_m), w, None, M, torch.float32, debug_acc=True, variant=variant)
    torch.cuda.synchronize()
    assert np.array_equal(an.cpu().numpy(), ref["acc_n"]) and np.array_equal(ao.cpu().numpy(), ref["acc_o"])
    assert check_y(Y, ref) == 0


# ------------------------------------------------------------- whole layer, end to end

def run_layer_gpu(L, out_dtype, forced_mask=None, variant=0):
    w = gpu_quantize_weight(L["W"], forced_mask=forced_mask)
    Xd = dev(L["X"])
    Xq, sx = q.quant_act(Xd, w.perm if w.K_o else None, w.K_o)
    M = L["X"].shape[0]
    Y, an, ao = q.w8a8_dual_gemm(Xq, sx, w, dev(L["bias"]), M, out_dtype, debug_acc=True, variant=variant)
    torch.cuda.synchronize()
    return w, Xq, sx, Y, an, ao


def assert_layer_equal(L, out_dtype, forced_mask=None, rows=None):
    w, Xq, sx, Y, an, ao = run_layer_gpu(L, out_dtype, forced_mask)
    o = oracle.quantize_weight(L["W"], forced_mask=forced_mask)
    assert_weight_equal(weight_to_numpy(w), o)
    X = L["X"]
    K = X.shape[1]
    Xq_l = logical(Xq, K, w.K_o)
    sx_g = sx.cpu().numpy()
    if rows is None:
        rows = np.arange(X.shape[0])
    Xq_o, sx_o = oracle.quant_act(X[rows], o["perm"])
    assert np.array_equal(Xq_l[rows], Xq_o) and np.array_equal(sx_g[rows].view(np.uint32), sx_o.view(np.uint32))
    ref = oracle.dual_gemm(Xq_o, sx_o, o["Wq"], o["s_normal"], o["s_outlier"], L["bias"], o["K_o"])
    rt = torch.from_numpy(rows).cuda()
    assert np.array_equal(an[rt].cpu().numpy(), ref["acc_n"])
    assert np.array_equal(ao[rt].cpu().numpy(), ref["acc_o"])
    mism = check_y(Y[rt], ref)
    return o, mism


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
def test_config1_end_to_end(out_dtype):
    L = wl.make_layer(wl.config1()[0])
    o, mism = assert_layer_equal(L, out_dtype)
    assert o["K_o"] == 32 and mism == 0


def test_invariants_on_gpu_match_single_scale_oracle():
    L = wl.small_random_case(77, 150, 320, 256, 0)
    s = oracle.single_scale_linear(L["X"], L["W"], L["bias"])
    for mask in (None, np.ones(256, np.uint8)):
        w, Xq, sx, Y, an, ao = run_layer_gpu(L, torch.float32, forced_mask=mask)
        assert w.K_o == (0 if mask is None else 256)
        acc = (an if mask is None else ao).cpu().numpy()
        zero = (ao if mask is None else an).cpu().numpy()
        assert np.array_equal(acc, s["acc"]) and np.all(zero == 0)
        assert np.array_equal(Y.cpu().numpy().view(np.uint32), s["Y_f32"].view(np.uint32))


def test_determinism_byte_identical_reruns():
    L = wl.make_layer(wl.config1()[0])
    a = run_layer_gpu(L, torch.bfloat16)
    b = run_layer_gpu(L, torch.bfloat16)
    kp = q.packed_k(L["W"].shape[1], a[0].K_o)
    # (the bytes between the packed extent and the padded row stride are never written)
    assert torch.equal(a[1][:, :kp], b[1][:, :kp]) and torch.equal(a[3].view(torch.int16), b[3].view(torch.int16))
    assert torch.equal(a[4], b[4]) and torch.equal(a[5], b[5]) and torch.equal(a[0].codes(), b[0].codes())


def _full_size_names():
    """Every layer of configs 2, 3 (all 30 blocks x 10 linears), 4 and 5."""
    return [s.name for cfg in (2, 3, 4, 5) for s in wl.config_layers(cfg)]


FULL_SIZE = _full_size_names()


def _compared_in_full(spec):
    """Configs 2, 4 and 5 and blocks 0, 14 and 29 of config 3 are compared on every token row; the other
    27 blocks of config 3 (the same six shapes again) on 48 sampled rows."""
    return spec.config != 3 or spec.tags.get("block") in (0, 14, 29)


@pytest.mark.parametrize("name", FULL_SIZE)
def test_full_size_layers(name):
    """BASELINE-size layers in the launch configuration the benchmark times: the whole weight step, and
    Xq, s_x, both accumulators and the bf16 output of EVERY token row and column against the oracle (the
    persistent kernels walk several tiles per workgroup only at these sizes)."""
    spec = wl.find_layer(name)
    L = wl.make_layer(spec)
    rows = None
    if not _compared_in_full(spec):
        rng = np.random.default_rng(spec.seed)
        rows = np.unique(np.concatenate([[0, spec.M - 1], rng.choice(spec.M, 46, replace=False)]))
    o, mism = assert_layer_equal(L, torch.bfloat16, rows=rows)
    assert mism == 0
    assert o["K_o"] == (spec.n_outlier + 31) // 32 * 32


@pytest.mark.parametrize("layer", [wl.TARGET_LAYER, "cfg2.ffn_up.c0", "cfg2.ffn_down.c64"])
def test_full_size_every_variant(layer):
    """Each kernel variant on full-size layers (several tiles per persistent workgroup, ragged last
    row tile): raw accumulators and bf16 outputs of all token rows against the oracle."""
    spec = wl.find_layer(layer)
    L = wl.make_layer(spec)
    w = gpu_quantize_weight(L["W"])
    Xq, sx = q.quant_act(dev(L["X"]), w.perm if w.K_o else None, w.K_o)
    o = oracle.quantize_weight(L["W"])
    Xq_o, sx_o = oracle.quant_act(L["X"], o["perm"])
    ref = oracle.dual_gemm(Xq_o, sx_o, o["Wq"], o["s_normal"], o["s_outlier"], L["bias"], o["K_o"])
    ref_an, ref_ao = torch.from_numpy(ref["acc_n"]).cuda(), torch.from_numpy(ref["acc_o"]).cuda()
    ref_y = torch.from_numpy(ref["Y_bf16"].view(np.int16)).cuda()
    ran = 0
    for variant in range(1, q.gemm_num_variants() + 1):
        try:
            Y, an, ao = q.w8a8_dual_gemm(Xq, sx, w, dev(L["bias"]), spec.M, torch.bfloat16, debug_acc=True, variant=variant)
        except q.QarvdError as e:
            if e.status == -2:                       # this variant cannot run the shape
                continue
            raise
        torch.cuda.synchronize()
        # (exact comparisons of whole matrices, done on the device: equality of integers and of bit patterns)
        assert torch.equal(an, ref_an), q.gemm_variant_name(variant)
        assert torch.equal(ao, ref_ao), q.gemm_variant_name(variant)
        assert torch.equal(Y.view(torch.int16), ref_y), q.gemm_variant_name(variant)
        # the timed path (no accumulator dumps) must give the same bytes
        Y2 = q.w8a8_dual_gemm(Xq, sx, w, dev(L["bias"]), spec.M, torch.bfloat16, variant=variant)
        torch.cuda.synchronize()
        assert torch.equal(Y2.view(torch.int16), Y.view(torch.int16)), q.gemm_variant_name(variant)
        ran += 1
    assert ran >= 4


# More tiles than workgroup slots at sizes the oracle does in full in a moment: every tile shape then walks
# several tiles per persistent workgroup (stage ring carried across tiles, second scale buffer, the next
# tile's prefetch under the epilogue), and every output of those later rounds is compared.
@pytest.mark.parametrize("M,N,K,K_o", [(4352, 4352, 128, 0), (4352, 4352, 256, 32), (2304, 2304, 256, 96),
                                       (2250, 2360, 384, 64), (4400, 4352, 192, 128)])
def test_more_tiles_than_slots_every_variant(M, N, K, K_o):
    Xq, Wq, sx, sn, so, b = _gemm_case(M + N + K + K_o, M, N, K, K_o)
    ref = oracle.dual_gemm(Xq, sx, Wq, sn, so, b, K_o)
    ref_an, ref_ao = torch.from_numpy(ref["acc_n"]).cuda(), torch.from_numpy(ref["acc_o"]).cuda()
    ref_y = {torch.bfloat16: torch.from_numpy(ref["Y_bf16"].view(np.int16)).cuda(),
             torch.float32: torch.from_numpy(ref["Y_f32"].view(np.int32)).cuda()}
    w = q.DualScaleWeight(dev(_pack(Wq, K, K_o)), dev(sn), dev(so), None, K_o, N, K)
    Xq_d, sx_d, b_d = dev(_pack(Xq, K, K_o)), dev(sx), dev(b)
    ran = 0
    for variant in range(0, q.gemm_num_variants() + 1):
        for out_dtype in (torch.bfloat16, torch.float32):
            try:
                Y, an, ao = q.w8a8_dual_gemm(Xq_d, sx_d, w, b_d, M, out_dtype, debug_acc=True, variant=variant)
            except q.QarvdError as e:
                if e.status == -2:
                    continue
                raise
            torch.cuda.synchronize()
            name = q.gemm_variant_name(variant) if variant else "heuristic"
            assert torch.equal(an, ref_an) and torch.equal(ao, ref_ao), name
            bits = Y.view(torch.int16) if out_dtype == torch.bfloat16 else Y.view(torch.int32)
            assert torch.equal(bits, ref_y[out_dtype]), name
            Y2 = q.w8a8_dual_gemm(Xq_d, sx_d, w, b_d, M, out_dtype, variant=variant)     # the timed build
            torch.cuda.synchronize()
            assert torch.equal(Y2.view(torch.int16), Y.view(torch.int16)), name
            ran += 1
    assert ran >= 8


@pytest.mark.parametrize("variant", [0, 1, 5, 9, 11, 13, 15, 17, 19, 21])
@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
def test_rows_below_a_ragged_last_tile_are_not_written(variant, out_dtype):
    """Y is a view of the first M rows of a larger sentinel-filled buffer: the rows of the last row of
    tiles that lie below the matrix (masked by the store's buffer range) and the columns beyond N must
    keep the sentinel."""
    M, N, K, K_o = 300 + 72, 392, 256, 32                 # 372 = 256 + 116: ragged for every tile height
    Xq, Wq, sx, sn, so, b = _gemm_case(variant + 5, M, N, K, K_o)
    ref = oracle.dual_gemm(Xq, sx, Wq, sn, so, b, K_o)
    w = q.DualScaleWeight(dev(_pack(Wq, K, K_o)), dev(sn), dev(so), None, K_o, N, K)
    big = torch.full((M + 300, N + 40), -7.0, dtype=out_dtype, device="cuda")
    try:
        q.w8a8_dual_gemm(dev(_pack(Xq, K, K_o)), dev(sx), w, dev(b), M, Y=big[:M, :N], variant=variant)
    except q.QarvdError as e:
        assert e.status == -2
        pytest.skip("variant does not support this shape")
    torch.cuda.synchronize()
    assert check_y(big[:M, :N], ref) == 0
    assert torch.all(big[M:, :] == -7.0) and torch.all(big[:M, N:] == -7.0)
