"""GPU parity of the percentile-clip scale search in the offline weight step (cfg.clip_search = 1; Sec. 4.1
"Quantization Implementation") against the oracle: permutation, both scales of every row and every code
bit-exact, for INT8 and packed INT4 weights."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2605_21072_amd")
from gpu_util import assert_weight_equal, dev, gpu_quantize_weight, weight_to_numpy  # noqa: E402


def heavy_tailed(seed, N, K, n_out):
    rng = np.random.default_rng(seed)
    W = (rng.standard_t(3, (N, K)) * 0.02).astype(np.float32)
    if n_out:
        W[:, rng.choice(K, n_out, replace=False)] *= 25
    return W


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("seed,N,K,c", [(0, 64, 128, 3), (1, 300, 320, 20), (2, 257, 1000, 9), (3, 96, 37, 0),
                                        (4, 130, 1536, 8), (5, 40, 5000, 30)])
def test_clip_search_matches_oracle(bits, seed, N, K, c):
    W = heavy_tailed(7000 + seed, N, K, c)
    W[N // 2] = 0                                                    # an all-zero row: scale 0, codes 0
    o = oracle.quantize_weight(W, bits=bits, clip_search=True)
    w = gpu_quantize_weight(W, bits=bits, clip_search=True)
    assert w.K_o == o["K_o"] and np.array_equal(w.perm.cpu().numpy(), o["perm"])
    assert np.array_equal(w.s_normal.cpu().numpy().view(np.uint32), o["s_normal"].view(np.uint32))
    assert np.array_equal(w.s_outlier.cpu().numpy().view(np.uint32), o["s_outlier"].view(np.uint32))
    assert np.array_equal(w.logical_Wq().cpu().numpy(), o["Wq"])
    base = oracle.quantize_weight(W, bits=bits)                      # and it is not the absmax result
    assert np.any(o["s_normal"] < base["s_normal"])


def test_clip_search_forced_splits_and_errors():
    W = heavy_tailed(7100, 48, 96, 0)
    for mask in (np.zeros(96, np.uint8), np.ones(96, np.uint8), (np.arange(96) % 3 == 0).astype(np.uint8)):
        o = oracle.quantize_weight(W, forced_mask=mask, clip_search=True)
        g = weight_to_numpy(gpu_quantize_weight(W, forced_mask=mask, clip_search=True))
        assert_weight_equal(g, o)
    big = torch.zeros((2, 16512), dtype=torch.float32, device="cuda")
    with pytest.raises(q.QarvdError) as e:
        q.quantize_weight(big, clip_search=True)                     # K above the search's limit
    assert e.value.status == -2


def test_clip_search_layer_end_to_end():
    """DiT-shaped layer (config 1) through the whole path with clip-searched scales: bf16 outputs within 1 ulp."""
    from gpu_util import bf16_bits, bf16_ulp_distance
    spec = wl.config_layers(1)[0]
    L = wl.make_layer(spec)
    o = oracle.quantize_weight(L["W"], clip_search=True)
    w = gpu_quantize_weight(L["W"], clip_search=True)
    assert_weight_equal(weight_to_numpy(w), o)
    Xq_o, sx_o = oracle.quant_act(L["X"], o["perm"])
    ref = oracle.dual_gemm(Xq_o, sx_o, o["Wq"], o["s_normal"], o["s_outlier"], L["bias"], o["K_o"])
    Y = q.w8a8_linear(dev(L["X"]), w, dev(L["bias"]))
    torch.cuda.synchronize()
    assert bf16_ulp_distance(bf16_bits(Y), ref["Y_bf16"]).max() <= 1


@pytest.mark.parametrize("layer", [wl.TARGET_LAYER, "cfg2.ffn_down.c64"])
def test_clip_search_full_size(layer):
    """Benchmark-size layers (8960 x 1536 and 1536 x 8960): every scale and every code against the oracle."""
    L = wl.make_layer(wl.find_layer(layer))
    o = oracle.quantize_weight(L["W"], clip_search=True)
    w = gpu_quantize_weight(L["W"], clip_search=True)
    assert_weight_equal(weight_to_numpy(w), o)
