"""Pins for the oracle's offline weight step (norms, detector, alignment, permutation).

None of these call the HIP library.  Each pin checks the oracle against something
other than itself: a hand-worked example, numpy / scipy library routines, a
textbook form of the same criterion, or a property the paper states.
"""
import math
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest
import scipy.stats

import oracle
import workloads as wl

GOLD = {}
for line in (Path(__file__).parent / "golden" / "paper_constants.txt").read_text().splitlines():
    line = line.split("#")[0].split()
    if len(line) == 2:
        GOLD[line[0]] = float(line[1])


def test_paper_constants_are_the_defaults():
    import inspect
    sig = inspect.signature(oracle.quantize_weight)
    assert sig.parameters["tau"].default == GOLD["tau"]
    assert sig.parameters["alpha"].default == GOLD["alpha"]
    assert sig.parameters["align"].default == GOLD["align"]
    # one aligned block of 32 in a 1536-wide layer is the paper's "2.1 %" of input channels
    assert round(100.0 * GOLD["align"] / wl.HIDDEN, 1) == GOLD["outlier_fraction_percent"]


def test_column_norms_exact_sum_and_axis():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((37, 11)).astype(np.float32)   # non-square: a wrong axis changes the length
    v = oracle.column_norms(W)
    assert v.shape == (11,)
    for k in range(11):
        exact = math.fsum(float(x) * float(x) for x in W[:, k])   # correctly rounded fp64 sum of exact squares
        ref = np.float32(math.sqrt(exact))
        assert abs(float(v[k]) - float(ref)) <= float(np.spacing(ref))
    # versus the library norm
    lib = np.linalg.norm(W.astype(np.float64), axis=0).astype(np.float32)
    assert np.all(np.abs(v - lib) <= np.spacing(lib))


def test_column_norms_closed_form():
    W = np.zeros((4, 3), np.float32)
    W[:, 0] = [3, 4, 0, 0]          # 5
    W[:, 1] = [1, 1, 1, 1]          # 2
    W[:, 2] = [0, 0, 0, -7]         # 7
    assert oracle.column_norms(W).tolist() == [5.0, 2.0, 7.0]


def test_column_norms_are_summed_in_double():
    # 4096^2 = 2^24: a single-precision running sum cannot absorb the 4095 ones that follow (it would
    # return exactly 4096), the double sum is the integer 16781311 and its root rounds to 4096.5
    W = np.ones((4096, 2), np.float32)
    W[0, 0] = 4096.0
    W[:, 1] = 0.25
    v = oracle.column_norms(W)
    assert float(v[0]) == float(np.float32(math.sqrt(4096 ** 2 + 4095))) == 4096.5
    assert float(v[1]) == 16.0


def test_detector_hand_worked_even_length():
    # v = 1,2,3,4: median 2.5; |v-med| = 1.5,.5,.5,1.5 -> MAD 1.0
    flag, st = oracle.detect(np.array([1, 2, 3, 4], np.float32), tau=3.5, alpha=1.2)
    assert st["med"] == 2.5 and st["mad"] == 1.0
    assert st["T"] == 2.5 + (3.5 / 0.6745) * 1.0      # Z-score term (7.689..) binds over 1.2*2.5
    assert flag.tolist() == [0, 0, 0, 0]


def test_detector_hand_worked_mad_zero():
    # seven equal norms and one large: MAD = 0, so the minimum-magnitude term alpha*med decides
    v = np.array([1, 1, 1, 1, 1, 1, 1, 10], np.float32)
    flag, st = oracle.detect(v)
    assert st["med"] == 1.0 and st["mad"] == 0.0 and st["T"] == 1.2
    assert flag.tolist() == [0] * 7 + [1]
    # strict inequality: a norm exactly on the threshold is not an outlier
    v2 = np.array([1, 1, 1, 1, 1, 1, 1, 1.5], np.float32)
    flag2, st2 = oracle.detect(v2, tau=3.5, alpha=1.5)
    assert st2["T"] == 1.5 and flag2.sum() == 0


def test_detector_odd_length_median():
    v = np.array([5, 1, 3], np.float32)
    _, st = oracle.detect(v)
    assert st["med"] == 3.0 and st["mad"] == 2.0


@pytest.mark.parametrize("seed,K", [(0, 64), (1, 257), (2, 1536), (3, 1000)])
def test_detector_matches_library_median_and_mad(seed, K):
    rng = np.random.default_rng(seed)
    v = np.abs(rng.standard_normal(K)).astype(np.float32) + 0.5
    v[rng.choice(K, 5, replace=False)] *= 8
    flag, st = oracle.detect(v)
    vd = v.astype(np.float64)
    med = np.median(vd)
    mad = scipy.stats.median_abs_deviation(vd, scale=1.0)
    assert st["med"] == med and st["mad"] == mad
    # textbook Modified Z-score (Iglewicz & Hoaglin) AND the minimum-magnitude condition
    Mz = 0.6745 * (vd - med) / mad
    both = (Mz > 3.5) & (vd > 1.2 * med)
    T = max(med + 3.5 / 0.6745 * mad, 1.2 * med)
    margin = np.abs(vd - T) > 1e-9 * T                   # the two forms may differ only on the boundary
    assert np.array_equal(flag.astype(bool)[margin], both[margin])
    assert flag.sum() == st["n_det"] < K / 2


def test_detector_tau_and_alpha_are_used():
    rng = np.random.default_rng(5)
    v = (1.0 + 0.05 * rng.standard_normal(512)).astype(np.float32)
    v[7] = 1.19
    v[9] = 1.3
    f, _ = oracle.detect(v, tau=3.5, alpha=1.2)
    assert f[9] == 1 and f[7] == 0
    f, _ = oracle.detect(v, tau=3.5, alpha=1.1)          # lower floor: 1.19 now passes both terms?
    vd = v.astype(np.float64)
    med = np.median(vd)
    mad = np.median(np.abs(vd - med))
    assert f[7] == (vd[7] > max(med + 3.5 / 0.6745 * mad, 1.1 * med))
    f_hi, st_hi = oracle.detect(v, tau=50.0, alpha=0.0)   # huge tau: Z term binds and rejects all
    assert st_hi["T"] == med + 50.0 / 0.6745 * mad and f_hi.sum() == 0


def test_planted_outliers_recovered_on_workload():
    # Gaussian columns have MAD ~ 0.6745*med/sqrt(2N): the Z term alone sits near 1.06*med for N=1536,
    # below alpha*med = 1.2*med, so the alpha term binds (the paper's "false outlier" situation).
    L = wl.make_layer(wl.config1()[0])
    q = oracle.quantize_weight(L["W"])
    assert q["stats"]["n_det"] == 8
    assert np.array_equal(np.flatnonzero(q["flag"]), L["planted"])
    assert q["stats"]["T"] == 1.2 * q["stats"]["med"]
    assert q["K_o"] == 32
    # the eight planted channels sit in the outlier block
    assert set(L["planted"]).issubset(set(q["perm"][:32].tolist()))


def test_alpha_term_prevents_false_outliers():
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((256, 8192)) * 0.02).astype(np.float32)   # smooth layer, no planted outliers
    q = oracle.quantize_weight(W)
    assert q["K_o"] == 0 and q["stats"]["n_det"] == 0
    assert np.array_equal(q["perm"], np.arange(8192))
    q0 = oracle.quantize_weight(W, alpha=0.0)           # Z-score alone flags a few of 8192 smooth channels
    assert q0["stats"]["n_det"] > 0
    assert q0["K_o"] % 32 == 0 and q0["K_o"] >= q0["stats"]["n_det"]


def test_constant_norm_layer_has_no_outliers():
    W = np.ones((8, 64), np.float32)
    q = oracle.quantize_weight(W)
    assert q["stats"]["mad"] == 0.0 and q["K_o"] == 0


def test_alignment_hand_worked():
    v = np.array([1, 9, 2, 8, 3, 7, 4, 7], np.float32)
    sel = np.array([0, 1, 0, 0, 0, 0, 0, 0], np.uint8)
    out, ko = oracle.align(v, sel, align=4)
    # grows to 4 with the largest remaining norms: 8 (idx 3), then 7 (idx 5 before idx 7: ties -> smaller index)
    assert ko == 4 and out.tolist() == [0, 1, 0, 1, 0, 1, 0, 1]
    out, ko = oracle.align(v, sel, align=3)
    assert ko == 3 and out.tolist() == [0, 1, 0, 1, 0, 1, 0, 0]
    out, ko = oracle.align(v, np.zeros(8, np.uint8), align=4)
    assert ko == 0 and out.sum() == 0                    # nothing detected: layer stays single-scale
    out, ko = oracle.align(v, np.array([1, 1, 1, 1, 1, 0, 0, 0], np.uint8), align=16)
    assert ko == 8 and out.sum() == 8                    # capped at K
    out, ko = oracle.align(v, sel, align=1)
    assert ko == 1 and out.tolist() == sel.tolist()


@pytest.mark.parametrize("seed", range(6))
def test_alignment_properties(seed):
    rng = np.random.default_rng(100 + seed)
    K, N = 320, 96
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    n_pl = int(rng.integers(1, 70))
    cols = rng.choice(K, n_pl, replace=False)
    W[:, cols] *= rng.uniform(10, 40, n_pl).astype(np.float32)
    q = oracle.quantize_weight(W)
    K_o, n_det, v, perm = q["K_o"], q["stats"]["n_det"], q["v"], q["perm"]
    assert n_det == n_pl
    assert K_o % 32 == 0 and 0 <= K_o - n_det < 32
    out_set, norm_set = perm[:K_o], perm[K_o:]
    assert set(np.flatnonzero(q["flag"])).issubset(set(out_set.tolist()))
    # every filler has a norm >= every channel left in the normal block
    assert v[out_set].min() >= v[norm_set].max()
    # permutation: bijection, both blocks strictly increasing
    assert np.array_equal(np.sort(perm), np.arange(K))
    assert np.all(np.diff(out_set) > 0) and np.all(np.diff(norm_set) > 0)


def test_forced_mask_bypasses_detection_and_alignment():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((5, 10)).astype(np.float32)
    mask = np.zeros(10, np.uint8)
    mask[[2, 7, 9]] = 1
    q = oracle.quantize_weight(W, forced_mask=mask)
    assert q["K_o"] == 3 and q["perm"].tolist() == [2, 7, 9, 0, 1, 3, 4, 5, 6, 8]
    q = oracle.quantize_weight(W, forced_mask=np.ones(10, np.uint8))
    assert q["K_o"] == 10 and q["perm"].tolist() == list(range(10))


def test_packed_size_ratio_is_close_to_the_papers():
    # INT8 weights + two fp32 scales per row + int32 perm vs bf16 weights: ~1.98-1.99x per layer;
    # the paper's whole-model 2.64 GB -> 1.34 GB is 1.97x (some modules stay bf16).
    for N, K in ((1536, 1536), (8960, 1536), (1536, 8960)):
        packed = N * K + 8 * N + 4 * K
        ratio = 2.0 * N * K / packed
        assert 1.97 <= ratio < 2.0
    assert round(GOLD["model_size_bf16_gb"] / GOLD["model_size_int8_gb"], 2) == 1.97
