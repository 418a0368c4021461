"""The GPU parity tests must be able to fail.  One mistake at a time is planted in a COPY of the CPU oracle
(never in a kernel: every GPU launch here is an ordinary, valid one), the copy is swapped in for the oracle's
library, and the parity test named beside the mistake has to report a mismatch against the unchanged HIP path.
"""
import ctypes as C
import importlib
import subprocess

import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2605_21072_amd")

SRC = (oracle._SRC).read_text()

GEMM_MERGE = ("            r = (float)acc_o * s_outlier[j];\n"
              "            r = fmaf((float)acc_n, s_normal[j], r);")

# (what is planted in the oracle, text, replacement, occurrences, test module, parity test, its arguments)
MISTAKES = [
    ("oracle rounds half away from zero",
     "r = rintf(x / s);", "r = roundf(x / s);", 1,
     "test_gpu_parity", "test_quant_act_rounding_boundaries", {"K": 1536, "amax": 100.3}),
    ("oracle applies the permutation as a scatter",
     "Xq[(size_t)m * K + p] = quantize_one(x[k], s);", "Xq[(size_t)m * K + k] = quantize_one(x[p], s);", 1,
     "test_gpu_parity", "test_quant_act_parity", {"M": 33, "K": 1536, "c": 8, "dtype": "f32"}),
    ("oracle's activation scale is absmax / 128",
     "s = a / 127.0f;\n        s_x[m] = s;", "s = a / 128.0f;\n        s_x[m] = s;", 1,
     "test_gpu_parity", "test_quant_act_parity", {"M": 9, "K": 8960, "c": 64, "dtype": "f32"}),
    ("oracle's activation absmax forgets the absolute value",
     "float t = fabsf(x[k]);", "float t = x[k];", 1,
     "test_gpu_parity", "test_quant_act_parity", {"M": 33, "K": 1536, "c": 8, "dtype": "f32"}),
    ("oracle's normal accumulator also sums the outlier block",
     "            for (int p = K_o; p < K; ++p)\n                acc_n +=",
     "            for (int p = 0; p < K; ++p)\n                acc_n +=", 2,
     "test_gpu_parity", "test_gemm_accumulators_and_outputs", {"variant": 0, "M": 300, "N": 200, "K": 384, "K_o": 32}),
    ("oracle swaps the two weight scales in the epilogue",
     GEMM_MERGE, GEMM_MERGE.replace("s_outlier", "s_tmp").replace("s_normal", "s_outlier").replace("s_tmp", "s_normal"), 2,
     "test_gpu_parity", "test_gemm_accumulators_and_outputs", {"variant": 0, "M": 300, "N": 200, "K": 384, "K_o": 32}),
    ("oracle merges the blocks in the other order (one rounding apart)",
     GEMM_MERGE, "            r = (float)acc_n * s_normal[j];\n            r = fmaf((float)acc_o, s_outlier[j], r);", 2,
     "test_gpu_parity", "test_gemm_accumulators_and_outputs", {"variant": 11, "M": 520, "N": 384, "K": 1536, "K_o": 64}),
    ("oracle drops the bias",
     "float b = bias ? bias[j] : 0.0f;", "float b = 0.0f;", 2,
     "test_gpu_parity", "test_gemm_accumulators_and_outputs", {"variant": 0, "M": 64, "N": 96, "K": 130, "K_o": 7}),
    ("oracle rounds the outlier count down to the alignment",
     "target = ((n + align - 1) / align) * align;", "target = (n / align) * align;", 1,
     "test_gpu_parity", "test_quantize_weight_detected", {"seed": 1, "N": 300, "K": 320, "c": 20}),
    ("oracle multiplies tau by 0.6745 instead of dividing",
     "c = tau / 0.6745;", "c = tau * 0.6745;", 1,
     "test_gpu_parity", "test_quantize_weight_detector_parameters", {"tau": 3.5, "alpha": 0.0}),
    ("oracle quantizes the outlier block with the normal scale",
     "Wq[(size_t)j * K + p] = quantize_sym(w[perm[p]], so, qmax);",
     "Wq[(size_t)j * K + p] = quantize_sym(w[perm[p]], sn, qmax);", 1,
     "test_gpu_parity", "test_quantize_weight_detected", {"seed": 0, "N": 64, "K": 128, "c": 3}),
    ("oracle sums the column norms in single precision",
     "double S = 0.0;\n        for (int j = 0; j < N; ++j) {\n            double w",
     "float S = 0.0f;\n        for (int j = 0; j < N; ++j) {\n            float w", 1,
     "test_gpu_parity", "test_quantize_weight_detected", {"seed": 4, "N": 1536, "K": 1536, "c": 8}),
    ("oracle's GELU takes the sigmoid form's constant (1.702 x) for the tanh argument",
     "sqrt(2.0 / 3.14159265358979323846) * (xd + 0.044715 * xd * xd * xd)", "0.851 * xd", 1,
     "test_gpu_chain", "test_q8_gemm_codes_match_oracle", {"act": 1, "variant": 0, "M": 300, "N": 208, "K": 384, "K_o": 32}),
    ("oracle's chained epilogue truncates instead of rounding",
     "r = rintf(x / s);", "r = truncf(x / s);", 1,
     "test_gpu_chain", "test_q8_gemm_codes_match_oracle", {"act": 0, "variant": 0, "M": 300, "N": 208, "K": 384, "K_o": 32}),
    ("oracle's clip search sums absolute instead of squared errors",
     "sse[c] += (double)e * (double)e;", "sse[c] += fabs((double)e);", 1,
     "test_gpu_clip", "test_clip_search_matches_oracle", {"bits": 8, "seed": 1, "N": 300, "K": 320, "c": 20}),
]


def _swap_in(tmp_path, monkeypatch, text):
    c_file, so_file = tmp_path / "oracle_copy.c", tmp_path / "liboracle_copy.so"
    c_file.write_text(text)
    flags = [f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.run(["gcc", *flags, str(c_file), "-o", str(so_file), "-lm"], check=True)
    oracle._load()
    monkeypatch.setattr(oracle, "_lib", C.CDLL(str(so_file)))


def _resolve(module, name):
    return getattr(importlib.import_module(module), name)


@pytest.mark.parametrize("what,old,new,count,module,test,kwargs", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_parity_test_reports_the_planted_mistake(tmp_path, monkeypatch, what, old, new, count, module, test, kwargs):
    assert torch.cuda.is_available(), "GPU tests need a device"
    assert SRC.count(old) == count, "the oracle's source no longer holds this text %d time(s)" % count
    fn = _resolve(module, test)
    _swap_in(tmp_path, monkeypatch, SRC.replace(old, new))
    with pytest.raises(AssertionError):
        fn(**kwargs)
    torch.cuda.synchronize()


def test_the_same_parity_tests_pass_against_an_unchanged_copy(tmp_path, monkeypatch):
    assert torch.cuda.is_available(), "GPU tests need a device"
    _swap_in(tmp_path, monkeypatch, SRC)
    for _, _, _, _, module, test, kwargs in MISTAKES:
        _resolve(module, test)(**kwargs)
    torch.cuda.synchronize()
