"""The pins must be able to fail: one plausible mistake at a time is planted in a COPY of the oracle's C
source (a dropped term, a wrong sign or index, a swapped operand, another rounding), the copy is compiled
and swapped in for the oracle's library, and the pin named beside the mistake has to raise.

Everything here runs on the CPU, in a temporary directory; the committed oracle is not touched and the
HIP library is not involved.
"""
import ctypes as C
import importlib
import subprocess

import pytest

import oracle

SRC = (oracle._SRC).read_text()

GEMM_MERGE = ("            r = (float)acc_o * s_outlier[j];\n"
              "            r = fmaf((float)acc_n, s_normal[j], r);")

# (what is planted, text in the source, its replacement, occurrences, pin module, pin function, its arguments)
MISTAKES = [
    ("median of an even-length vector takes the lower middle value",
     "m = (t[n / 2 - 1] + t[n / 2]) / 2.0;", "m = t[n / 2 - 1];", 1,
     "test_oracle_detector", "test_detector_hand_worked_even_length", {}),
    ("deviations enter the MAD with their sign",
     "d[k] = fabs(vd[k] - med);", "d[k] = vd[k] - med;", 1,
     "test_oracle_detector", "test_detector_hand_worked_even_length", {}),
    ("0.6745 mistyped",
     "c = tau / 0.6745;", "c = tau / 0.6475;", 1,
     "test_oracle_detector", "test_detector_hand_worked_even_length", {}),
    ("the smaller of the two thresholds",
     "T = (T1 > T2) ? T1 : T2;", "T = (T1 < T2) ? T1 : T2;", 1,
     "test_oracle_detector", "test_detector_hand_worked_even_length", {}),
    ("the alpha term of the threshold dropped",
     "T = (T1 > T2) ? T1 : T2;", "T = T1;", 1,
     "test_oracle_detector", "test_detector_hand_worked_mad_zero", {}),
    ("a channel AT the threshold is flagged",
     "flag[k] = (vd[k] > T) ? 1 : 0;", "flag[k] = (vd[k] >= T) ? 1 : 0;", 1,
     "test_oracle_detector", "test_detector_hand_worked_mad_zero", {}),
    ("column norms as sums of magnitudes",
     "S = S + w * w;", "S = S + fabs(w);", 1,
     "test_oracle_detector", "test_column_norms_exact_sum_and_axis", {}),
    ("column norms summed in single precision",
     "double S = 0.0;\n        for (int j = 0; j < N; ++j) {\n            double w",
     "float S = 0.0f;\n        for (int j = 0; j < N; ++j) {\n            float w", 1,
     "test_oracle_detector", "test_column_norms_are_summed_in_double", {}),
    ("the outlier count rounded down to the alignment",
     "target = ((n + align - 1) / align) * align;", "target = (n / align) * align;", 1,
     "test_oracle_detector", "test_alignment_hand_worked", {}),
    ("alignment fills with the smallest norms",
     "if (best < 0 || v[k] > v[best])", "if (best < 0 || v[k] < v[best])", 1,
     "test_oracle_detector", "test_alignment_hand_worked", {}),
    ("alignment breaks ties towards the larger index",
     "if (best < 0 || v[k] > v[best])", "if (best < 0 || v[k] >= v[best])", 1,
     "test_oracle_detector", "test_alignment_hand_worked", {}),
    ("outlier channels in descending order",
     "    for (int k = 0; k < K; ++k)\n        if (sel[k])\n            perm[p++] = k;\n    if (K_o)",
     "    for (int k = K - 1; k >= 0; --k)\n        if (sel[k])\n            perm[p++] = k;\n    if (K_o)", 1,
     "test_oracle_detector", "test_alignment_properties", {"seed": 0}),
    ("a forced outlier set is aligned as well",
     "            if (flag_out)\n                memcpy(flag_out, sel, (size_t)K);\n        } else {",
     "            if (flag_out)\n                memcpy(flag_out, sel, (size_t)K);\n"
     "            rc = oracle_align(v, K, align, sel, &K_o);\n        } else {", 1,
     "test_oracle_detector", "test_forced_mask_bypasses_detection_and_alignment", {}),
    ("round half away from zero",
     "r = rintf(x / s);", "r = roundf(x / s);", 1,
     "test_oracle_quant_gemm", "test_round_half_to_even_and_clip", {}),
    ("the code -128 allowed",
     "r = -qmax;", "r = -qmax - 1.0f;", 1,
     "test_oracle_quant_gemm", "test_static_activation_scale_variant", {}),
    ("activation scale absmax / 128",
     "s = a / 127.0f;\n        s_x[m] = s;", "s = a / 128.0f;\n        s_x[m] = s;", 1,
     "test_oracle_quant_gemm", "test_quant_act_matches_numpy_recomputation_and_bounds", {}),
    ("the permutation applied as a scatter",
     "Xq[(size_t)m * K + p] = quantize_one(x[k], s);", "Xq[(size_t)m * K + k] = quantize_one(x[p], s);", 1,
     "test_oracle_quant_gemm", "test_quant_act_perm_is_a_gather", {}),
    ("a zero scale divides",
     "    if (s == 0.0f)\n        return 0;\n", "", 1,
     "test_oracle_quant_gemm", "test_static_activation_scale_variant", {}),
    ("the outlier block quantized with the normal scale",
     "Wq[(size_t)j * K + p] = quantize_sym(w[perm[p]], so, qmax);",
     "Wq[(size_t)j * K + p] = quantize_sym(w[perm[p]], sn, qmax);", 1,
     "test_oracle_quant_gemm", "test_weight_scales_and_blocks", {}),
    ("the normal scale taken over all channels",
     "        for (int p = K_o; p < K; ++p) {\n            float a = fabsf(w[perm[p]]);\n            if (a > a_n)",
     "        for (int p = 0; p < K; ++p) {\n            float a = fabsf(w[perm[p]]);\n            if (a > a_n)", 1,
     "test_oracle_quant_gemm", "test_weight_scales_and_blocks", {}),
    ("the two weight scales swapped in the epilogue",
     GEMM_MERGE, GEMM_MERGE.replace("s_outlier", "s_tmp").replace("s_normal", "s_outlier").replace("s_tmp", "s_normal"), 2,
     "test_oracle_quant_gemm", "test_invariant_all_outliers_equals_single_scale", {"seed": 0}),
    ("the normal accumulator also sums the outlier block",
     "            for (int p = K_o; p < K; ++p)\n                acc_n +=",
     "            for (int p = 0; p < K; ++p)\n                acc_n +=", 2,
     "test_oracle_quant_gemm", "test_accumulators_brute_force_int64", {"seed": 1}),
    ("codes of X read as unsigned bytes",
     "acc_n += (int32_t)x[p] * (int32_t)w[p];", "acc_n += (int32_t)(uint8_t)x[p] * (int32_t)w[p];", 2,
     "test_oracle_quant_gemm", "test_accumulators_brute_force_int64", {"seed": 1}),
    ("the last epilogue step as a multiply and an add",
     "            r = fmaf(r, s_x[m], b);", "            r = r * s_x[m];\n            r = r + b;", 2,
     "test_oracle_quant_gemm", "test_epilogue_exact_rational_check", {}),
    ("the blocks merged in the other order",
     GEMM_MERGE, "            r = (float)acc_n * s_normal[j];\n            r = fmaf((float)acc_o, s_outlier[j], r);", 2,
     "test_oracle_quant_gemm", "test_epilogue_exact_rational_check", {}),
    ("the bias dropped",
     "float b = bias ? bias[j] : 0.0f;", "float b = 0.0f;", 2,
     "test_oracle_quant_gemm", "test_epilogue_exact_rational_check", {}),
    ("bf16 rounds half up",
     "u += 0x7FFFu + ((u >> 16) & 1u);", "u += 0x8000u;", 1,
     "test_oracle_quant_gemm", "test_bf16_rounding_ties_to_even", {}),
    ("the GELU's cubic term written as a square",
     "0.044715 * xd * xd * xd", "0.044715 * xd * xd", 1,
     "test_oracle_chain", "test_gelu_matches_the_tanh_definition_in_double", {}),
    ("the GELU's sqrt(2/pi) written as sqrt(pi/2)",
     "sqrt(2.0 / 3.14159265358979323846)", "sqrt(3.14159265358979323846 / 2.0)", 1,
     "test_oracle_chain", "test_gelu_matches_the_tanh_definition_in_double", {}),
    ("the activation applied when it is switched off",
     "            if (act == 1)\n                r = oracle_gelu_tanh(r);",
     "            if (act == 0)\n                r = oracle_gelu_tanh(r);", 1,
     "test_oracle_chain", "test_q8_epilogue_codes", {"act": 0}),
    ("the percentile position taken as n p",
     "double h = (double)(n - 1) * P[c];", "double h = (double)n * P[c]; if (h > n - 1) h = n - 1;", 1,
     "test_oracle_clip", "test_clip_values_errors_and_choice", {"n": 1000, "qmax": 127.0}),
    ("the clipped value without interpolation",
     "clip[c] = (float)((double)a[lo] + frac * ((double)a[hi] - (double)a[lo]));", "clip[c] = a[lo];", 1,
     "test_oracle_clip", "test_small_example_by_hand", {}),
    ("a tie in the clip search goes to the smaller percentile",
     "if (sse[c] < sse[best])", "if (sse[c] <= sse[best])", 1,
     "test_oracle_clip", "test_each_percentile_can_win", {}),
    ("the clip search of the normal block runs over the whole row",
     "oracle_clip_search(blk + K_o, K - K_o, qmax, &sn, &cn, NULL, NULL)",
     "oracle_clip_search(blk, K, qmax, &sn, &cn, NULL, NULL)", 1,
     "test_oracle_clip", "test_rows_with_clip_search", {"bits": 8}),
]


@pytest.mark.parametrize("what,old,new,count,module,pin,kwargs", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_the_named_pin_catches_the_planted_mistake(tmp_path, monkeypatch, what, old, new, count, module, pin, kwargs):
    assert SRC.count(old) == count, "the oracle's source no longer holds this text %d time(s)" % count
    c_file, so_file = tmp_path / "mistake.c", tmp_path / "libmistake.so"
    c_file.write_text(SRC.replace(old, new))
    flags = [f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.run(["gcc", *flags, str(c_file), "-o", str(so_file), "-lm"], check=True)
    oracle._load()                                      # the real library is built and loaded first
    monkeypatch.setattr(oracle, "_lib", C.CDLL(str(so_file)))
    check = getattr(importlib.import_module(module), pin)
    with pytest.raises(AssertionError):
        check(**kwargs)


def test_the_pins_pass_on_an_unchanged_copy(tmp_path, monkeypatch):
    """The swap itself breaks nothing: an unmodified copy passes the same pins."""
    c_file, so_file = tmp_path / "copy.c", tmp_path / "libcopy.so"
    c_file.write_text(SRC)
    flags = [f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.run(["gcc", *flags, str(c_file), "-o", str(so_file), "-lm"], check=True)
    oracle._load()
    monkeypatch.setattr(oracle, "_lib", C.CDLL(str(so_file)))
    for _, _, _, _, module, pin, kwargs in MISTAKES:
        getattr(importlib.import_module(module), pin)(**kwargs)
