"""Host-side checks of the C ABI: the library loads, exports every declared symbol, and rejects
bad arguments with status codes before anything is launched (no GPU needed)."""
import ctypes as C
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def lib():
    import paper_2605_21072_amd as q
    if not q.lib_path().exists():
        from paper_2605_21072_amd import build
        build.build()
    return q.load_library()


def declared_symbols():
    text = (ROOT / "include" / "qarvd.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qarvd_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"qarvd_quantize_weight", "qarvd_quant_act", "qarvd_w8a8_dual_gemm"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "libqarvd.so does not export %s" % n


def test_packed_geometry(lib):
    import paper_2605_21072_amd as q
    assert q.packed_normal_offset(0) == 0 and q.packed_normal_offset(1) == 32 and q.packed_normal_offset(64) == 64
    assert q.packed_k(1536, 0) == 1536 and q.packed_k(1536, 32) == 1536 and q.packed_k(8960, 96) == 8960
    assert q.packed_k(130, 7) == 256            # 32 + 123 -> 155 -> 256
    assert q.packed_k(96, 96) == 128
    assert q.packed_k(1536, -1) == 1664
    assert q.packed_ld(1536, 32) == 1664 and q.packed_ld(8960, 0) == 9088 and q.packed_ld(0, 0) == 0
    for K in (96, 384, 1536, 5120, 13824, 20000):
        for ko in (0, 32, -1):
            ld = q.packed_ld(K, ko)
            assert ld % 128 == 0 and ld % 512 != 0 and 128 <= ld - q.packed_k(K, ko) <= 256
    assert q.packed_k(0, 0) == 0 and q.packed_k(10, 11) == 0 and q.packed_k(133144, 0) == 0
    for K in (1, 37, 128, 1000, 1536):
        worst = max(q.packed_k(K, ko) for ko in range(0, K + 1))
        assert worst <= q.packed_k(K, -1)
    assert q.quantize_weight_workspace(16, 1536) >= 33 * 1536
    assert q.quantize_weight_workspace(0, 5) == 0


def test_defaults_and_status_strings(lib):
    from paper_2605_21072_amd.binding import _DetectCfg
    cfg = _DetectCfg()
    lib.qarvd_default_detect_cfg(C.byref(cfg))
    assert (cfg.tau, cfg.alpha, cfg.align, cfg.clip_search, cfg.forced_mask) == (3.5, 1.2, 32, 0, None)
    assert lib.qarvd_status_string(0) == b"QARVD_OK"
    assert lib.qarvd_status_string(-2) == b"QARVD_ERR_UNSUPPORTED"
    assert lib.qarvd_gemm_num_variants() >= 1
    assert lib.qarvd_gemm_variant_name(1) != b"" and lib.qarvd_gemm_variant_name(0) == b""


def test_bad_arguments_are_rejected_on_the_host(lib):
    p = C.c_void_p(0x1000)          # never dereferenced: validation fails first
    null = None
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    qa = lib.qarvd_quant_act
    assert qa(null, 0, 4, 128, 128, null, 0, p, 128, p, null) == INVALID
    assert qa(p, 0, 0, 128, 128, null, 0, p, 128, p, null) == INVALID          # M = 0
    assert qa(p, 0, 4, 128, 100, null, 0, p, 128, p, null) == INVALID          # ldx < K
    assert qa(p, 0, 4, 128, 128, null, 32, p, 128, p, null) == INVALID         # K_o without perm
    assert qa(p, 0, 4, 128, 128, p, 129, p, 256, p, null) == INVALID           # K_o > K
    assert qa(p, 0, 4, 200, 200, null, 0, p, 200, p, null) == INVALID          # ldxq < packed extent
    assert qa(p, 7, 4, 128, 128, null, 0, p, 128, p, null) == UNSUPPORTED      # dtype
    assert qa(p, 0, 4, 128, 128, null, 0, C.c_void_p(0x1004), 128, p, null) == UNSUPPORTED
    assert qa(p, 0, 4, 133144, 133144, null, 0, p, 133248, p, null) == INVALID  # accumulator could overflow
    assert lib.qarvd_quant_act_static(p, 0, 4, 128, 128, null, 0, C.c_float(-1.0), p, 128, null) == INVALID

    gm = lib.qarvd_w8a8_dual_gemm
    ok_args = [p, 128, p, p, 128, p, p, null, 4, 4, 128, 0, p, 1, 4, null, null, null]

    def gemm_with(i, v):
        a = list(ok_args)
        a[i] = v
        return gm(*a)

    assert gemm_with(0, null) == INVALID
    assert gemm_with(8, 0) == INVALID               # M
    assert gemm_with(11, 129) == INVALID            # K_o > K
    assert gemm_with(1, 64) == INVALID              # ldxq < packed extent
    assert gemm_with(14, 3) == INVALID              # ldy < N
    assert gemm_with(13, 9) == UNSUPPORTED          # dtype
    assert gemm_with(1, 136) == UNSUPPORTED         # stride not a multiple of 16
    assert gemm_with(3, C.c_void_p(0x1001)) == UNSUPPORTED
    assert lib.qarvd_w8a8_dual_gemm_variant(999, *ok_args) == INVALID

    qw = lib.qarvd_quantize_weight
    ko = C.c_int32(0)
    assert qw(null, 4, 128, 128, None, p, 128, p, p, p, C.byref(ko), null, p, 1 << 20, null) == INVALID
    assert qw(p, 4, 128, 64, None, p, 128, p, p, p, C.byref(ko), null, p, 1 << 20, null) == INVALID     # ldw < K
    assert qw(p, 4, 130, 130, None, p, 144, p, p, p, C.byref(ko), null, p, 1 << 20, null) == INVALID    # ldwq too small
    assert qw(p, 4, 128, 128, None, p, 128, p, p, p, C.byref(ko), null, null, 1 << 20, null) == WORKSPACE
    assert qw(p, 4, 128, 128, None, p, 128, p, p, p, C.byref(ko), null, p, 16, null) == WORKSPACE
    assert qw(p, 4, 128, 128, None, p, 128, p, p, p, C.byref(ko), null, C.c_void_p(0x1010), 1 << 20, null) == WORKSPACE


def test_bad_arguments_of_the_widened_entry_points(lib):
    from paper_2605_21072_amd.binding import _DetectCfg
    p = C.c_void_p(0x1000)          # never dereferenced: validation fails first
    null = None
    INVALID, UNSUPPORTED = -1, -2
    f = C.c_float
    # chained-layer GEMM: Xq, ldxq, s_x, Wq, ldwq, s_n, s_o, bias, M, N, K, K_o, act, out_scale, Y8, ldy8, variant, stream
    q8 = lib.qarvd_w8a8_dual_gemm_q8
    ok = [p, 128, p, p, 128, p, p, null, 4, 16, 128, 0, 0, f(0.1), p, 16, 0, null]

    def q8_with(i, v):
        a = list(ok)
        a[i] = v
        return q8(*a)

    assert q8_with(14, null) == INVALID                       # no output
    assert q8_with(12, 5) == INVALID                          # unknown activation
    for bad in (0.0, -1.0, float("nan"), float("inf"), 1e-38):
        assert q8_with(13, f(bad)) == INVALID
    assert q8_with(15, 8) == INVALID                          # ldy8 < N
    assert q8_with(16, 99) == INVALID                         # unknown variant
    assert q8_with(9, 24) == INVALID                          # N = 24 > ldy8 = 16
    a = list(ok)
    a[9], a[15] = 24, 32
    assert q8(*a) == UNSUPPORTED                              # N not a multiple of 16
    assert q8_with(14, C.c_void_p(0x1008)) == UNSUPPORTED     # output not 16-byte aligned
    # INT4 GEMM: ldwq4 is in bytes, at least half the packed extent
    w4 = lib.qarvd_w4a8_dual_gemm
    ok4 = [p, 128, p, p, 64, p, p, null, 4, 8, 128, 0, p, 1, 8, null, null, 0, null]
    a = list(ok4)
    a[4] = 32
    assert w4(*a) == INVALID
    a = list(ok4)
    a[17] = 9
    assert w4(*a) == INVALID
    a = list(ok4)
    a[9], a[14], a[17] = 12, 12, 1
    assert w4(*a) == UNSUPPORTED                              # N % 8 != 0: not for the LDS-direct tile asked for
    # percentile-clip search: flag values and its K limit
    ko = C.c_int32(0)
    cfg = _DetectCfg()
    lib.qarvd_default_detect_cfg(C.byref(cfg))
    cfg.clip_search = 2
    qw = lib.qarvd_quantize_weight
    assert qw(p, 4, 128, 128, C.byref(cfg), p, 128, p, p, p, C.byref(ko), null, p, 1 << 20, null) == INVALID
    cfg.clip_search = 1
    assert qw(p, 4, 16512, 16512, C.byref(cfg), p, 16512, p, p, p, C.byref(ko), null, p, 1 << 30, null) == UNSUPPORTED
    assert lib.qarvd_q8_gemm_num_variants() >= 1 and lib.qarvd_w4_gemm_num_variants() >= 1


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    import paper_2605_21072_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", tmp_path / "libqarvd.so")
    with pytest.raises(FileNotFoundError):
        b.load_library()
