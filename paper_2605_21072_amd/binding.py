"""ctypes binding of the C ABI declared in ``include/qarvd.h``.

Argument marshalling only: every step of the path runs in the HIP kernels of ``libqarvd.so``.
There is no CPU or PyTorch fallback; a missing library raises at first use.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from pathlib import Path
from typing import Optional

import torch

_PKG = Path(__file__).resolve().parent
_LIB_PATH = _PKG / "libqarvd.so"
_lib = None

QARVD_F32, QARVD_BF16 = 0, 1
_STATUS = {0: "QARVD_OK", -1: "QARVD_ERR_INVALID_ARG", -2: "QARVD_ERR_UNSUPPORTED",
           -3: "QARVD_ERR_WORKSPACE", -4: "QARVD_ERR_HIP"}


class QarvdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s returned %s (%d)" % (where, _STATUS.get(status, "?"), status))


class _DetectCfg(C.Structure):
    _fields_ = [("tau", C.c_double), ("alpha", C.c_double), ("align", C.c_int32), ("clip_search", C.c_int32),
                ("forced_mask", C.c_void_p)]


def lib_path() -> Path:
    return _LIB_PATH


def load_library():
    """Load libqarvd.so (built in-tree by ``paper_2605_21072_amd.build``).  Fails loudly."""
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise FileNotFoundError(
            "%s is missing: run `python -m paper_2605_21072_amd.build` (or __graft_entry__.build()) "
            "first; there is no fallback path" % _LIB_PATH)
    lib = C.CDLL(str(_LIB_PATH))
    i32, i64, vp, f32 = C.c_int32, C.c_int64, C.c_void_p, C.c_float
    lib.qarvd_default_detect_cfg.argtypes = [C.POINTER(_DetectCfg)]
    lib.qarvd_default_detect_cfg.restype = None
    lib.qarvd_status_string.argtypes = [C.c_int]
    lib.qarvd_status_string.restype = C.c_char_p
    lib.qarvd_packed_normal_offset.argtypes = [i32]
    lib.qarvd_packed_normal_offset.restype = i32
    lib.qarvd_packed_k.argtypes = [i32, i32]
    lib.qarvd_packed_k.restype = i32
    lib.qarvd_packed_ld.argtypes = [i32, i32]
    lib.qarvd_packed_ld.restype = i32
    lib.qarvd_quantize_weight_workspace.argtypes = [i32, i32]
    lib.qarvd_quantize_weight_workspace.restype = C.c_size_t
    lib.qarvd_quantize_weight.argtypes = [vp, i32, i32, i64, C.POINTER(_DetectCfg), vp, i64, vp, vp, vp,
                                          C.POINTER(i32), vp, vp, C.c_size_t, vp]
    lib.qarvd_quantize_weight.restype = C.c_int
    lib.qarvd_quantize_weight_static.argtypes = [vp, i32, i32, i64, C.POINTER(_DetectCfg), vp, i64, vp, vp, vp,
                                                 C.POINTER(i32), vp, vp]
    lib.qarvd_quantize_weight_static.restype = C.c_int
    lib.qarvd_quantize_weight_static_max_k.argtypes = []
    lib.qarvd_quantize_weight_static_max_k.restype = i32
    lib.qarvd_quant_act.argtypes = [vp, C.c_int, i32, i32, i64, vp, i32, vp, i64, vp, vp]
    lib.qarvd_quant_act.restype = C.c_int
    lib.qarvd_quant_act_static.argtypes = [vp, C.c_int, i32, i32, i64, vp, i32, f32, vp, i64, vp]
    lib.qarvd_quant_act_static.restype = C.c_int
    gemm_args = [vp, i64, vp, vp, i64, vp, vp, vp, i32, i32, i32, i32, vp, C.c_int, i64, vp, vp, vp]
    lib.qarvd_w8a8_dual_gemm.argtypes = gemm_args
    lib.qarvd_w8a8_dual_gemm.restype = C.c_int
    lib.qarvd_w8a8_dual_gemm_variant.argtypes = [i32] + gemm_args
    lib.qarvd_w8a8_dual_gemm_variant.restype = C.c_int
    lib.qarvd_quantize_weight_w4_workspace.argtypes = [i32, i32]
    lib.qarvd_quantize_weight_w4_workspace.restype = C.c_size_t
    lib.qarvd_quantize_weight_w4.argtypes = lib.qarvd_quantize_weight.argtypes
    lib.qarvd_quantize_weight_w4.restype = C.c_int
    lib.qarvd_w4a8_dual_gemm.argtypes = gemm_args[:-1] + [i32, C.c_void_p]
    lib.qarvd_w4a8_dual_gemm.restype = C.c_int
    lib.qarvd_w4_gemm_num_variants.argtypes = []
    lib.qarvd_w4_gemm_num_variants.restype = i32
    lib.qarvd_w8a8_dual_gemm_q8.argtypes = [vp, i64, vp, vp, i64, vp, vp, vp, i32, i32, i32, i32, C.c_int, f32, vp, i64,
                                            i32, vp]
    lib.qarvd_w8a8_dual_gemm_q8.restype = C.c_int
    lib.qarvd_q8_gemm_num_variants.argtypes = []
    lib.qarvd_q8_gemm_num_variants.restype = i32
    lib.qarvd_gemm_num_variants.argtypes = []
    lib.qarvd_gemm_num_variants.restype = i32
    lib.qarvd_gemm_variant_name.argtypes = [i32]
    lib.qarvd_gemm_variant_name.restype = C.c_char_p
    lib.qarvd_probe_mfma_peak.argtypes = [i32, vp, C.c_size_t, C.POINTER(C.c_double), vp]
    lib.qarvd_probe_mfma_peak.restype = C.c_int
    _lib = lib
    return lib


def _check(status: int, where: str):
    if status != 0:
        raise QarvdError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return QARVD_F32
    if t.dtype == torch.bfloat16:
        return QARVD_BF16
    raise TypeError("expected float32 or bfloat16, got %s" % t.dtype)


def _dev2d(t: torch.Tensor, what: str):
    if not t.is_cuda or t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("%s must be a 2-D device tensor with unit inner stride" % what)


def packed_normal_offset(K_o: int) -> int:
    return int(load_library().qarvd_packed_normal_offset(K_o))


def packed_k(K: int, K_o: int = -1) -> int:
    return int(load_library().qarvd_packed_k(K, K_o))


def packed_ld(K: int, K_o: int = -1) -> int:
    """qarvd_packed_ld: the recommended row stride of packed INT8 operands (packed extent + 128 bytes)."""
    return int(load_library().qarvd_packed_ld(K, K_o))


def quantize_weight_workspace(N: int, K: int) -> int:
    return int(load_library().qarvd_quantize_weight_workspace(N, K))


def gemm_num_variants() -> int:
    return int(load_library().qarvd_gemm_num_variants())


def gemm_variant_name(i: int) -> str:
    return load_library().qarvd_gemm_variant_name(i).decode()


def probe_mfma_peak(iters: int = 20000, stream=None) -> float:
    """qarvd_probe_mfma_peak: measured issue-bound INT8 MFMA rate of the current device in TOPS."""
    lib = load_library()
    ws = torch.empty(8192, dtype=torch.uint8, device="cuda")
    tops = C.c_double(0.0)
    _check(lib.qarvd_probe_mfma_peak(int(iters), _ptr(ws), ws.numel(), C.byref(tops), _stream(stream)), "qarvd_probe_mfma_peak")
    return float(tops.value)


@dataclass
class DualScaleWeight:
    """Packed dual-scale layer: the buffers qarvd_quantize_weight fills (all device tensors)."""
    Wq: torch.Tensor          # int8 [N, ldwq] packed
    s_normal: torch.Tensor    # f32 [N]
    s_outlier: torch.Tensor   # f32 [N]
    perm: torch.Tensor        # int32 [K]
    K_o: int
    N: int
    K: int
    v: Optional[torch.Tensor] = None   # f32 [K] column norms
    bits: int = 8                      # 4: Wq is uint8 [N, ldwq4], two INT4 codes per byte (see qarvd.h)

    @property
    def kp(self) -> int:
        return packed_k(self.K, self.K_o)

    @property
    def n_off(self) -> int:
        return packed_normal_offset(self.K_o)

    def codes(self) -> torch.Tensor:
        """int8 [N, kp]: one code per packed position (the INT4 layout unpacked; marshalling only)."""
        if self.bits == 8:
            return self.Wq[:, :self.kp]
        b = self.Wq[:, :self.kp // 2].to(torch.int16).reshape(self.N, -1, 8)       # groups of 16 positions
        lo = ((b & 0xF) ^ 8) - 8
        hi = (((b >> 4) & 0xF) ^ 8) - 8
        g = torch.stack([lo[:, :, 0:4], hi[:, :, 0:4], lo[:, :, 4:8], hi[:, :, 4:8]], dim=2)   # [N, G, 4, 4]
        return g.reshape(self.N, -1).to(torch.int8)

    def logical_Wq(self) -> torch.Tensor:
        """int8 [N, K] in packed channel order without the zero padding."""
        c = self.codes()
        return torch.cat([c[:, :self.K_o], c[:, self.n_off:self.n_off + self.K - self.K_o]], dim=1)


def quantize_weight(W: torch.Tensor, tau: float = 3.5, alpha: float = 1.2, align: int = 32,
                    forced_mask=None, ldwq: Optional[int] = None, want_norms: bool = True,
                    stream=None, bits: int = 8, clip_search: bool = False) -> DualScaleWeight:
    """qarvd_quantize_weight (bits=8) / qarvd_quantize_weight_w4 (bits=4): W f32 [N,K] on the device ->
    packed dual-scale layer.  For bits=4 `ldwq` is in bytes (two codes per byte).  clip_search: scales from
    the percentile-clip search instead of the block absmax."""
    lib = load_library()
    _dev2d(W, "W")
    if W.dtype != torch.float32:
        raise TypeError("W must be float32")
    N, K = W.shape
    dev = W.device
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    if ldwq is None:
        ldwq = packed_ld(K, -1) if (forced_mask is not None or align % 32) else (K + 127) // 128 * 128 + 128
        if bits == 4:
            ldwq //= 2
    Wq = torch.empty((N, ldwq), dtype=torch.int8 if bits == 8 else torch.uint8, device=dev)
    sn = torch.empty(N, dtype=torch.float32, device=dev)
    so = torch.empty(N, dtype=torch.float32, device=dev)
    perm = torch.empty(K, dtype=torch.int32, device=dev)
    v = torch.empty(K, dtype=torch.float32, device=dev) if want_norms else None
    ws_bytes = quantize_weight_workspace(N, K) if bits == 8 else int(lib.qarvd_quantize_weight_w4_workspace(N, K))
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=dev)
    ws_ptr = (ws.data_ptr() + 255) // 256 * 256
    cfg = _DetectCfg(float(tau), float(alpha), int(align), int(bool(clip_search)), None)
    keep = None
    if forced_mask is not None:
        import numpy as np
        keep = np.ascontiguousarray(np.asarray(forced_mask, dtype=np.uint8))
        if keep.shape != (K,):
            raise ValueError("forced_mask must have K entries")
        cfg.forced_mask = keep.ctypes.data
    ko = C.c_int32(-1)
    fn = lib.qarvd_quantize_weight if bits == 8 else lib.qarvd_quantize_weight_w4
    st = fn(_ptr(W), N, K, W.stride(0), C.byref(cfg), _ptr(Wq), ldwq, _ptr(sn), _ptr(so),
            _ptr(perm), C.byref(ko), _ptr(v), C.c_void_p(ws_ptr), ws_bytes, _stream(stream))
    _check(st, "qarvd_quantize_weight" if bits == 8 else "qarvd_quantize_weight_w4")
    del keep
    return DualScaleWeight(Wq, sn, so, perm, int(ko.value), N, K, v, bits)


def quantize_weight_static_max_k() -> int:
    return int(load_library().qarvd_quantize_weight_static_max_k())


def quantize_weight_static(W: torch.Tensor, out: DualScaleWeight, tau: float = 3.5, alpha: float = 1.2,
                           align: int = 32, stream=None) -> DualScaleWeight:
    """qarvd_quantize_weight_static: the offline step into the caller's buffers (`out`: Wq, s_normal,
    s_outlier, perm and optionally v, already allocated) with the library's fixed device array as the
    workspace; nothing is allocated by this call.  Sets out.K_o and returns `out`."""
    lib = load_library()
    _dev2d(W, "W")
    if W.dtype != torch.float32:
        raise TypeError("W must be float32")
    N, K = W.shape
    cfg = _DetectCfg(float(tau), float(alpha), int(align), 0, None)
    ko = C.c_int32(-1)
    st = lib.qarvd_quantize_weight_static(_ptr(W), N, K, W.stride(0), C.byref(cfg), _ptr(out.Wq), out.Wq.stride(0),
                                          _ptr(out.s_normal), _ptr(out.s_outlier), _ptr(out.perm), C.byref(ko),
                                          _ptr(out.v), _stream(stream))
    _check(st, "qarvd_quantize_weight_static")
    out.K_o, out.N, out.K = int(ko.value), N, K
    return out


def quant_act(X: torch.Tensor, perm: Optional[torch.Tensor], K_o: int, Xq: Optional[torch.Tensor] = None,
              s_x: Optional[torch.Tensor] = None, stream=None):
    """qarvd_quant_act: X [M,K] f32/bf16 -> (Xq int8 [M, ld] packed for (K, K_o), s_x f32 [M])."""
    lib = load_library()
    _dev2d(X, "X")
    M, K = X.shape
    if Xq is None:
        Xq = torch.empty((M, packed_ld(K, K_o)), dtype=torch.int8, device=X.device)   # row stride: see qarvd_packed_ld
    if s_x is None:
        s_x = torch.empty(M, dtype=torch.float32, device=X.device)
    st = lib.qarvd_quant_act(_ptr(X), _dt(X), M, K, X.stride(0), _ptr(perm), K_o, _ptr(Xq), Xq.stride(0), _ptr(s_x),
                             _stream(stream))
    _check(st, "qarvd_quant_act")
    return Xq, s_x


def quant_act_static(X: torch.Tensor, perm: Optional[torch.Tensor], K_o: int, scale: float,
                     Xq: Optional[torch.Tensor] = None, stream=None):
    """qarvd_quant_act_static: same packing with a given per-tensor scale."""
    lib = load_library()
    _dev2d(X, "X")
    M, K = X.shape
    if Xq is None:
        Xq = torch.empty((M, packed_ld(K, K_o)), dtype=torch.int8, device=X.device)
    st = lib.qarvd_quant_act_static(_ptr(X), _dt(X), M, K, X.stride(0), _ptr(perm), K_o, C.c_float(scale), _ptr(Xq),
                                    Xq.stride(0), _stream(stream))
    _check(st, "qarvd_quant_act_static")
    return Xq


def w8a8_dual_gemm(Xq: torch.Tensor, s_x: torch.Tensor, w: DualScaleWeight, bias: Optional[torch.Tensor], M: int,
                   out_dtype=torch.bfloat16, Y: Optional[torch.Tensor] = None, debug_acc: bool = False,
                   variant: int = 0, stream=None):
    """qarvd_w8a8_dual_gemm (or qarvd_w4a8_dual_gemm when `w` holds INT4 codes).  Returns Y, or
    (Y, acc_normal, acc_outlier) with debug_acc."""
    lib = load_library()
    if Y is None:
        Y = torch.empty((M, w.N), dtype=out_dtype, device=Xq.device)
    an = ao = None
    if debug_acc:
        an = torch.empty((M, w.N), dtype=torch.int32, device=Xq.device)
        ao = torch.empty((M, w.N), dtype=torch.int32, device=Xq.device)
    if w.bits == 4:
        st = lib.qarvd_w4a8_dual_gemm(_ptr(Xq), Xq.stride(0), _ptr(s_x), _ptr(w.Wq), w.Wq.stride(0),
                                      _ptr(w.s_normal), _ptr(w.s_outlier), _ptr(bias), M, w.N, w.K, w.K_o,
                                      _ptr(Y), _dt(Y), Y.stride(0), _ptr(an), _ptr(ao), variant, _stream(stream))
        _check(st, "qarvd_w4a8_dual_gemm")
        return (Y, an, ao) if debug_acc else Y
    st = lib.qarvd_w8a8_dual_gemm_variant(variant, _ptr(Xq), Xq.stride(0), _ptr(s_x), _ptr(w.Wq), w.Wq.stride(0),
                                          _ptr(w.s_normal), _ptr(w.s_outlier), _ptr(bias), M, w.N, w.K, w.K_o,
                                          _ptr(Y), _dt(Y), Y.stride(0), _ptr(an), _ptr(ao), _stream(stream))
    _check(st, "qarvd_w8a8_dual_gemm")
    return (Y, an, ao) if debug_acc else Y


ACT_NONE, ACT_GELU_TANH = 0, 1


def q8_gemm_num_variants() -> int:
    return int(load_library().qarvd_q8_gemm_num_variants())


def w8a8_dual_gemm_q8(Xq: torch.Tensor, s_x: torch.Tensor, w: DualScaleWeight, bias: Optional[torch.Tensor], M: int,
                      out_scale: float, act: int = ACT_NONE, Y8: Optional[torch.Tensor] = None, variant: int = 0,
                      stream=None) -> torch.Tensor:
    """qarvd_w8a8_dual_gemm_q8: the dual GEMM with activation and the next layer's static-scale
    quantization in its epilogue.  Returns Y8 int8 [M, >= N]."""
    lib = load_library()
    if w.bits != 8:
        raise ValueError("the chained epilogue takes INT8 weights")
    if Y8 is None:
        Y8 = torch.empty((M, w.N), dtype=torch.int8, device=Xq.device)
    st = lib.qarvd_w8a8_dual_gemm_q8(_ptr(Xq), Xq.stride(0), _ptr(s_x), _ptr(w.Wq), w.Wq.stride(0), _ptr(w.s_normal),
                                     _ptr(w.s_outlier), _ptr(bias), M, w.N, w.K, w.K_o, int(act), C.c_float(out_scale),
                                     _ptr(Y8), Y8.stride(0), variant, _stream(stream))
    _check(st, "qarvd_w8a8_dual_gemm_q8")
    return Y8


def packed_channel_map(w: DualScaleWeight) -> torch.Tensor:
    """int64 [kp]: the input channel each packed position of `w` holds, -1 at pad positions.  A producing
    layer whose weight rows are gathered with this map (zero rows at -1) emits `w`'s Xq directly."""
    m = torch.full((w.kp,), -1, dtype=torch.int64, device=w.perm.device)
    p = w.perm.to(torch.int64)
    m[:w.K_o] = p[:w.K_o]
    m[w.n_off:w.n_off + w.K - w.K_o] = p[w.K_o:]
    return m


def w8a8_linear(X: torch.Tensor, w: DualScaleWeight, bias: Optional[torch.Tensor], out_dtype=torch.bfloat16,
                stream=None) -> torch.Tensor:
    """The online pair: quant_act followed by the dual GEMM."""
    Xq, s_x = quant_act(X, w.perm if w.K_o > 0 else None, w.K_o, stream=stream)
    return w8a8_dual_gemm(Xq, s_x, w, bias, X.shape[0], out_dtype, stream=stream)
