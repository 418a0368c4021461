"""ctypes front end of the CPU oracle (``qarvd_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  Nothing in the product
package imports it, and it imports nothing from the product package.

All arrays are host numpy arrays, row-major, unpadded.  See the header of
``qarvd_oracle.c`` for the definitions and the paper passages they follow.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "qarvd_oracle.c"
_LIB = _HERE / "liboracle.so"
_lib = None

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-fPIC", "-shared", "-fopenmp",
          "-Wall", "-Wextra"]


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (about a second)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.run(["gcc", *CFLAGS, str(_SRC), "-o", str(tmp), "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(str(_LIB))
    return _lib


def num_threads() -> int:
    """Threads the OpenMP row loops will use (OMP_NUM_THREADS or the core count)."""
    omp = C.CDLL("libgomp.so.1")
    omp.omp_get_max_threads.restype = C.c_int
    return int(omp.omp_get_max_threads())


def set_num_threads(n: int) -> None:
    omp = C.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(C.c_int(int(n)))


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _check(rc):
    if rc != 0:
        raise ValueError("oracle returned %d" % rc)


def column_norms(W):
    W = _f32(W)
    N, K = W.shape
    v = np.empty(K, np.float32)
    _check(_load().oracle_column_norms(_p(W, C.c_float), N, K, _p(v, C.c_float)))
    return v


def detect(v, tau=3.5, alpha=1.2):
    """Returns (flag uint8[K], dict(med, mad, T, n_det))."""
    v = _f32(v)
    K = v.shape[0]
    flag = np.empty(K, np.uint8)
    st = np.empty(4, np.float64)
    _check(_load().oracle_detect(_p(v, C.c_float), K, C.c_double(tau), C.c_double(alpha),
                                 _p(flag, C.c_uint8), _p(st, C.c_double)))
    return flag, dict(med=st[0], mad=st[1], T=st[2], n_det=int(st[3]))


def align(v, sel, align=32):
    """Grow the selected set to a multiple of ``align``; returns (sel, K_o)."""
    v = _f32(v)
    sel = np.array(sel, dtype=np.uint8, copy=True)
    ko = C.c_int(0)
    _check(_load().oracle_align(_p(v, C.c_float), v.shape[0], int(align), _p(sel, C.c_uint8),
                                C.byref(ko)))
    return sel, ko.value


def build_perm(sel):
    sel = np.ascontiguousarray(sel, dtype=np.uint8)
    perm = np.empty(sel.shape[0], np.int32)
    ko = C.c_int(0)
    _check(_load().oracle_build_perm(_p(sel, C.c_uint8), sel.shape[0], _p(perm, C.c_int32),
                                     C.byref(ko)))
    return perm, ko.value


def quantize_rows(W, perm, K_o):
    W = _f32(W)
    N, K = W.shape
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    Wq = np.empty((N, K), np.int8)
    sn = np.empty(N, np.float32)
    so = np.empty(N, np.float32)
    _check(_load().oracle_quantize_rows(_p(W, C.c_float), N, K, _p(perm, C.c_int32), int(K_o),
                                        _p(Wq, C.c_int8), _p(sn, C.c_float), _p(so, C.c_float)))
    return Wq, sn, so


def clip_search(w, qmax=127.0):
    """Percentile-clip scale of one block (Sec. 4.1): returns dict(s, choice, clip[3], sse[3])."""
    w = np.ascontiguousarray(w, dtype=np.float32).ravel()
    s = C.c_float(0.0)
    ch = C.c_int(0)
    clip = np.zeros(3, np.float32)
    sse = np.zeros(3, np.float64)
    _check(_load().oracle_clip_search(_p(w, C.c_float), int(w.size), C.c_float(qmax), C.byref(s), C.byref(ch),
                                      _p(clip, C.c_float), _p(sse, C.c_double)))
    return dict(s=np.float32(s.value), choice=int(ch.value), clip=clip, sse=sse)


def quantize_rows_clip(W, perm, K_o, bits=8):
    """quantize_rows with percentile-clip scales.  Returns (Wq, s_normal, s_outlier, choice_n, choice_o)."""
    W = _f32(W)
    N, K = W.shape
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    Wq = np.empty((N, K), np.int8)
    sn = np.empty(N, np.float32)
    so = np.empty(N, np.float32)
    cn = np.empty(N, np.int8)
    co = np.empty(N, np.int8)
    _check(_load().oracle_quantize_rows_clip(_p(W, C.c_float), N, K, _p(perm, C.c_int32), int(K_o), int(bits),
                                             _p(Wq, C.c_int8), _p(sn, C.c_float), _p(so, C.c_float),
                                             _p(cn, C.c_int8), _p(co, C.c_int8)))
    return Wq, sn, so, cn, co


def quantize_weight(W, tau=3.5, alpha=1.2, align=32, forced_mask=None, bits=8, clip_search=False):
    """Returns dict(Wq, s_normal, s_outlier, perm, K_o, v, flag, stats).  bits=4: codes in [-7, 7]
    (one per int8 element), scales = block absmax / 7 (the W4A8 setting of Sec. 4.2).  clip_search:
    scales from the percentile-clip search of Sec. 4.1 instead of the block absmax."""
    W = _f32(W)
    N, K = W.shape
    Wq = np.empty((N, K), np.int8)
    sn = np.empty(N, np.float32)
    so = np.empty(N, np.float32)
    perm = np.empty(K, np.int32)
    v = np.empty(K, np.float32)
    flag = np.empty(K, np.uint8)
    st = np.zeros(4, np.float64)
    ko = C.c_int32(0)
    fm = None if forced_mask is None else np.ascontiguousarray(forced_mask, dtype=np.uint8)
    _check(_load().oracle_quantize_weight_clip(
        _p(W, C.c_float), N, K, C.c_double(tau), C.c_double(alpha), int(align), _p(fm, C.c_uint8), int(bits),
        int(bool(clip_search)), _p(Wq, C.c_int8), _p(sn, C.c_float), _p(so, C.c_float), _p(perm, C.c_int32), C.byref(ko),
        _p(v, C.c_float), _p(flag, C.c_uint8), _p(st, C.c_double)))
    return dict(Wq=Wq, s_normal=sn, s_outlier=so, perm=perm, K_o=int(ko.value), v=v, flag=flag,
                stats=dict(med=st[0], mad=st[1], T=st[2], n_det=int(st[3])))


def quant_act(X, perm=None):
    """Per-token dynamic INT8.  Returns (Xq int8[M,K], s_x f32[M])."""
    X = _f32(X)
    M, K = X.shape
    pm = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    Xq = np.empty((M, K), np.int8)
    sx = np.empty(M, np.float32)
    _check(_load().oracle_quant_act(_p(X, C.c_float), M, K, _p(pm, C.c_int32), _p(Xq, C.c_int8),
                                    _p(sx, C.c_float)))
    return Xq, sx


def quant_act_static(X, s, perm=None):
    X = _f32(X)
    M, K = X.shape
    pm = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    Xq = np.empty((M, K), np.int8)
    _check(_load().oracle_quant_act_static(_p(X, C.c_float), M, K, _p(pm, C.c_int32),
                                           C.c_float(float(s)), _p(Xq, C.c_int8)))
    return Xq


def dual_gemm(Xq, s_x, Wq, s_normal, s_outlier, bias, K_o, want_acc=True, want_f32=True,
              want_bf16=True):
    """Returns dict(Y_f32, Y_bf16 (uint16 bit patterns), acc_n, acc_o)."""
    Xq = np.ascontiguousarray(Xq, dtype=np.int8)
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    M, K = Xq.shape
    N = Wq.shape[0]
    assert Wq.shape[1] == K
    s_x = _f32(s_x)
    sn = _f32(s_normal)
    so = _f32(s_outlier)
    b = None if bias is None else _f32(bias)
    Yf = np.empty((M, N), np.float32) if want_f32 else None
    Yb = np.empty((M, N), np.uint16) if want_bf16 else None
    an = np.empty((M, N), np.int32) if want_acc else None
    ao = np.empty((M, N), np.int32) if want_acc else None
    _check(_load().oracle_dual_gemm(
        _p(Xq, C.c_int8), _p(s_x, C.c_float), _p(Wq, C.c_int8), _p(sn, C.c_float),
        _p(so, C.c_float), _p(b, C.c_float), M, N, K, int(K_o), _p(Yf, C.c_float),
        _p(Yb, C.c_uint16), _p(an, C.c_int32), _p(ao, C.c_int32)))
    return dict(Y_f32=Yf, Y_bf16=Yb, acc_n=an, acc_o=ao)


def single_scale_linear(X, W, bias):
    """Independent single-scale W8A8 linear.  Returns dict(Y_f32, Y_bf16, acc, s_w, s_x)."""
    X = _f32(X)
    W = _f32(W)
    M, K = X.shape
    N = W.shape[0]
    b = None if bias is None else _f32(bias)
    Yf = np.empty((M, N), np.float32)
    Yb = np.empty((M, N), np.uint16)
    acc = np.empty((M, N), np.int32)
    sw = np.empty(N, np.float32)
    sx = np.empty(M, np.float32)
    _check(_load().oracle_single_scale_linear(
        _p(X, C.c_float), _p(W, C.c_float), _p(b, C.c_float), M, N, K, _p(Yf, C.c_float),
        _p(Yb, C.c_uint16), _p(acc, C.c_int32), _p(sw, C.c_float), _p(sx, C.c_float)))
    return dict(Y_f32=Yf, Y_bf16=Yb, acc=acc, s_w=sw, s_x=sx)


def linear(X, W, bias, tau=3.5, alpha=1.2, align=32, forced_mask=None):
    """quantize_weight -> quant_act -> dual_gemm in one call (all oracle)."""
    qw = quantize_weight(W, tau, alpha, align, forced_mask)
    Xq, sx = quant_act(X, qw["perm"])
    out = dual_gemm(Xq, sx, qw["Wq"], qw["s_normal"], qw["s_outlier"], bias, qw["K_o"])
    out.update(qw)
    out.update(Xq=Xq, s_x=sx)
    return out


def gelu_tanh(x):
    """Element-wise oracle_gelu_tanh on an fp32 array."""
    x = _f32(x)
    lib = _load()
    lib.oracle_gelu_tanh.restype = C.c_float
    lib.oracle_gelu_tanh.argtypes = [C.c_float]
    return np.array([lib.oracle_gelu_tanh(float(v)) for v in x.ravel()], np.float32).reshape(x.shape)


def dual_gemm_q8(Xq, s_x, Wq, s_normal, s_outlier, bias, K_o, s_out, act=0, want_act=False):
    """Dual GEMM whose epilogue quantizes for the next layer.  Returns int8 [M, N]; with want_act also
    the fp32 value each code was rounded from (after the activation)."""
    Xq = np.ascontiguousarray(Xq, dtype=np.int8)
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    M, K = Xq.shape
    N = Wq.shape[0]
    b = None if bias is None else _f32(bias)
    Y8 = np.empty((M, N), np.int8)
    A = np.empty((M, N), np.float32) if want_act else None
    _check(_load().oracle_dual_gemm_q8(_p(Xq, C.c_int8), _p(_f32(s_x), C.c_float), _p(Wq, C.c_int8),
                                       _p(_f32(s_normal), C.c_float), _p(_f32(s_outlier), C.c_float),
                                       _p(b, C.c_float), M, N, K, int(K_o), int(act), C.c_float(float(s_out)),
                                       _p(Y8, C.c_int8), _p(A, C.c_float)))
    return (Y8, A) if want_act else Y8
