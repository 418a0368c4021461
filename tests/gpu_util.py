"""Helpers of the GPU parity tests: run the HIP library through its C ABI binding and bring the
results back as numpy arrays in the oracle's logical (unpadded) layout."""
import numpy as np
import torch

import paper_2605_21072_amd as q


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def logical(packed: torch.Tensor, K: int, K_o: int):
    """Strip the zero padding of a packed [rows, ld] INT8 tensor; also checks the padding is zero."""
    n_off = q.packed_normal_offset(K_o)
    kp = q.packed_k(K, K_o)
    p = packed.cpu().numpy()
    assert np.all(p[:, K_o:n_off] == 0), "outlier-block padding not zero"
    assert np.all(p[:, n_off + K - K_o:kp] == 0), "tail padding not zero"
    return np.concatenate([p[:, :K_o], p[:, n_off:n_off + K - K_o]], axis=1)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in bf16 units of last place between two arrays of bf16 bit patterns."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def gpu_quantize_weight(W, **kw):
    w = q.quantize_weight(dev(W), **kw)
    torch.cuda.synchronize()
    return w


def weight_to_numpy(w):
    return dict(Wq=logical(w.Wq, w.K, w.K_o), s_normal=w.s_normal.cpu().numpy(), s_outlier=w.s_outlier.cpu().numpy(),
                perm=w.perm.cpu().numpy(), K_o=w.K_o, v=None if w.v is None else w.v.cpu().numpy())


def assert_weight_equal(g, o):
    """g: weight_to_numpy(...) of the GPU result, o: oracle.quantize_weight(...) dict.  Bit-exact."""
    assert g["K_o"] == o["K_o"]
    assert np.array_equal(g["perm"], o["perm"])
    if g["v"] is not None:
        assert np.array_equal(g["v"].view(np.uint32), o["v"].view(np.uint32))
    assert np.array_equal(g["s_normal"].view(np.uint32), o["s_normal"].view(np.uint32))
    assert np.array_equal(g["s_outlier"].view(np.uint32), o["s_outlier"].view(np.uint32))
    assert np.array_equal(g["Wq"], o["Wq"])


def assert_q8_codes(got, ref, a, s_out, act):
    """Parity rule of the chained epilogue's INT8 codes.  Without an activation the code is a function of
    the (bit-exact) fp32 result alone: equal.  With GELU the oracle rounds the double-precision definition
    once, the kernel evaluates the same function in fp32 by its own operation sequence (within
    2e-7 + 1.1e-6 |a| of the definition), so the codes must be equal wherever the oracle's a / s_out is
    farther than that bound (plus the quotients' own rounding) from every rounding boundary k + 1/2, and
    may differ by one next to a boundary.  Returns the number of codes that differ."""
    got, ref = np.asarray(got), np.asarray(ref)
    if not act:
        assert np.array_equal(got, ref)
        return 0
    qd = a.astype(np.float64) / np.float64(np.float32(s_out))
    dist = np.abs(qd - np.floor(qd) - 0.5)
    eps = (4e-7 + 2e-6 * np.abs(a.astype(np.float64))) / np.float64(np.float32(s_out)) + 1e-4
    diff = np.abs(got.astype(np.int32) - ref.astype(np.int32))
    assert np.all(diff[dist > eps] == 0), "codes differ away from every rounding boundary"
    assert diff.max() <= 1, "codes more than one apart"
    n = int(np.count_nonzero(diff))
    assert n <= max(2, 2e-3 * diff.size), "too many codes next to a boundary differ: %d of %d" % (n, diff.size)
    return n
