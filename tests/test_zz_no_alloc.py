"""qarvd_quantize_weight_static (the entry point that allocates nothing: its workspace is a fixed device array
inside the library) against qarvd_quantize_weight on the same inputs, through the C ABI: every output bit for
bit, on two calls in a row, the second with a smaller layer (the array still holds the first call's data)."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2605_21072_amd")


def _outputs(N, K):
    ld = q.packed_k(K, -1)
    return q.DualScaleWeight(torch.full((N, ld), 0x33, dtype=torch.int8, device="cuda"),
                             torch.empty(N, dtype=torch.float32, device="cuda"),
                             torch.empty(N, dtype=torch.float32, device="cuda"),
                             torch.empty(K, dtype=torch.int32, device="cuda"), -1, N, K,
                             torch.empty(K, dtype=torch.float32, device="cuda"))


def _allocations():
    """How many device allocations torch's allocator has served so far (frees, e.g. of an earlier test's garbage
    collected in between, do not change it)."""
    return torch.cuda.memory_stats().get("allocation.all.allocated", 0)


def _same(a, b):
    assert a.K_o == b.K_o
    kp = q.packed_k(a.K, a.K_o)
    assert torch.equal(a.perm, b.perm)
    assert torch.equal(a.Wq[:, :kp], b.Wq[:, :kp])
    assert torch.equal(a.s_normal.view(torch.int32), b.s_normal.view(torch.int32))
    assert torch.equal(a.s_outlier.view(torch.int32), b.s_outlier.view(torch.int32))
    assert torch.equal(a.v.view(torch.int32), b.v.view(torch.int32))


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    assert torch.cuda.is_available(), "GPU tests need a device"
    q.load_library()
    assert q.quantize_weight_static_max_k() == 16384
    cases = [wl.small_random_case(9001, 4, 640, 8960, 70), wl.small_random_case(9002, 4, 200, 1000, 9),
             wl.small_random_case(9003, 4, 96, 1536, 0)]
    for L in cases:                                   # the second and third layers are smaller than the first
        W = torch.from_numpy(L["W"]).cuda()
        N, K = W.shape
        ref = q.quantize_weight(W)                    # the existing entry point (caller-provided workspace)
        out = _outputs(N, K)                          # the caller's buffers
        before = _allocations()
        q.quantize_weight_static(W, out)              # fills `out` in place
        assert _allocations() == before               # nothing of torch's was allocated by the call either
        torch.cuda.synchronize()
        _same(out, ref)
        assert out.K_o == (L["spec"].n_outlier + 31) // 32 * 32
        del out, ref


def test_static_scratch_entry_point_rejects_a_k_beyond_its_array():
    q.load_library()
    K = q.quantize_weight_static_max_k() + 128
    W = torch.zeros((8, K), dtype=torch.float32, device="cuda")
    with pytest.raises(q.QarvdError) as e:
        q.quantize_weight_static(W, _outputs(8, K))
    assert e.value.status == -3
