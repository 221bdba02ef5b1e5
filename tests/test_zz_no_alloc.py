"""The entry point that allocates nothing (cb_sum_squared_diff_noalloc: partial sums in a statically
allocated device array of the library) against cb_sum_squared_diff with a caller-provided workspace:
same kernels, so the float64 results must agree bit for bit.  Two calls in a row, the second with a
smaller input, so that what the first call left in the shared array would show."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_1808_05488_amd as cb
from paper_1808_05488_amd import binding
from parity import prep, to_dev

pytestmark = pytest.mark.gpu


def _workspace():
    ws = torch.empty(cb.CB_METRIC_WORKSPACE_BYTES + 256, dtype=torch.uint8, device="cuda")
    off = (-ws.data_ptr()) % 256
    return ws[off:]


@pytest.mark.parametrize("bf16", [False, True])
def test_noalloc_metric_matches_the_workspace_form(bf16):
    dt = cb.CB_BF16 if bf16 else cb.CB_F32
    st = torch.cuda.current_stream().cuda_stream
    ws = _workspace()
    rng = np.random.default_rng(5)
    for n in (1 << 20 | 77, 4099, 1, 300001):                 # large, then smaller, then larger again
        print(f"noalloc metric: n = {n}, bf16 = {bf16}", flush=True)
        a = prep(rng.standard_normal(n).astype(np.float32), bf16)
        b = prep(rng.standard_normal(n).astype(np.float32), bf16)
        ad, bd = to_dev(a, bf16), to_dev(b, bf16)
        want = cb.cb_sum_squared_diff(ad, bd, n, dt, ws, st)
        before = torch.cuda.memory_allocated()
        got = cb.cb_sum_squared_diff_noalloc(ad, bd, n, dt, st)
        assert torch.cuda.memory_allocated() == before
        assert got == want, f"n = {n}: {got!r} != {want!r}"
        ref = float(np.sum((a.astype(np.float64) - b.astype(np.float64)) ** 2))
        assert abs(got - ref) <= 1e-12 * max(ref, 1.0)
    # n = 0 is legal and gives 0 whatever the last call left behind
    assert cb.cb_sum_squared_diff_noalloc(ad, bd, 0, dt, st) == 0.0


def test_noalloc_metric_rejects_what_it_cannot_take():
    a = torch.zeros(16, device="cuda")
    L = binding.lib()
    out = C.c_double()
    too_many = C.c_size_t((1 << 32) + 1)
    assert L.cb_sum_squared_diff_noalloc(a.data_ptr(), a.data_ptr(), too_many, cb.CB_F32, C.byref(out), None) == cb.CB_ENOMEM
    assert L.cb_sum_squared_diff_noalloc(None, a.data_ptr(), 16, cb.CB_F32, C.byref(out), None) == cb.CB_EINVAL
    assert L.cb_sum_squared_diff_noalloc(a.data_ptr(), a.data_ptr(), 16, 7, C.byref(out), None) == cb.CB_EINVAL
    assert L.cb_sum_squared_diff_noalloc(a.data_ptr(), a.data_ptr(), 16, cb.CB_F32, None, None) == cb.CB_EINVAL
