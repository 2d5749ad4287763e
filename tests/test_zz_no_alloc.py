"""The analysis entry point that allocates nothing (its work vectors are a static device array of the
library) against the entry point it is a variant of, through the raw C ABI: two calls in a row, the second
on a smaller input, so that whatever the first call left in the array would show."""
from __future__ import annotations

import ctypes

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cq():
    import paper_2410_07505_amd as pkg
    return pkg


def analysis_pair(cq, X, alpha, bits):
    """(xrk, counters) from crossquant_kernel_analysis and from crossquant_kernel_analysis_static."""
    import torch
    T, I = X.shape
    Xg = torch.from_numpy(X).cuda()
    t, c = cq.crossquant_absmax(Xg)
    xrk_ref, cnt_ref = cq.crossquant_kernel_analysis(Xg, t, c, alpha, bits)
    xrk = torch.full((T, I), 7.0, dtype=torch.float16, device="cuda")
    cnt = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    rc = cq.raw.crossquant_kernel_analysis_static(
        ctypes.c_void_p(Xg.data_ptr()), T, I, Xg.stride(0), ctypes.c_void_p(t.data_ptr()), ctypes.c_void_p(c.data_ptr()),
        alpha, bits, ctypes.c_void_p(xrk.data_ptr()), ctypes.c_void_p(cnt.data_ptr()), ctypes.c_void_p(stream))
    assert rc == 0, cq.crossquant_status_string(rc)
    torch.cuda.synchronize()
    return xrk_ref.cpu().numpy(), cnt_ref.cpu().numpy(), xrk.cpu().numpy(), cnt.cpu().numpy()


def test_static_analysis_matches_the_work_vector_form_twice_in_a_row(cq):
    print("no-alloc analysis: 300 x 1537 then 37 x 520", flush=True)
    for (T, I), alpha, bits in (((300, 1537), 0.15, 8), ((37, 520), 0.45, 4)):
        X = workloads.activation(T, I, seed=T + I, n_outlier=3, scale_lo=60.0, scale_hi=60.0)
        xrk_ref, cnt_ref, xrk, cnt = analysis_pair(cq, X, alpha, bits)
        assert np.array_equal(cnt, cnt_ref), (cnt, cnt_ref)
        assert np.array_equal(xrk.view(np.uint16), xrk_ref.view(np.uint16))
        assert cnt[0] > 0 and cnt[0] < X.size                      # a real kernel, not a degenerate count


def test_static_analysis_limits_and_argument_errors(cq):
    f = cq.raw.crossquant_kernel_analysis_static
    P = 0x10000
    big = (1 << 19) + 1
    assert f(P, big, 8, 8, P, P, 0.15, 8, P, P, None) == -2          # over the static array's limit: nothing launched
    assert f(P, 8, big, big, P, P, 0.15, 8, P, P, None) == -2
    assert f(P, 4, 8, 8, P, P, 0.15, 8, P, 0, None) == -1
    assert f(P, 4, 8, 8, P, P, 0.15, 5, P, P, None) == -3
    assert f(P, 4, 8, 8, P, P, 1.5, 8, P, P, None) == -4
