"""The entry point that allocates nothing (thi_linear_static) against thi_linear, through the C ABI.

Same kernels, same dispatch: the results must be identical bit for bit (and thi_linear itself is held to
|gpu - y| <= 4e-3 * S against the oracle elsewhere).  Two calls in a row, the second with a smaller input,
on shapes whose kernels use the scratch array (shared row blocks: arrival counters and hand-over slots;
stream-K: flags and slots), then the limit and the argument errors."""
import ctypes

import numpy as np
import pytest

from paper_2605_25655_amd import synth
from tests.gpu_common import new_out, say, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def thi():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2605_25655_amd as thi
    thi.load_library()
    thi.thi_set_kernel_family(0)
    thi.thi_set_rowblock_split(0)
    return thi


def _both(thi, x, w, ws):
    xd, wd = to_dev(x), to_dev(w)
    a = new_out(x.shape[0], w.shape[0])
    thi.thi_linear(xd, wd, a, ws)
    b = new_out(x.shape[0], w.shape[0])
    thi.thi_linear_static(xd, wd, b)
    return to_host(a), to_host(b)


@pytest.mark.parametrize("family", [0, 1, 4])
def test_static_scratch_matches_the_workspace_entry_point(thi, family):
    # 7B down-projection shape (shared row blocks under the automatic choice; every stream-K tile is
    # shared), then a smaller problem on the same scratch array
    big, small = (32, 4096, 11008), (5, 1000, 2048)
    ws = thi.Workspace(thi.thi_workspace_bytes(1, 32, 4096, 11008))
    prev = thi.thi_set_kernel_family(family)
    try:
        for M, N, K in (big, small):
            say(f"[case] thi_linear_static family={family} M={M} N={N} K={K}")
            x, w, _ = synth.random_problem(7100 + M + N + K, M, N, K)
            a, b = _both(thi, x, w, ws)
            assert np.isfinite(a.astype(np.float32)).all()
            assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), f"differs at family={family} M={M} N={N} K={K}"
    finally:
        thi.thi_set_kernel_family(prev)


def test_static_scratch_limits_and_errors(thi):
    lib = thi.load_library()
    x, w, _ = synth.random_problem(7200, 33, 64, 64)
    xd, wd = to_dev(x), to_dev(w)
    out = new_out(33, 64)
    assert thi.thi_linear_static(xd, wd, out, check=False) == 2          # M beyond the static scratch's limit
    null = ctypes.c_void_p(0)
    p = ctypes.c_void_p(xd.data_ptr())
    assert lib.thi_linear_static(null, p, p, 1, 8, 8, null) == 1
    assert lib.thi_linear_static(p, p, p, 1, 8, 12, null) == 2
    assert lib.thi_linear_static(ctypes.c_void_p(p.value + 2), p, p, 1, 8, 8, null) == 3
    prev = thi.thi_set_kernel_family(2)
    try:
        assert thi.thi_linear_static(xd[:4], wd, out[:4], check=False) == thi.THI_ERR_WORKSPACE
    finally:
        thi.thi_set_kernel_family(prev)
