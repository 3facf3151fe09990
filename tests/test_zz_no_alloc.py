"""tman_mpgemv_noalloc (the entry point for callers that cannot allocate: its workspace is a fixed device
array owned by the library) against tman_mpgemv with a caller workspace: same kernels, so bit-identical
outputs, and both within tolerance of the fp64 oracle.  Two calls in a row, the second with a smaller input,
so whatever the first call left in the shared array must not disturb the second."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
from gpu_helpers import TOL, build_lut, dev, gemv_workspace, pack, rand_case, to_dev

pytestmark = pytest.mark.gpu


def _both(shape, q, s, z, x):
    N = x.shape[0]
    blob = pack(shape, q, s, z)
    lut = build_lut(to_dev(x), shape.group)
    y_ws = torch.full((N, shape.M), float("nan"), dtype=torch.float16, device=dev())
    y_na = torch.full((N, shape.M), float("nan"), dtype=torch.float16, device=dev())
    tman.tman_mpgemv(shape, blob, lut, N, y_ws, gemv_workspace(shape, N))
    tman.tman_mpgemv_noalloc(shape, blob, lut, N, y_na)
    torch.cuda.synchronize()
    return y_ws.cpu().numpy(), y_na.cpu().numpy()


def test_two_calls_in_a_row_the_second_smaller(oracle_lib):
    tman.tman_noalloc_init()
    # K longer than one segment in both calls, so tickets and partial sums in the fixed array are really used
    cases = [(512, 11008, 2, 64, 4, 71), (130, 8320, 4, 64, 1, 72)]
    for M, K, bits, group, N, seed in cases:
        shape = tman.Shape(M, K, bits, group)
        assert 0 < tman.tman_mpgemv_workspace_bytes(shape, N) <= 2 * 1024 * 1024
        q, s, z, x = rand_case(seed, M, K, N, bits, group)
        y_ws, y_na = _both(shape, q, s, z, x)
        assert np.all(np.isfinite(y_na.astype(np.float32)))
        assert np.array_equal(y_ws.view(np.uint16), y_na.view(np.uint16))
        assert oracle.row_relative_error(y_na, oracle.matmul(q, s, z, x, bits, group)).max() <= TOL


def test_repeated_calls_are_identical_and_oversized_shapes_are_refused(oracle_lib):
    M, K, bits, group, N = 200, 9000 // 64 * 64, 4, 64, 8
    shape = tman.Shape(M, K, bits, group)
    q, s, z, x = rand_case(73, M, K, N, bits, group)
    a_ws, a = _both(shape, q, s, z, x)
    b_ws, b = _both(shape, q, s, z, x)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16)) and np.array_equal(a.view(np.uint16), a_ws.view(np.uint16))
    big = tman.Shape(1 << 20, 16384, 4, 64)  # workspace far beyond the fixed array
    assert tman.tman_mpgemv_workspace_bytes(big, 8) > 2 * 1024 * 1024
    with pytest.raises(tman.TmanError) as e:
        tman.tman_mpgemv_noalloc(big, 16, 16, 8, 16)  # refused on the sizes alone, before any pointer is used
    assert e.value.status == -5
