"""Packed blobs carry a header; a blob used with another shape must not be consumed silently.  The host-side
check (tman_check_packed) reports it at once; the compute calls check on the device, leave the outputs of the
affected GEMV untouched and record TMAN_ERR_HEADER in the status word that tman_device_status returns.
Every foreign shape used here is SMALLER than the blob's own, so all reads stay inside the blob."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
from gpu_helpers import TOL, build_lut, dev, gemv_workspace, pack, rand_case, to_dev

pytestmark = pytest.mark.gpu
ERR_HEADER = -8


def _untouched(y):
    return bool(torch.isnan(y).all())


def test_host_side_check():
    M, K, bits, group = 128, 512, 4, 64
    q, s, z, _ = rand_case(5, M, K, 1, bits, group)
    good = tman.Shape(M, K, bits, group)
    blob = pack(good, q, s, z)
    assert tman.tman_check_packed(good, blob) == 0
    for other in (tman.Shape(64, K, bits, group), tman.Shape(M, 256, bits, group), tman.Shape(M, K, 2, group),
                  tman.Shape(M, K, bits, 32), tman.Shape(M, K, 1, group, False)):
        assert tman.tman_check_packed(other, blob) == ERR_HEADER
    blob2 = blob.clone()
    blob2[13 * 4] = 9  # a layout version this build does not read
    assert tman.tman_check_packed(good, blob2) == ERR_HEADER


def test_single_calls_refuse_a_foreign_blob(oracle_lib):
    M, K, bits, group, N = 128, 512, 4, 64, 2
    q, s, z, x = rand_case(6, M, K, N, bits, group)
    good, wrong = tman.Shape(M, K, bits, group), tman.Shape(64, K, bits, group)
    blob = pack(good, q, s, z)
    assert tman.tman_device_status() == 0
    xd = to_dev(x)
    lut = build_lut(xd, group)
    nan = lambda rows, cols: torch.full((rows, cols), float("nan"), dtype=torch.float16, device=dev())
    # each of the three compute calls, with the wrong shape first: nothing written, status raised once
    y = nan(N, 64)
    tman.tman_mpgemv(wrong, blob, lut, N, y, gemv_workspace(wrong, N))
    assert tman.tman_device_status() == ERR_HEADER and _untouched(y)
    assert tman.tman_device_status() == 0  # reading clears it
    y = nan(1, 64)
    tman.tman_mpgemv_x(wrong, blob, xd[0], y, gemv_workspace(wrong, 1))
    assert tman.tman_device_status() == ERR_HEADER and _untouched(y)
    y = nan(N, 64)
    tman.tman_mpgemm(wrong, blob, xd, N, y, None)
    assert tman.tman_device_status() == ERR_HEADER and _untouched(y)
    # and with the right one: results, no status
    Y = oracle.matmul(q, s, z, x, bits, group)
    y = nan(N, M)
    tman.tman_mpgemv(good, blob, lut, N, y, gemv_workspace(good, N))
    y1 = nan(1, M)
    tman.tman_mpgemv_x(good, blob, xd[0], y1, gemv_workspace(good, 1))
    y2 = nan(N, M)
    tman.tman_mpgemm(good, blob, xd, N, y2, None)
    assert tman.tman_device_status() == 0
    assert oracle.row_relative_error(y.cpu().numpy(), Y).max() <= TOL
    assert oracle.row_relative_error(y1.cpu().numpy(), Y[:1]).max() <= TOL
    assert oracle.row_relative_error(y2.cpu().numpy(), Y).max() <= TOL


@pytest.mark.parametrize("one_launch", [True, False])
def test_a_batch_skips_the_foreign_blob_and_computes_the_rest(oracle_lib, one_launch):
    bits, group = 2, 64
    dims = [(128, 512), (192, 4608), (70, 256)]
    shapes, blobs, xs, luts, ys, wss, refs = [], [], [], [], [], [], []
    for i, (M, K) in enumerate(dims):
        q, s, z, x = rand_case(40 + i, M, K, 1, bits, group)
        shape = tman.Shape(M, K, bits, group)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); xs.append(to_dev(x))
        luts.append(build_lut(xs[-1], group))
        ys.append(torch.full((1, M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, 1)); refs.append((q, s, z, x))
    # GEMV 1 is declared with fewer rows than its blob was packed for
    shapes[1] = tman.Shape(128, 4608, bits, group)
    ys[1] = torch.full((1, 128), float("nan"), dtype=torch.float16, device=dev())
    wss[1] = gemv_workspace(shapes[1], 1)
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(3), dtype=torch.uint8, device=dev())
    if one_launch:
        tman.tman_mpgemv_x_batch_prepare(shapes, blobs, xs, ys, wss, desc)
        assert tman.tman_device_status() == ERR_HEADER  # found when the table is written
        tman.tman_mpgemv_x_batch_run(shapes, desc)
    else:
        tman.tman_mpgemv_batch_prepare(shapes, blobs, luts, 1, ys, wss, desc)
        assert tman.tman_device_status() == ERR_HEADER
        tman.tman_mpgemv_batch_run(shapes, 1, desc)
    torch.cuda.synchronize()
    assert _untouched(ys[1])
    for i in (0, 2):
        q, s, z, x = refs[i]
        assert oracle.row_relative_error(ys[i].cpu().numpy(), oracle.matmul(q, s, z, x, bits, group)).max() <= TOL
