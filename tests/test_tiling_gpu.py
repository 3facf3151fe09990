"""Results do not depend on the tiling: every admissible setting of tman_tiling_t gives outputs within the
tolerance of the oracle (the tiling changes how K is cut across workgroups and how many rows a prefill workgroup
takes, i.e. only the order of fp32 additions)."""
import numpy as np
import pytest

import oracle
import paper_2511_11248_amd as tman
from gpu_helpers import TOL, mpgemm, mpgemv, mpgemv_x, pack, rand_case

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def restore():
    yield
    tman.tman_set_tiling(tman.tman_default_tiling())


@pytest.mark.parametrize("setting", [
    dict(decode_x_long_seg_tiles=7, decode_seg_tiles=5, decode_seg_tiles_many=9, small_seg_tiles=11, prefill_row_blocks=1),
    dict(decode_x_seg_tiles=16, decode_x_long_seg_tiles=16, decode_seg_tiles=64, decode_seg_tiles_many=40, small_seg_tiles=200,
         prefill_row_blocks=4),
    dict(decode_x_whole_bytes=4096, prefill_row_blocks=2),
    dict(decode_x_long_seg_tiles=32, prefill_row_blocks=3),
    dict(prefill_k_split=2), dict(prefill_k_split=3, i8_token_blocks=3),
])
def test_every_kernel_under_other_tilings(oracle_lib, setting):
    t = tman.tman_default_tiling()
    for k, v in setting.items():
        setattr(t, k, v)
    tman.tman_set_tiling(t)
    M, K, bits, group = 200, 8320, 4, 64
    q, s, z, x = rand_case(1234, M, K, 8, bits, group)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    Y = oracle.matmul(q, s, z, x, bits, group)
    assert oracle.row_relative_error(mpgemv_x(shape, blob, x[:1]), Y[:1]).max() <= TOL
    assert oracle.row_relative_error(mpgemv(shape, blob, x[:1]), Y[:1]).max() <= TOL
    assert oracle.row_relative_error(mpgemv(shape, blob, x), Y).max() <= TOL
    assert oracle.row_relative_error(mpgemm(shape, blob, x), Y).max() <= TOL          # small-batch kernel
    xp = np.concatenate([x] * 38)[:300]                                                 # tiled prefill kernel
    assert oracle.row_relative_error(mpgemm(shape, blob, xp), np.concatenate([Y] * 38)[:300]).max() <= TOL
