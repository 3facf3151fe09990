"""The tiling setting (Sec. 4.1 unified tiling, Eq. 1-4 in this machine's terms): defaults, constraint checks and
its effect on the host-side plans, without a GPU."""
import pytest

import paper_2511_11248_amd as tman


@pytest.fixture(autouse=True)
def restore():
    yield
    tman.tman_set_tiling(tman.tman_default_tiling())


def _with(**kw):
    t = tman.tman_default_tiling()
    for k, v in kw.items():
        setattr(t, k, v)
    return t


def test_defaults_are_current_and_consistent():
    d, c = tman.tman_default_tiling().as_dict(), tman.tman_get_tiling().as_dict()
    assert d == c
    assert d["decode_x_seg_tiles"] == 32 and 1 <= d["decode_x_long_seg_tiles"] <= 32
    assert d["prefill_row_blocks"] == 0 and d["small_seg_tiles"] == 43


@pytest.mark.parametrize("bad", [
    dict(decode_x_seg_tiles=33),            # Eq. 1: 33 KB of tables do not fit the workgroup's 32 KB
    dict(decode_x_seg_tiles=0),
    dict(decode_x_long_seg_tiles=40),       # longer than a whole segment may be
    dict(decode_x_long_seg_tiles=0),
    dict(prefill_row_blocks=5),             # Eq. 4: 4 x (320 x 80 + 256 x 64) bytes exceed 160 KB
    dict(prefill_row_blocks=-1),
    dict(decode_seg_tiles=0), dict(decode_seg_tiles_many=0), dict(small_seg_tiles=0), dict(decode_x_whole_bytes=0),
    dict(i8_token_blocks=2), dict(i8_token_blocks=8), dict(i8_token_blocks=-1),  # only 0, 1, 3, 4, 7 and 9 exist
    dict(prefill_k_split=4), dict(prefill_k_split=-1),
])
def test_constraint_violations_are_refused_and_change_nothing(bad):
    with pytest.raises(tman.TmanError) as e:
        tman.tman_set_tiling(_with(**bad))
    assert e.value.status == -4
    assert tman.tman_get_tiling().as_dict() == tman.tman_default_tiling().as_dict()


def test_tiling_enters_the_plans():
    down = tman.Shape(4096, 11008, 2, 64)  # 86 K tiles, 64 row blocks
    ws_default = tman.tman_mpgemv_workspace_bytes(down, 8)
    assert ws_default == 256 + 64 * 4 * 8 * 64 * 4          # 24-tile cap: four segments of 22, 22, 22, 20
    tman.tman_set_tiling(_with(decode_seg_tiles_many=43))
    assert tman.tman_mpgemv_workspace_bytes(down, 8) == 256 + 64 * 2 * 8 * 64 * 4  # two segments of 43
    tman.tman_set_tiling(_with(decode_seg_tiles_many=86))
    assert tman.tman_mpgemv_workspace_bytes(down, 8) == 256  # one segment: tickets only
    tman.tman_set_tiling(tman.tman_default_tiling())
    assert tman.tman_mpgemm_workspace_bytes(down, 8) > 0
    tman.tman_set_tiling(_with(small_seg_tiles=86))
    assert tman.tman_mpgemm_workspace_bytes(down, 8) == 0
    pre = tman.Shape(11008, 4096, 4, 64)
    assert tman.tman_mpgemm_tile_rows(pre, 1024) == 192
    tman.tman_set_tiling(_with(prefill_row_blocks=2))
    assert tman.tman_mpgemm_tile_rows(pre, 1024) == 128
    # small grids go to the kernel whose waves split K, unless told otherwise
    tman.tman_set_tiling(tman.tman_default_tiling())
    assert (tman.tman_mpgemm_splits_k(pre, 256), tman.tman_mpgemm_tile_rows(pre, 256)) == (1, 128)
    assert (tman.tman_mpgemm_splits_k(pre, 100), tman.tman_mpgemm_tile_rows(pre, 100)) == (1, 64)
    tman.tman_set_tiling(_with(prefill_k_split=1))
    assert (tman.tman_mpgemm_splits_k(pre, 256), tman.tman_mpgemm_tile_rows(pre, 256)) == (0, 64)
    tman.tman_set_tiling(_with(prefill_k_split=2))
    assert (tman.tman_mpgemm_splits_k(pre, 4096), tman.tman_mpgemm_tile_rows(pre, 4096)) == (1, 64)
    tman.tman_set_tiling(_with(prefill_k_split=3))
    assert (tman.tman_mpgemm_splits_k(pre, 4096), tman.tman_mpgemm_tile_rows(pre, 4096)) == (1, 128)
    # the integer prefill kernel: chosen per call (a short token range: the 128 x 128 kernel; long ones: the kernel that
    # dequantizes in registers, with the token tile that fills 256 units best), or forced
    tman.tman_set_tiling(tman.tman_default_tiling())
    assert tman.tman_mpgemm_i8_token_blocks(pre, 256) == 9
    assert tman.tman_mpgemm_i8_token_blocks(pre, 1024) in (3, 4, 7)
    assert tman.tman_mpgemm_i8_token_blocks(tman.Shape(256, 512, 4, 64), 128) == 1
    assert tman.tman_mpgemm_i8_token_blocks(tman.Shape(256, 500, 4, 64), 128) == 0
    for forced in (1, 3, 4, 7, 9):
        tman.tman_set_tiling(_with(i8_token_blocks=forced))
        assert tman.tman_mpgemm_i8_token_blocks(pre, 1024) == forced
        assert tman.tman_mpgemm_i8_token_blocks(pre, 5) == forced
