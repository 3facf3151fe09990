"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, answers the size
queries consistently with the documented layout, and rejects bad arguments before launching
anything (so none of this needs a GPU)."""
import ctypes as C
import os
import re

import pytest

import oracle
import paper_2511_11248_amd as tman
from paper_2511_11248_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(tman.library_path()):
        from paper_2511_11248_amd import build

        build.build(verbose=False)
    return api._load()


def test_every_declared_symbol_is_exported(lib):
    with open(os.path.join(ROOT, "include", "tman.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    names = set(re.findall(r"\b(tman_[a-z_]+)\s*\(", text))
    assert {"tman_pack_weights", "tman_build_lut", "tman_mpgemv", "tman_mpgemm"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in tman.h but not exported"


def test_binding_has_same_names():
    for n in ("tman_pack_weights", "tman_unpack_weights", "tman_build_lut", "tman_mpgemv", "tman_mpgemm",
              "tman_packed_bytes", "tman_lut_bytes", "tman_mpgemv_workspace_bytes", "tman_mpgemm_workspace_bytes",
              "tman_status_string", "tman_layout_version"):
        assert callable(getattr(tman, n))


@pytest.mark.parametrize("M,K,bits,group,hz", [
    (256, 512, 4, 64, True), (12288, 4096, 2, 64, True), (4096, 11008, 4, 128, True), (3072, 8192, 1, 64, False),
    (33, 96, 2, 32, True), (1, 32, 4, 32, True), (100, 384, 1, 128, True),
])
def test_packed_bytes_match_layout(lib, M, K, bits, group, hz):
    L = oracle.PackedLayout(M, K, bits, group, hz)
    assert tman.tman_packed_bytes(tman.Shape(M, K, bits, group, hz)) == L.total_bytes


def test_packed_bytes_are_the_algorithmic_bytes_on_aligned_shapes(lib):
    # bits/8 + 4/group bytes per weight (2/group without zeros), plus the 128-byte header
    for M, K, bits, group, hz, per_w in [(12288, 4096, 2, 64, True, 0.3125), (4096, 11008, 4, 128, True, 0.53125),
                                         (11008, 4096, 4, 64, True, 0.5625), (3072, 8192, 1, 64, False, 0.15625)]:
        assert tman.tman_packed_bytes(tman.Shape(M, K, bits, group, hz)) == 128 + int(M * K * per_w)


def test_lut_bytes(lib):
    assert tman.tman_lut_bytes(1, 4096, 64) == 4096 // 4 * 16 * 2 + (4096 // 64) * 4
    assert tman.tman_lut_bytes(3, 512, 64) == (512 // 4 * 16 * 2 + (512 // 64) * 4) * 4  # padded to 4 tokens
    assert tman.tman_lut_bytes(8, 11008, 128) == (11008 // 4 * 16 * 2 + (11008 // 128) * 4) * 8
    assert tman.tman_lut_bytes(1, 96, 32) == 1024 + 4 * 4  # K padded to one 128-column tile
    assert tman.tman_lut_bytes(0, 4096, 64) == 0
    assert tman.tman_lut_bytes(9, 4096, 64) == 0
    assert tman.tman_lut_bytes(1, 4096, 48) == 0
    assert tman.tman_lut_bytes(1, 100, 64) == 0


def _shape(M=64, K=256, bits=4, group=64, flags=1):
    return api._CShape(M, K, bits, group, flags)


FAKE = 0x1000  # non-NULL, 16-byte aligned, never dereferenced: validation fails first


@pytest.mark.parametrize("shape,status", [
    (_shape(bits=3), -2), (_shape(bits=0), -2), (_shape(bits=8), -2),
    (_shape(group=48), -3), (_shape(group=256), -3), (_shape(group=0), -3),
    (_shape(M=0), -4), (_shape(K=0), -4), (_shape(K=200), -4), (_shape(flags=2), -4),
    (_shape(bits=2, flags=0), -4),
])
def test_bad_shapes_are_rejected_everywhere(lib, shape, status):
    assert lib.tman_packed_bytes(C.byref(shape)) == 0
    assert lib.tman_mpgemv_workspace_bytes(C.byref(shape), 1) == 0
    assert lib.tman_pack_weights(C.byref(shape), FAKE, FAKE, FAKE, FAKE, None) == status
    assert lib.tman_unpack_weights(C.byref(shape), FAKE, FAKE, None, None, None) == status
    assert lib.tman_mpgemv(C.byref(shape), FAKE, FAKE, 1, FAKE, FAKE, 1 << 30, None) == status
    assert lib.tman_mpgemv_x(C.byref(shape), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == status
    assert lib.tman_mpgemm(C.byref(shape), FAKE, FAKE, 1, FAKE, None, 0, None) == status


def test_null_alignment_tokens_workspace(lib):
    s = _shape()
    assert lib.tman_pack_weights(None, FAKE, FAKE, FAKE, FAKE, None) == -1
    assert lib.tman_pack_weights(C.byref(s), None, FAKE, FAKE, FAKE, None) == -1
    assert lib.tman_pack_weights(C.byref(s), FAKE, None, FAKE, FAKE, None) == -1
    assert lib.tman_pack_weights(C.byref(s), FAKE, FAKE, None, FAKE, None) == -1  # zeros required with HAS_ZERO
    assert lib.tman_pack_weights(C.byref(s), FAKE, FAKE, FAKE, None, None) == -1
    assert lib.tman_pack_weights(C.byref(s), FAKE, FAKE, FAKE, FAKE + 4, None) == -6
    sign = _shape(bits=1, flags=0)
    assert lib.tman_pack_weights(C.byref(sign), FAKE, FAKE, FAKE, FAKE, None) == -4  # zeros given, format has none
    assert lib.tman_build_lut(None, 1, 256, 64, FAKE, None) == -1
    assert lib.tman_build_lut(FAKE, 1, 256, 64, None, None) == -1
    assert lib.tman_build_lut(FAKE, 0, 256, 64, FAKE, None) == -4
    assert lib.tman_build_lut(FAKE, 9, 256, 64, FAKE, None) == -4
    assert lib.tman_build_lut(FAKE, 1, 250, 64, FAKE, None) == -4
    assert lib.tman_build_lut(FAKE, 1, 256, 100, FAKE, None) == -3
    assert lib.tman_build_lut(FAKE, 1, 256, 64, FAKE + 8, None) == -6
    assert lib.tman_mpgemv(C.byref(s), None, FAKE, 1, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.tman_mpgemv(C.byref(s), FAKE, FAKE, 0, FAKE, FAKE, 1 << 30, None) == -4
    assert lib.tman_mpgemv(C.byref(s), FAKE, FAKE, 9, FAKE, FAKE, 1 << 30, None) == -4
    need = lib.tman_mpgemv_workspace_bytes(C.byref(s), 1)
    assert need > 0
    assert lib.tman_mpgemv(C.byref(s), FAKE, FAKE, 1, FAKE, None, 0, None) == -5
    assert lib.tman_mpgemv(C.byref(s), FAKE, FAKE, 1, FAKE, FAKE, need - 1, None) == -5
    assert lib.tman_mpgemv(C.byref(s), FAKE + 2, FAKE, 1, FAKE, FAKE, need, None) == -6
    assert lib.tman_mpgemm(C.byref(s), FAKE, None, 4, FAKE, None, 0, None) == -1
    assert lib.tman_mpgemm(C.byref(s), FAKE, FAKE, 0, FAKE, None, 0, None) == -4
    assert lib.tman_mpgemm(C.byref(s), FAKE, FAKE + 6, 4, FAKE, None, 0, None) == -6


def test_status_strings(lib):
    seen = {tman.tman_status_string(c) for c in range(0, -8, -1)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert tman.tman_status_string(-99) == "unknown status"
    with pytest.raises(tman.TmanError) as e:
        api._check(-3, "here")
    assert "group" in str(e.value)


def _ptrs(*vals):
    return (C.c_void_p * len(vals))(*vals)


def test_batched_lut_build_rejects_bad_arguments(lib):
    x, lut, K = _ptrs(FAKE, FAKE), _ptrs(FAKE, FAKE), (C.c_int32 * 2)(256, 512)
    assert lib.tman_build_lut_batch(2, None, 1, K, 64, lut, None) == -1
    assert lib.tman_build_lut_batch(2, x, 1, None, 64, lut, None) == -1
    assert lib.tman_build_lut_batch(2, x, 1, K, 64, None, None) == -1
    assert lib.tman_build_lut_batch(2, x, 1, K, 48, lut, None) == -3
    assert lib.tman_build_lut_batch(0, x, 1, K, 64, lut, None) == -4
    assert lib.tman_build_lut_batch(257, x, 1, K, 64, lut, None) == -4
    assert lib.tman_build_lut_batch(2, x, 0, K, 64, lut, None) == -4
    assert lib.tman_build_lut_batch(2, x, 9, K, 64, lut, None) == -4
    assert lib.tman_build_lut_batch(2, _ptrs(FAKE, None), 1, K, 64, lut, None) == -1
    assert lib.tman_build_lut_batch(2, x, 1, K, 64, _ptrs(FAKE, None), None) == -1
    assert lib.tman_build_lut_batch(2, x, 1, (C.c_int32 * 2)(256, 500), 64, lut, None) == -4
    assert lib.tman_build_lut_batch(2, x, 1, (C.c_int32 * 2)(256, 0), 64, lut, None) == -4
    assert lib.tman_build_lut_batch(2, x, 1, K, 64, _ptrs(FAKE, FAKE + 8), None) == -6


def test_batched_gemv_rejects_bad_arguments(lib):
    shapes = (api._CShape * 2)(_shape(M=64, K=256), _shape(M=128, K=512))
    packed, lut, y = _ptrs(FAKE, FAKE), _ptrs(FAKE, FAKE), _ptrs(FAKE, FAKE)
    ws = _ptrs(FAKE, FAKE + 0x10000)
    need = [lib.tman_mpgemv_workspace_bytes(C.byref(shapes[i]), 1) for i in range(2)]
    wsb = (C.c_size_t * 2)(*need)
    assert lib.tman_mpgemv_batch_desc_bytes(2) >= 2 * 64 and lib.tman_mpgemv_batch_desc_bytes(2) % 16 == 0
    assert lib.tman_mpgemv_batch_desc_bytes(0) == 0 and lib.tman_mpgemv_batch_desc_bytes(257) == 0

    def prepare(count=2, shapes=shapes, packed=packed, lut=lut, N=1, y=y, ws=ws, wsb=wsb, desc=FAKE):
        return lib.tman_mpgemv_batch_prepare(count, shapes, packed, lut, N, y, ws, wsb, desc, None)

    assert prepare(shapes=None) == -1
    assert prepare(count=0) == -4 and prepare(count=257) == -4
    assert prepare(N=0) == -4 and prepare(N=9) == -4
    assert prepare(packed=None) == -1 and prepare(lut=None) == -1 and prepare(y=None) == -1
    assert prepare(ws=None) == -1 and prepare(wsb=None) == -1 and prepare(desc=None) == -1
    assert prepare(desc=FAKE + 4) == -6
    assert prepare(packed=_ptrs(FAKE, None)) == -1
    assert prepare(lut=_ptrs(FAKE, FAKE + 2)) == -6
    assert prepare(wsb=(C.c_size_t * 2)(need[0], need[1] - 1)) == -5
    assert prepare(ws=_ptrs(FAKE, FAKE)) == -5  # two GEMVs of a launch may not share a workspace
    mixed = (api._CShape * 2)(_shape(M=64, K=256, bits=4), _shape(M=128, K=512, bits=2))
    assert prepare(shapes=mixed) == -4  # one launch runs one weight format
    bad = (api._CShape * 2)(_shape(M=64, K=256), _shape(M=128, K=500))
    assert prepare(shapes=bad) == -4

    assert lib.tman_mpgemv_batch_run(2, None, 1, FAKE, None) == -1
    assert lib.tman_mpgemv_batch_run(2, shapes, 1, None, None) == -1
    assert lib.tman_mpgemv_batch_run(2, shapes, 1, FAKE + 8, None) == -6
    assert lib.tman_mpgemv_batch_run(0, shapes, 1, FAKE, None) == -4
    assert lib.tman_mpgemv_batch_run(2, shapes, 9, FAKE, None) == -4
    assert lib.tman_mpgemv_batch_run(2, mixed, 1, FAKE, None) == -4


def test_one_token_gemv_with_own_tables_rejects_bad_arguments(lib):
    s = _shape()
    need = lib.tman_mpgemv_workspace_bytes(C.byref(s), 1)
    assert lib.tman_mpgemv_x(None, FAKE, FAKE, FAKE, FAKE, need, None) == -1
    assert lib.tman_mpgemv_x(C.byref(s), None, FAKE, FAKE, FAKE, need, None) == -1
    assert lib.tman_mpgemv_x(C.byref(s), FAKE, None, FAKE, FAKE, need, None) == -1
    assert lib.tman_mpgemv_x(C.byref(s), FAKE, FAKE, None, FAKE, need, None) == -1
    assert lib.tman_mpgemv_x(C.byref(s), FAKE, FAKE, FAKE, None, 0, None) == -5
    assert lib.tman_mpgemv_x(C.byref(s), FAKE, FAKE, FAKE, FAKE, need - 1, None) == -5
    assert lib.tman_mpgemv_x(C.byref(s), FAKE, FAKE + 2, FAKE, FAKE, need, None) == -6  # x: 16-byte aligned
    assert lib.tman_mpgemv_x(C.byref(s), FAKE + 8, FAKE, FAKE, FAKE, need, None) == -6

    shapes = (api._CShape * 2)(_shape(M=64, K=256), _shape(M=128, K=512))
    packed, xs, y = _ptrs(FAKE, FAKE), _ptrs(FAKE, FAKE), _ptrs(FAKE, FAKE)
    ws = _ptrs(FAKE, FAKE + 0x10000)
    needs = [lib.tman_mpgemv_workspace_bytes(C.byref(shapes[i]), 1) for i in range(2)]
    wsb = (C.c_size_t * 2)(*needs)

    def prepare(count=2, shapes=shapes, packed=packed, xs=xs, y=y, ws=ws, wsb=wsb, desc=FAKE):
        return lib.tman_mpgemv_x_batch_prepare(count, shapes, packed, xs, y, ws, wsb, desc, None)

    assert prepare(shapes=None) == -1
    assert prepare(count=0) == -4 and prepare(count=257) == -4
    assert prepare(packed=None) == -1 and prepare(xs=None) == -1 and prepare(y=None) == -1
    assert prepare(ws=None) == -1 and prepare(wsb=None) == -1 and prepare(desc=None) == -1
    assert prepare(desc=FAKE + 4) == -6
    assert prepare(xs=_ptrs(FAKE, None)) == -1
    assert prepare(xs=_ptrs(FAKE, FAKE + 2)) == -6
    assert prepare(wsb=(C.c_size_t * 2)(needs[0], needs[1] - 1)) == -5
    assert prepare(ws=_ptrs(FAKE, FAKE)) == -5
    mixed = (api._CShape * 2)(_shape(M=64, K=256, bits=4), _shape(M=128, K=512, bits=2))
    assert prepare(shapes=mixed) == -4
    assert lib.tman_mpgemv_x_batch_run(2, None, FAKE, None) == -1
    assert lib.tman_mpgemv_x_batch_run(2, shapes, None, None) == -1
    assert lib.tman_mpgemv_x_batch_run(2, shapes, FAKE + 8, None) == -6
    assert lib.tman_mpgemv_x_batch_run(0, shapes, FAKE, None) == -4
    assert lib.tman_mpgemv_x_batch_run(2, mixed, FAKE, None) == -4


def test_prefill_tile_rows_query(lib):
    """The tile height follows the number of workgroups it yields (256 compute units assumed without a
    device): a grid of at most one workgroup per unit takes the lowest tile, 512 / 768 / 1024 row blocks fill
    one round with 128 / 192 / 256 rows."""
    assert tman.tman_mpgemm_tile_rows(tman.Shape(256, 512, 4, 64, True), 128) == 64
    assert tman.tman_mpgemm_tile_rows(tman.Shape(11008, 4096, 4, 64, True), 256) == 128   # the K-split kernel's tall tile
    assert tman.tman_mpgemm_splits_k(tman.Shape(11008, 4096, 4, 64, True), 256) == 1
    assert tman.tman_mpgemm_tile_rows(tman.Shape(11008, 4096, 4, 64, True), 128) == 64    # ... its wide tile
    assert tman.tman_mpgemm_splits_k(tman.Shape(11008, 4096, 4, 64, True), 1024) == 0
    assert tman.tman_mpgemm_splits_k(tman.Shape(256, 512, 4, 64, True), 128) == 0          # K too short to split
    assert tman.tman_mpgemm_splits_k(tman.Shape(256, 500, 4, 64, True), 128) == -1
    assert tman.tman_mpgemm_tile_rows(tman.Shape(11008, 4096, 4, 64, True), 512) == 128
    assert tman.tman_mpgemm_tile_rows(tman.Shape(32768, 384, 4, 64, True), 200) == 128
    assert tman.tman_mpgemm_tile_rows(tman.Shape(11008, 4096, 4, 64, True), 1024) == 192
    assert tman.tman_mpgemm_tile_rows(tman.Shape(49152, 384, 4, 64, True), 200) == 192
    assert tman.tman_mpgemm_tile_rows(tman.Shape(65536, 384, 4, 64, True), 200) == 256
    assert tman.tman_mpgemm_tile_rows(tman.Shape(256, 500, 4, 64, True), 128) == 0
    assert tman.tman_mpgemm_tile_rows(tman.Shape(256, 512, 4, 64, True), 0) == 0


def test_noalloc_entry_point_validates_before_touching_the_gpu(lib):
    ok = _shape(M=64, K=256)
    assert lib.tman_mpgemv_noalloc(None, FAKE, FAKE, 1, FAKE, None) == -1
    assert lib.tman_mpgemv_noalloc(C.byref(ok), None, FAKE, 1, FAKE, None) == -1
    assert lib.tman_mpgemv_noalloc(C.byref(ok), FAKE, FAKE, 0, FAKE, None) == -4
    assert lib.tman_mpgemv_noalloc(C.byref(ok), FAKE, FAKE, 9, FAKE, None) == -4
    assert lib.tman_mpgemv_noalloc(C.byref(ok), FAKE + 8, FAKE, 1, FAKE, None) == -6
    assert lib.tman_mpgemv_noalloc(C.byref(_shape(bits=3)), FAKE, FAKE, 1, FAKE, None) == -2
    # the fixed array is 2 MiB: a workspace beyond it is refused on the sizes alone
    huge = _shape(M=1 << 20, K=16384)
    assert tman.tman_mpgemv_workspace_bytes(tman.Shape(1 << 20, 16384, 4, 64), 8) > 2 * 1024 * 1024
    assert lib.tman_mpgemv_noalloc(C.byref(huge), FAKE, FAKE, 8, FAKE, None) == -5


def test_header_check_validates_its_arguments(lib):
    ok = _shape()
    assert lib.tman_check_packed(None, FAKE, None) == -1
    assert lib.tman_check_packed(C.byref(ok), None, None) == -1
    assert lib.tman_check_packed(C.byref(_shape(group=48)), FAKE, None) == -3
    assert tman.tman_status_string(-8) != tman.tman_status_string(-99)
