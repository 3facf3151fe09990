"""The numbering of a one-token batch's workgroups (tman_mpgemv_x_batch_order): host logic.  The dispatcher deals
the workgroups of a launch that is resident at once to the compute units by position (id mod units), so the
numbering must (a) name every workgroup of every GEMV exactly once and (b) give the units equal work."""
import pytest

import paper_2511_11248_amd as tman
import synth


def _layer_shapes(name):
    w = synth.WORKLOADS[name]
    return [tman.Shape(l.M, l.K, w.bits, w.group, w.has_zero) for l in w.layers]


def _plan(shape, t):
    """(segments per row block, tiles per segment) of tman_mpgemv_x under tiling t, restated from the header's rule."""
    tile_bytes = shape.bits * 1024 + 64 * (128 // shape.group) * (4 if shape.has_zero else 2)
    n_kt = -(-shape.K // 128)
    whole = max(1, min(t.decode_x_whole_bytes // tile_bytes, t.decode_x_seg_tiles))
    cap = whole if n_kt <= whole else t.decode_x_long_seg_tiles
    n_seg = -(-n_kt // cap)
    return n_seg, -(-n_kt // n_seg), n_kt


@pytest.mark.parametrize("name,n_units", [("7b_w2g64", 256), ("7b_w4g128", 256), ("3p8b_w2g64", 256),
                                          ("3p8b_w1g64", 256), ("7b_w2g64", 304), ("tiny_w4g64", 256)])
def test_numbering_is_a_balanced_permutation(name, n_units):
    shapes = _layer_shapes(name)
    t = tman.tman_get_tiling()
    order = tman.tman_mpgemv_x_batch_order(shapes, n_units)
    expected = set()
    tiles_of = {}
    for g, s in enumerate(shapes):
        n_seg, seg, n_kt = _plan(s, t)
        for rb in range(-(-s.M // 64)):
            for k in range(n_seg):
                expected.add((g, rb * n_seg + k))
                tiles_of[(g, rb * n_seg + k)] = min(seg, n_kt - k * seg)
    assert order, "a batch of five GEMVs that is resident at once is numbered"
    assert len(order) == len(expected) and set(order) == expected
    load = [0] * n_units
    for i, e in enumerate(order):
        load[i % n_units] += tiles_of[e]
    biggest = max(tiles_of.values())
    assert max(load) - min(load) <= biggest, (min(load), max(load))
    # inside a unit the ids ascend with falling work
    for j in range(min(n_units, len(order))):
        mine = [tiles_of[order[i]] for i in range(j, len(order), n_units)]
        assert mine == sorted(mine, reverse=True)


def test_batches_that_do_not_qualify_keep_the_plain_grid():
    nine = [tman.Shape(256, 512, 4, 64)] * 9
    assert tman.tman_mpgemv_x_batch_order(nine, 256) == []
    whole_model = _layer_shapes("7b_w2g64") * 32
    assert tman.tman_mpgemv_x_batch_order(whole_model, 256) == []
    # more workgroups than are resident at once: 8 GEMVs of 12288 x 4096 -> 1536 workgroups of 32 tiles, 4 per unit
    big = [tman.Shape(12288, 4096, 2, 64)] * 8
    assert tman.tman_mpgemv_x_batch_order(big, 256) == []
    assert tman.tman_mpgemv_x_batch_order(big[:5], 256)  # 960 fit
    t = tman.tman_get_tiling()
    try:
        off = tman.tman_get_tiling()
        off.decode_balance = 0
        tman.tman_set_tiling(off)
        assert tman.tman_mpgemv_x_batch_order(_layer_shapes("7b_w2g64"), 256) == []
    finally:
        tman.tman_set_tiling(t)
