"""Host logic of the one-token decode launch: the cut of a batch's tile blocks into slots (one per resident
workgroup) that tman_mpgemv_x_batch_prepare makes, read back through tman_mpgemv_x_plan.  Checked by replaying
the walk the kernel makes over its slot: every tile block is visited exactly once and in order, the slots are
balanced, and the bookkeeping of row blocks shared by several slots (index of an interval among the row
block's intervals, their number) is what the exchange through the workspace needs."""
import random

import pytest

import paper_2511_11248_amd as tman

CHUNK = 40  # tile blocks whose tables a workgroup holds at a time
L7B = [(12288, 4096), (4096, 4096), (11008, 4096), (11008, 4096), (4096, 11008)]
L3B = [(9216, 3072), (3072, 3072), (8192, 3072), (8192, 3072), (3072, 8192)]


def _shapes(dims, bits=2, group=64):
    return [tman.Shape(M, K, bits, group) for M, K in dims]


def _replay(shapes, plan):
    """Walks every slot as the kernel does; returns per (gemv, row block) the list of (k0, len, index, count)."""
    rows, nk = [-(-s.M // 64) for s in shapes], [-(-s.K // 128) for s in shapes]
    seen = {}
    cursor = (0, 0)  # (gemv, linear tile) where the next slot has to start
    for gemv, first, count, pidx0, np_first, np_last in plan:
        g, pos, rem, is_first = gemv, first, count, True
        while cursor[0] < len(shapes) and cursor[1] >= rows[cursor[0]] * nk[cursor[0]]:
            cursor = (cursor[0] + 1, 0)
        assert (g, pos) == cursor, "slots must tile the sequence without gaps or overlaps"
        assert count > 0
        while rem > 0:
            if pos >= rows[g] * nk[g]:
                g, pos = g + 1, 0
                continue
            rb, k0 = divmod(pos, nk[g])
            ln = min(rem, nk[g] - k0)
            idx = pidx0 if is_first else 0
            cnt = 1 if (k0 == 0 and ln == nk[g]) else (np_first if is_first else np_last)
            seen.setdefault((g, rb), []).append((k0, ln, idx, cnt))
            pos, rem, is_first = pos + ln, rem - ln, False
        cursor = (g, pos)
    while cursor[0] < len(shapes) and cursor[1] >= rows[cursor[0]] * nk[cursor[0]]:
        cursor = (cursor[0] + 1, 0)
    assert cursor == (len(shapes), 0), "the last slot ends with the last tile block"
    return rows, nk, seen


def _check(shapes, max_slots):
    plan = tman.tman_mpgemv_x_plan(shapes, max_slots)
    assert 1 <= len(plan) <= max_slots
    rows, nk, seen = _replay(shapes, plan)
    assert len(seen) == sum(rows)
    for (g, rb), parts in seen.items():
        # the intervals of a row block cover its K tiles once, in order, numbered 0, 1, ... and all know the count
        assert [p[2] for p in parts] == list(range(len(parts)))
        assert all(p[3] == len(parts) for p in parts)
        k = 0
        for k0, ln, _, _ in parts:
            assert k0 == k and ln >= 1
            k += ln
        assert k == nk[g]
        assert len(parts) <= nk[g] // 8 + 2  # room reserved in the workspace
        if nk[g] <= CHUNK and max(c for _, _, c, _, _, _ in plan) >= nk[g]:
            assert len(parts) == 1, "a row block that fits a chunk and a slot is never split"
    total = sum(r * k for r, k in zip(rows, nk))
    longest = max(c for _, _, c, _, _, _ in plan)
    return plan, total, longest


def test_benchmark_layer_sets_are_balanced():
    plan, total, longest = _check(_shapes(L7B), 768)
    assert total == 24704 and longest <= 33 and len(plan) >= 760  # ideal 32.2 tile blocks per workgroup
    plan, total, longest = _check(_shapes(L7B, 4, 128), 768)
    assert longest <= 33
    plan, total, longest = _check(_shapes(L3B), 768)
    assert total == 13824 and longest == 18 and len(plan) == 768
    plan, total, longest = _check(_shapes(L3B * 32), 768)  # the whole 32-layer model in one launch
    assert longest * 768 <= total * 1.01


@pytest.mark.parametrize("max_slots", [1, 7, 256, 768, 4096])
def test_single_shapes(max_slots):
    for M, K in [(256, 512), (1, 32), (64, 4096), (70, 96), (130, 8320), (100, 11008), (33, 160), (5000, 5248), (64, 128 * 41)]:
        _check([tman.Shape(M, K, 4, 32)], max_slots)


def test_random_batches():
    rnd = random.Random(2511)
    for _ in range(60):
        n = rnd.randint(1, 12)
        dims = [(rnd.randint(1, 3000), 32 * rnd.randint(1, 400)) for _ in range(n)]
        _check([tman.Shape(M, K, 2, 32) for M, K in dims], rnd.choice([3, 64, 300, 768, 1024]))


def test_invalid_arguments_give_no_plan():
    sh = _shapes(L7B)
    assert tman.tman_mpgemv_x_plan(sh, 0) == []
    assert tman.tman_mpgemv_x_plan(sh, 5000) == []
    assert tman.tman_mpgemv_x_plan([tman.Shape(64, 100, 4, 64)], 768) == []
    assert tman.tman_mpgemv_x_plan([tman.Shape(64, 128, 4, 64), tman.Shape(64, 128, 2, 64)], 768) == []  # mixed formats
