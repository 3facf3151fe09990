"""Seeded random shapes and formats through all three matmul entry points, every output against the oracle.
The hand-picked cases of the other files pin the known edges; this sweep looks for the ones nobody thought of."""
import numpy as np
import pytest

import oracle
import paper_2511_11248_amd as tman
from gpu_helpers import TOL, mpgemm, mpgemv, mpgemv_x, pack, rand_case

pytestmark = pytest.mark.gpu

FORMATS = [(4, 32, True), (4, 64, True), (4, 128, True), (2, 32, True), (2, 64, True), (2, 128, True),
           (1, 32, False), (1, 64, False), (1, 128, True), (1, 64, True)]


@pytest.mark.parametrize("block", range(4))
def test_random_shapes(oracle_lib, block):
    rng = np.random.default_rng(2511_11248 + block)
    for it in range(20):
        bits, group, hz = FORMATS[rng.integers(len(FORMATS))]
        M = int(rng.integers(33, 700))                 # enough outputs per token for the row-normalised metric
        K = group * int(rng.integers(1, 6000 // group))
        kind = int(rng.integers(3))
        N = 1 if kind == 1 else int(rng.integers(1, 9)) if kind == 0 else int(rng.integers(1, 600))
        q, s, z, x = rand_case(50000 + 100 * block + it, M, K, N, bits, group, hz)
        shape = tman.Shape(M, K, bits, group, hz)
        y = (mpgemv, mpgemv_x, mpgemm)[kind](shape, pack(shape, q, s, z), x)
        err = oracle.row_relative_error(y, oracle.matmul(q, s, z, x, bits, group)).max()
        assert np.isfinite(err) and err <= TOL, f"{('mpgemv', 'mpgemv_x', 'mpgemm')[kind]} {shape} N={N}: {err:.3e}"


@pytest.mark.parametrize("mode", [2, 3])
def test_random_shapes_through_the_k_split_prefill_kernel(oracle_lib, mode):
    """The same sweep for the prefill kernel whose waves split K, which the launcher only picks for long K on small
    grids: forced here (tiling.prefill_k_split) for random shapes with its 64 x 256 (2) and 128 x 128 (3) tile."""
    t = tman.tman_default_tiling()
    t.prefill_k_split = mode
    tman.tman_set_tiling(t)
    try:
        rng = np.random.default_rng(2511_11248 + 10 * mode)
        for it in range(16):
            bits, group, hz = FORMATS[rng.integers(len(FORMATS))]
            M = int(rng.integers(33, 500))
            K = group * int(rng.integers(1, 5000 // group))
            N = int(rng.integers(33, 420))
            q, s, z, x = rand_case(70000 + 100 * mode + it, M, K, N, bits, group, hz)
            shape = tman.Shape(M, K, bits, group, hz)
            assert tman.tman_mpgemm_splits_k(shape, N) == 1
            y = mpgemm(shape, pack(shape, q, s, z), x)
            err = oracle.row_relative_error(y, oracle.matmul(q, s, z, x, bits, group)).max()
            assert np.isfinite(err) and err <= TOL, f"k split {mode} {shape} N={N}: {err:.3e}"
    finally:
        tman.tman_set_tiling(tman.tman_default_tiling())


def test_ternary_weights_with_one_scale_per_tensor(oracle_lib):
    """The paper's BitNet configuration (Sec. 6.1: ternary weights treated as 2-bit, one scale per tensor; kernel
    shapes 2560 / 6912) expressed in the group format: codes in {0, 1, 2}, zero = 1, every group the same scale.
    Decode (both forms) and prefill against the oracle; with scale 1 and small integer activations the
    result is an exact integer."""
    import synth
    M, K, bits, group = 2560, 6912, 2, 64
    q = (synth.uniform_codes(901, M * K, 2) % 3).astype(np.uint8).reshape(M, K)
    z = np.ones((M, K // group), dtype=np.float16)
    s = np.full((M, K // group), 0.0123, dtype=np.float16)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    x = synth.normal_fp16(902, 3 * K).reshape(3, K)
    Y = oracle.matmul(q, s, z, x, bits, group)
    assert oracle.row_relative_error(mpgemv(shape, blob, x), Y).max() <= TOL
    assert oracle.row_relative_error(mpgemv_x(shape, blob, x[:1]), Y[:1]).max() <= TOL
    assert oracle.row_relative_error(mpgemm(shape, blob, x), Y).max() <= TOL
    # exact case: scale 1, activations in {-1, 0, 1}: every partial sum is a small integer
    ones = np.ones_like(s)
    xi = (synth.uniform_codes(903, K, 2) % 3).astype(np.int64).reshape(1, K) - 1
    ref = xi @ (q.astype(np.int64) - 1).T
    assert np.abs(ref).max() < 2048
    blob1 = pack(shape, q, ones, z)
    xf = xi.astype(np.float16)
    assert np.array_equal(mpgemv_x(shape, blob1, xf).astype(np.int64), ref)
    assert np.array_equal(mpgemv(shape, blob1, xf).astype(np.int64), ref)
    assert np.array_equal(mpgemm(shape, blob1, xf).astype(np.int64), ref)
