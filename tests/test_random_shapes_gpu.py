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
