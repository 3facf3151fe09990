"""tman_mpgemm (prefill, table dequantization + MFMA) against the fp64 definition oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
import synth
from gpu_helpers import TOL, mpgemm, pack, rand_case, to_dev

pytestmark = pytest.mark.gpu


def _check(shape, q, s, z, x):
    y = mpgemm(shape, pack(shape, q, s, z), x)
    Y = oracle.matmul(q, s, z, x, shape.bits, shape.group)
    assert np.all(np.isfinite(y.astype(np.float32)))
    err = oracle.row_relative_error(y, Y)
    assert err.max() <= TOL, f"row-normalised error {err.max():.3e} > {TOL}"


SMALL = [
    # M, K, bits, group, has_zero, N
    (256, 512, 4, 64, True, 128),
    (256, 512, 4, 64, True, 1),
    (70, 96, 4, 32, True, 37),       # ragged everywhere, K < one tile
    (130, 2816, 2, 64, True, 130),   # N spills into a second token tile
    (96, 1024, 4, 128, True, 256),
    (64, 768, 1, 64, False, 64),
    (64, 512, 1, 128, True, 33),
    (64, 256, 2, 32, True, 200),
    (1, 32, 4, 32, True, 1),
    (300, 1280, 4, 64, True, 260),
]


@pytest.fixture
def restore_tiling():
    yield
    tman.tman_set_tiling(tman.tman_default_tiling())


def _k_split(mode):
    t = tman.tman_default_tiling()
    t.prefill_k_split = mode
    tman.tman_set_tiling(t)


@pytest.mark.parametrize("M,K,bits,group,hz,N", SMALL)
def test_small_shapes(oracle_lib, M, K, bits, group, hz, N):
    q, s, z, x = rand_case(3000 + M + K + bits + N, M, K, N, bits, group, hz)
    _check(tman.Shape(M, K, bits, group, hz), q, s, z, x)


# the kernel whose waves split K, forced for every call: 2 = 64 rows x 256 tokens, 3 = 128 rows x 128 tokens per workgroup
K_SPLIT_SHAPES = SMALL + [
    (130, 4128, 4, 32, True, 300),   # an odd number of row blocks, K = 129 stages (the four waves get 33, 32, 32, 32)
    (192, 2048, 2, 64, True, 129),
    (64, 6912, 1, 64, False, 257),
]


@pytest.mark.parametrize("mode", [2, 3])
@pytest.mark.parametrize("M,K,bits,group,hz,N", K_SPLIT_SHAPES)
def test_k_split_kernel_on_small_shapes(oracle_lib, restore_tiling, M, K, bits, group, hz, N, mode):
    _k_split(mode)
    q, s, z, x = rand_case(3300 + M + K + bits + N, M, K, N, bits, group, hz)
    shape = tman.Shape(M, K, bits, group, hz)
    assert tman.tman_mpgemm_splits_k(shape, max(N, 33)) == 1
    assert tman.tman_mpgemm_tile_rows(shape, max(N, 33)) == (64 if mode == 2 else 128)
    _check(shape, q, s, z, x)


def test_identity_activations_return_dequantized_weights(oracle_lib):
    """X = I (K tokens): Y is dequant(W)^T.  The kernel forms fp16((1024 + c) * s - (1024 + z) * s) in fp32
    with one rounding; against the oracle's table entry fp16((c - z) * s) that is the same value except
    where the fp32 rounding of the constant term moves a result across a rounding boundary (one fp16
    step, a few percent of the entries at most)."""
    M, K, bits, group = 96, 256, 4, 64
    q, s, z, _ = rand_case(81, M, K, 1, bits, group)
    shape = tman.Shape(M, K, bits, group)
    y16 = mpgemm(shape, pack(shape, q, s, z), np.eye(K, dtype=np.float16))
    y = y16.astype(np.float64)
    Wd = (q.astype(np.float64) - np.repeat(z.astype(np.float64), group, axis=1)) * np.repeat(s.astype(np.float64), group, axis=1)
    smax = float(s.astype(np.float64).max())
    const_err = 2.0 ** -23 * 1033.0 * smax  # fp32 rounding of the constant term (1024 + z) * s
    assert np.all(np.abs(y - Wd.T) <= 2.0 ** -11 * np.abs(Wd.T) + const_err + 1e-12)
    D = np.empty((M, K), dtype=np.float16)
    for m in range(M):
        for G in range(K // group):
            tab = oracle.dequant_table(int(s[m, G].view(np.uint16)), int(z[m, G].view(np.uint16)), bits)
            D[m, G * group:(G + 1) * group] = tab[q[m, G * group:(G + 1) * group]]
    same = (y16.T.view(np.uint16) == D.view(np.uint16))
    assert same.mean() > 0.95
    step = np.abs(y16.T.view(np.uint16).astype(np.int32) - D.view(np.uint16).astype(np.int32))
    big = np.abs(D.astype(np.float64)) > 0.25 * smax  # tiny weights (c close to z) have tiny fp16 steps
    assert step[big].max() <= 1  # neighbouring fp16 values at worst


@pytest.mark.parametrize("N", [256, 1024, 2048])
def test_full_size_prefill_sampled_tokens(oracle_lib, N):
    """11008 x 4096 uint4 g64 at the benchmarked sizes; the oracle recomputes 24 whole tokens (all 11008
    outputs each), including the first and last of the batch and of every 128-token tile boundary."""
    w = synth.WORKLOADS["prefill_w4g64"]
    spec = w.layers[0]
    q, s, z = synth.layer_tensors(w, 0, 0)
    x = synth.activation(w, 0, 0, N)
    shape = tman.Shape(spec.M, spec.K, w.bits, w.group, True)
    # 172 workgroups of one tile block at N = 256: the call goes to the kernel whose waves split K
    assert tman.tman_mpgemm_splits_k(shape, N) == (1 if N == 256 else 0)
    y = mpgemm(shape, pack(shape, q, s, z), x)
    assert np.all(np.isfinite(y.astype(np.float32)))
    rng = np.random.default_rng(N)
    rows = sorted(set([0, 1, 127, 128, N // 2, N - 129, N - 128, N - 1]) | set(rng.integers(0, N, 16).tolist()))
    Y = oracle.matmul(q, s, z, x[rows], w.bits, w.group)
    err = oracle.row_relative_error(y[rows], Y)
    assert err.max() <= TOL, f"row-normalised error {err.max():.3e}"


@pytest.mark.parametrize("mode", [1, 2, 3])
def test_full_size_256_tokens_through_every_kernel(oracle_lib, restore_tiling, mode):
    """11008 x 4096 uint4 g64, N = 256 (the grid where the three kernels compete): the tiled kernel with one tile
    block per workgroup (1) and both tiles of the K-split kernel (2, 3), 20 whole tokens each against the oracle."""
    _k_split(mode)
    N = 256
    w = synth.WORKLOADS["prefill_w4g64"]
    spec = w.layers[0]
    q, s, z = synth.layer_tensors(w, 0, 0)
    x = synth.activation(w, 0, 0, N)
    shape = tman.Shape(spec.M, spec.K, w.bits, w.group, True)
    assert tman.tman_mpgemm_splits_k(shape, N) == (0 if mode == 1 else 1)
    y = mpgemm(shape, pack(shape, q, s, z), x)
    assert np.all(np.isfinite(y.astype(np.float32)))
    rng = np.random.default_rng(mode)
    rows = sorted(set([0, 31, 32, 63, 64, 127, 128, 255]) | set(rng.integers(0, N, 12).tolist()))
    Y = oracle.matmul(q, s, z, x[rows], w.bits, w.group)
    err = oracle.row_relative_error(y[rows], Y)
    assert err.max() <= TOL, f"row-normalised error {err.max():.3e}"


@pytest.mark.parametrize("N", [256, 1024])
def test_full_size_prefill_every_token_on_row_bands(oracle_lib, N):
    """The same launch checked along the other axis: EVERY token of the batch, on three bands of 192 output rows
    (the first rows, a band across a row-tile edge in the middle, the last rows), so no token tile, wave or lane
    of the token dimension goes unchecked at full size."""
    w = synth.WORKLOADS["prefill_w4g64"]
    spec = w.layers[0]
    q, s, z = synth.layer_tensors(w, 0, 0)
    x = synth.activation(w, 0, 0, N)
    shape = tman.Shape(spec.M, spec.K, w.bits, w.group, True)
    y = mpgemm(shape, pack(shape, q, s, z), x)
    rows_per_tile = tman.tman_mpgemm_tile_rows(shape, N)
    edge = (spec.M // 2) // rows_per_tile * rows_per_tile
    for lo in (0, edge - 96, spec.M - 192):
        band = slice(lo, lo + 192)
        Y = oracle.matmul(q[band], s[band], z[band], x, w.bits, w.group)
        err = oracle.row_relative_error(y[:, band], Y)
        assert err.max() <= TOL, f"rows {lo}..{lo + 191}: row-normalised error {err.max():.3e}"


@pytest.mark.parametrize("M,rows", [(16384, 64), (32768, 128), (49152, 192), (65536, 256)])
def test_every_tile_height(oracle_lib, M, rows):
    """Row counts that make the launcher pick each of its four tile heights (the small cases above all run
    with 64 rows, the benchmark shape with 192); ragged token count, K = 12 stages so the stage ring
    wraps three times.  The oracle recomputes eight tokens in full."""
    K, bits, group, N = 384, 4, 64, 200
    shape = tman.Shape(M, K, bits, group, True)
    assert tman.tman_mpgemm_tile_rows(shape, N) == rows
    q, s, z, x = rand_case(5000 + M, M, K, N, bits, group)
    y = mpgemm(shape, pack(shape, q, s, z), x)
    assert np.all(np.isfinite(y.astype(np.float32)))
    tokens = [0, 1, 63, 64, 127, 128, 198, 199]
    Y = oracle.matmul(q, s, z, x[tokens], bits, group)
    err = oracle.row_relative_error(y[tokens], Y)
    assert err.max() <= TOL, f"row-normalised error {err.max():.3e}"


@pytest.mark.parametrize("mode", [0, 2, 3])
@pytest.mark.parametrize("poison", [float("nan"), float("inf")])
@pytest.mark.parametrize("M,K,bits,group,N", [(70, 160, 4, 32, 300), (200, 1056, 2, 32, 513), (64, 96, 1, 32, 7)])
def test_activations_and_outputs_stay_inside_their_buffers(oracle_lib, restore_tiling, poison, M, K, bits, group, N, mode):
    """X and Y are slices of tensors filled with NaN / Inf; the last token tile is ragged (N % 256 != 0) and K
    is not a multiple of the 128-column tile.  A read beyond X would reach the result as NaN, a write beyond Y
    would overwrite the filler.  For the tiled kernel and both tiles of the K-split kernel."""
    import torch
    from gpu_helpers import dev

    _k_split(mode)
    hz = bits != 1
    q, s, z, x = rand_case(4000 + M + K + N, M, K, N, bits, group, hz)
    shape = tman.Shape(M, K, bits, group, hz)
    blob = pack(shape, q, s, z)
    xbig = torch.full((512 + N * K + 70000,), poison, dtype=torch.float16, device=dev())
    xbig[512:512 + N * K] = to_dev(x).reshape(-1)
    xs = xbig[512:512 + N * K].view(N, K)
    ybig = torch.full((64 + N * M + 64,), poison, dtype=torch.float16, device=dev())
    ys = ybig[64:64 + N * M].view(N, M)
    tman.tman_mpgemm(shape, blob, xs, N, ys, None)
    torch.cuda.synchronize()
    y = ys.cpu().numpy()
    assert np.all(np.isfinite(y.astype(np.float32)))
    assert oracle.row_relative_error(y, oracle.matmul(q, s, z, x, bits, group)).max() <= TOL
    filler = torch.cat([ybig[:64], ybig[64 + N * M:]])
    assert bool(torch.isnan(filler).all() if poison != poison else torch.isinf(filler).all())


@pytest.mark.parametrize("M,rows", [(16384, 64), (32768, 128), (49152, 192), (65536, 256)])
def test_every_token_of_a_full_tile_at_every_tile_height(oracle_lib, M, rows):
    """All 256 tokens of one full token tile, for each tile height, against the oracle on the first two and the
    last workgroup's rows (every token row of the output tile that is staged through LDS in the epilogue,
    including the part of it that overlaps the stage ring's activation slots)."""
    K, bits, group, N = 256, 4, 64, 256
    shape = tman.Shape(M, K, bits, group, True)
    assert tman.tman_mpgemm_tile_rows(shape, N) == rows
    q, s, z, x = rand_case(6000 + M, M, K, N, bits, group)
    y = mpgemm(shape, pack(shape, q, s, z), x)
    assert np.all(np.isfinite(y.astype(np.float32)))
    sel = np.r_[0:2 * rows, M - rows:M]
    Y = oracle.matmul(q[sel], s[sel], z[sel], x, bits, group)
    err = oracle.row_relative_error(y[:, sel], Y)
    assert err.max() <= TOL, f"row-normalised error {err.max():.3e}"
