"""tman_mpgemv (decode, table lookup) against the fp64 definition oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
import synth
from gpu_helpers import TOL, dev, gemv_workspace, mpgemv, pack, rand_case, to_dev

pytestmark = pytest.mark.gpu


def _check(shape, q, s, z, x, tol=TOL):
    blob = pack(shape, q, s, z)
    y = mpgemv(shape, blob, x)
    Y = oracle.matmul(q, s, z, x, shape.bits, shape.group)
    assert y.shape == Y.shape
    assert np.all(np.isfinite(y.astype(np.float32)))
    err = oracle.row_relative_error(y, Y)
    assert err.max() <= tol, f"row-normalised error {err.max():.3e} > {tol}"
    return y


SMALL = [
    # M, K, bits, group, has_zero, N
    (256, 512, 4, 64, True, 1),      # BASELINE config 0
    (70, 96, 4, 32, True, 1),        # ragged rows, K < one tile
    (33, 384, 2, 64, True, 1),
    (130, 2816, 2, 64, True, 1),     # 11 K tiles (odd), rows over 5 row blocks
    (96, 1024, 4, 128, True, 1),
    (64, 768, 1, 64, False, 1),      # sign plane
    (64, 512, 1, 128, True, 1),      # 1-bit affine
    (64, 256, 2, 32, True, 1),
    (200, 1024, 4, 128, True, 4),
    (200, 1024, 4, 128, True, 8),
    (100, 512, 2, 64, True, 2),
    (100, 512, 2, 64, True, 3),      # padded to 4 tokens
    (100, 768, 1, 64, False, 5),     # padded to 8
    (64, 512, 4, 32, True, 7),
    (1, 32, 4, 32, True, 1),         # degenerate: one row, one group
]


@pytest.mark.parametrize("M,K,bits,group,hz,N", SMALL)
def test_small_shapes(oracle_lib, M, K, bits, group, hz, N):
    q, s, z, x = rand_case(2000 + M + K + bits + N, M, K, N, bits, group, hz)
    _check(tman.Shape(M, K, bits, group, hz), q, s, z, x)


def test_unit_vectors_return_dequantized_columns(oracle_lib):
    """x = e_k picks column k of dequant(W); any k or m permutation in the layout or the kernel fails."""
    M, K, bits, group = 64, 512, 4, 64
    q, s, z, _ = rand_case(31, M, K, 1, bits, group)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    for k in (0, 3, 4, 31, 32, 127, 128, 255, 256, 511):
        x = np.zeros((1, K), dtype=np.float16)
        x[0, k] = 1.0
        y = mpgemv(shape, blob, x)[0].astype(np.float64)
        col = (q[:, k].astype(np.float64) - z[:, k // group].astype(np.float64)) * s[:, k // group].astype(np.float64)
        assert np.all(np.abs(y - col) <= 1e-3 * np.abs(col).max())


def test_integer_case_is_exact(oracle_lib):
    """zero = 0, scale = 1, small integer activations: every intermediate is an exactly representable
    integer, so the result must equal the integer product."""
    M, K, bits, group = 96, 256, 2, 64
    q = synth.uniform_codes(41, M * K, bits).reshape(M, K)
    xi = (synth.uniform_codes(42, K, 2).astype(np.int64) - 1).reshape(1, K)  # in {-1,0,1,2}
    s = np.ones((M, K // group), dtype=np.float16)
    z = np.zeros((M, K // group), dtype=np.float16)
    shape = tman.Shape(M, K, bits, group)
    y = mpgemv(shape, pack(shape, q, s, z), xi.astype(np.float16))
    ref = xi @ q.astype(np.int64).T
    assert np.abs(ref).max() < 2048
    assert np.array_equal(y.astype(np.int64), ref)


def test_all_zero_and_all_max_codes(oracle_lib):
    M, K, bits, group = 64, 512, 4, 64
    _, s, z, x = rand_case(51, M, K, 2, bits, group)
    shape = tman.Shape(M, K, bits, group)
    for fill in (0, 15):
        q = np.full((M, K), fill, dtype=np.uint8)
        _check(shape, q, s, z, x)


def test_deterministic_and_workspace_reusable(oracle_lib):
    M, K, bits, group = 4096, 4096, 2, 64  # split over several K slices: exercises the ticketed reduction
    q, s, z, x = rand_case(61, 128, K, 1, bits, group)
    q = np.tile(q, (M // 128, 1)); s = np.tile(s, (M // 128, 1)); z = np.tile(z, (M // 128, 1))
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    ws = gemv_workspace(shape, 1)
    y1 = mpgemv(shape, blob, x, ws)
    y2 = mpgemv(shape, blob, x, ws)   # same workspace again: the call must have left it ready
    y3 = mpgemv(shape, blob, x)
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
    assert np.array_equal(y1.view(np.uint16), y3.view(np.uint16))
    assert np.array_equal(y1[0, :128].view(np.uint16), y1[0, 128:256].view(np.uint16))  # repeated rows agree
    assert int(ws[: (M // 128) * 4].view(torch.int32).abs().sum().item()) == 0  # tickets back to zero
    Y = oracle.matmul(q[:128], s[:128], z[:128], x, bits, group)
    assert oracle.row_relative_error(y1[:, :128], Y).max() <= TOL


def test_shared_table_serves_several_layers(oracle_lib):
    """One tman_build_lut result feeds several GEMVs with the same K (Sec. 5 graph optimization)."""
    K, bits, group, N = 1024, 4, 64, 2
    x = synth.normal_fp16(71, N * K).reshape(N, K)
    xd = to_dev(x)
    lut = torch.empty(tman.tman_lut_bytes(N, K, group), dtype=torch.uint8, device=dev())
    tman.tman_build_lut(xd, N, K, group, lut)
    for M, seed in ((96, 72), (160, 73), (33, 74)):
        q, s, z, _ = rand_case(seed, M, K, 1, bits, group)
        shape = tman.Shape(M, K, bits, group)
        blob = pack(shape, q, s, z)
        y = torch.empty((N, M), dtype=torch.float16, device=dev())
        tman.tman_mpgemv(shape, blob, lut, N, y, gemv_workspace(shape, N))
        torch.cuda.synchronize()
        Y = oracle.matmul(q, s, z, x, bits, group)
        assert oracle.row_relative_error(y.cpu().numpy(), Y).max() <= TOL


FULL = [
    ("7b_w2g64", 1), ("7b_w4g128", 1), ("7b_w4g128", 4), ("7b_w4g128", 8), ("3p8b_w2g64", 1), ("3p8b_w1g64", 1),
]


@pytest.mark.parametrize("name,N", FULL)
def test_full_size_layer_sets(oracle_lib, name, N):
    """Every layer of the benchmark workloads at full size, all outputs, launch configuration as benchmarked."""
    w = synth.WORKLOADS[name]
    for li, spec in enumerate(w.layers):
        q, s, z = synth.layer_tensors(w, 0, li)
        x = synth.activation(w, 0, li, N)
        shape = tman.Shape(spec.M, spec.K, w.bits, w.group, w.has_zero)
        print(f"{name} layer {spec.name} {spec.M}x{spec.K} N={N}", flush=True)
        _check(shape, q, s, z, x)


def _run_batch(w, instance, N, layer_ids):
    """One tman_mpgemv_batch launch over the given layers of a workload; returns (outputs, oracle inputs)."""
    shapes, blobs, luts, ys, wss, ref = [], [], [], [], [], []
    lut_of_act = {}
    for li in layer_ids:
        spec = w.layers[li]
        q, s, z = synth.layer_tensors(w, instance, li)
        x = synth.activation(w, instance, li, N)
        shape = tman.Shape(spec.M, spec.K, w.bits, w.group, w.has_zero)
        if spec.act not in lut_of_act:
            xd = to_dev(x)
            lut = torch.empty(tman.tman_lut_bytes(N, spec.K, w.group), dtype=torch.uint8, device=dev())
            tman.tman_build_lut(xd, N, spec.K, w.group, lut)
            lut_of_act[spec.act] = lut
        shapes.append(shape)
        blobs.append(pack(shape, q, s, z))
        luts.append(lut_of_act[spec.act])
        ys.append(torch.full((N, spec.M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, N))
        ref.append((q, s, z, x))
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_batch_prepare(shapes, blobs, luts, N, ys, wss, desc)
    tman.tman_mpgemv_batch_run(shapes, N, desc)
    torch.cuda.synchronize()
    first = [y.cpu().numpy() for y in ys]
    for y in ys:
        y.fill_(float("nan"))
    tman.tman_mpgemv_batch_run(shapes, N, desc)  # the table and the workspaces are reusable
    torch.cuda.synchronize()
    second = [y.cpu().numpy() for y in ys]
    return shapes, first, second, ref, wss


@pytest.mark.parametrize("name,N", [("7b_w2g64", 1), ("7b_w4g128", 4), ("3p8b_w1g64", 1)])
def test_batched_layer_set_full_size(oracle_lib, name, N):
    """The whole layer set in one launch (the configuration bench.py times): every output against the
    oracle, two runs bit-identical, tickets left at zero."""
    w = synth.WORKLOADS[name]
    shapes, first, second, ref, wss = _run_batch(w, 1, N, list(range(len(w.layers))))
    for shape, y1, y2, (q, s, z, x), ws in zip(shapes, first, second, ref, wss):
        assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
        Y = oracle.matmul(q, s, z, x, w.bits, w.group)
        err = oracle.row_relative_error(y1, Y).max()
        assert err <= TOL, f"{shape}: {err:.3e}"
        n_rb = -(-shape.M // 64)
        assert int(ws[: n_rb * 4].view(torch.int32).abs().sum().item()) == 0


def test_batch_of_mixed_small_shapes(oracle_lib):
    """Ragged M, K below one segment and K over several segments in one launch."""
    N, bits, group = 2, 4, 64
    dims = [(70, 192), (64, 4608), (130, 8320), (1, 64), (257, 4096)]
    shapes, blobs, luts, ys, wss, refs = [], [], [], [], [], []
    for i, (M, K) in enumerate(dims):
        q, s, z, x = rand_case(900 + i, M, K, N, bits, group)
        shape = tman.Shape(M, K, bits, group)
        lut = torch.empty(tman.tman_lut_bytes(N, K, group), dtype=torch.uint8, device=dev())
        tman.tman_build_lut(to_dev(x), N, K, group, lut)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); luts.append(lut)
        ys.append(torch.full((N, M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, N)); refs.append((q, s, z, x))
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_batch_prepare(shapes, blobs, luts, N, ys, wss, desc)
    tman.tman_mpgemv_batch_run(shapes, N, desc)
    torch.cuda.synchronize()
    for shape, y, blob, (q, s, z, x) in zip(shapes, ys, blobs, refs):
        Y = oracle.matmul(q, s, z, x, bits, group)
        assert oracle.row_relative_error(y.cpu().numpy(), Y).max() <= TOL
        single = mpgemv(shape, blob, x)
        assert np.array_equal(single.view(np.uint16), y.cpu().numpy().view(np.uint16))  # same schedule, same bits


def test_largest_batch(oracle_lib):
    """TMAN_MAX_BATCH = 256 GEMVs in one launch, small ragged shapes, three tokens, every output checked."""
    N, bits, group, count = 3, 4, 32, 256
    shapes, blobs, luts, ys, wss, refs = [], [], [], [], [], []
    for i in range(count):
        M, K = 40 + (i * 41) % 140, 32 * (1 + i % 7)  # enough rows for the row-normalised metric
        q, s, z, x = rand_case(15000 + i, M, K, N, bits, group)
        shape = tman.Shape(M, K, bits, group)
        lut = torch.empty(tman.tman_lut_bytes(N, K, group), dtype=torch.uint8, device=dev())
        tman.tman_build_lut(to_dev(x), N, K, group, lut)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); luts.append(lut)
        ys.append(torch.full((N, M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, N)); refs.append((q, s, z, x))
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(count), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_batch_prepare(shapes, blobs, luts, N, ys, wss, desc)
    tman.tman_mpgemv_batch_run(shapes, N, desc)
    torch.cuda.synchronize()
    for y, (q, s, z, x) in zip(ys, refs):
        assert oracle.row_relative_error(y.cpu().numpy(), oracle.matmul(q, s, z, x, bits, group)).max() <= TOL


@pytest.mark.parametrize("poison", [float("nan"), float("inf")])
@pytest.mark.parametrize("M,K,bits,group,N", [(70, 160, 4, 32, 3), (130, 4672, 4, 64, 1), (64, 4000, 2, 32, 8)])
def test_activations_and_outputs_stay_inside_their_buffers(oracle_lib, poison, M, K, bits, group, N):
    """x (read by tman_build_lut) and y (written by tman_mpgemv) are slices of tensors filled with NaN / Inf.
    A read beyond x reaches the result (the padded groups have zero scale and zero, which hides finite
    values but not 0 * NaN); a write beyond y overwrites the filler.  Ragged K, tokens padded to 4 / 8."""
    q, s, z, x = rand_case(88 + K, M, K, N, bits, group)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    xbig = torch.full((1024 + N * K + 8192,), poison, dtype=torch.float16, device=dev())
    xbig[1024:1024 + N * K] = to_dev(x).reshape(-1)
    xs = xbig[1024:1024 + N * K].view(N, K)
    ybig = torch.full((64 + N * M + 64,), poison, dtype=torch.float16, device=dev())
    ys = ybig[64:64 + N * M].view(N, M)
    lut = torch.empty(tman.tman_lut_bytes(N, K, group), dtype=torch.uint8, device=dev())
    tman.tman_build_lut(xs, N, K, group, lut)
    tman.tman_mpgemv(shape, blob, lut, N, ys, gemv_workspace(shape, N))
    torch.cuda.synchronize()
    y = ys.cpu().numpy()
    assert np.all(np.isfinite(y.astype(np.float32)))
    assert oracle.row_relative_error(y, oracle.matmul(q, s, z, x, bits, group)).max() <= TOL
    filler = torch.cat([ybig[:64], ybig[64 + N * M:]])
    assert bool(torch.isnan(filler).all() if poison != poison else torch.isinf(filler).all())
