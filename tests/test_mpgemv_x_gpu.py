"""tman_mpgemv_x (one-token decode, tables built inside the lookup kernel) against the fp64 definition
oracle, element by element, and against the two-call path it replaces."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
import synth
from gpu_helpers import TOL, dev, gemv_workspace, mpgemv, mpgemv_x, pack, rand_case, to_dev

pytestmark = pytest.mark.gpu


SMALL = [
    # M, K, bits, group, has_zero
    (256, 512, 4, 64, True),       # BASELINE config 0
    (70, 96, 4, 32, True),         # ragged rows, K below one tile
    (33, 160, 2, 32, True),        # K not a multiple of the 128-column tile
    (33, 384, 2, 64, True),
    (130, 2816, 2, 64, True),      # 22 K tiles: the four waves get 6, 6, 6 and 4
    (96, 1024, 4, 128, True),
    (64, 768, 1, 64, False),       # sign plane
    (64, 512, 1, 128, True),       # 1-bit affine
    (64, 256, 2, 32, True),
    (64, 4096, 2, 64, True),       # exactly one full segment: all 1024 tables of the workgroup
    (64, 4608, 4, 64, True),       # two segments of 18 tiles
    (130, 8320, 4, 64, True),      # three segments, ragged rows
    (100, 11008, 2, 64, True),     # the longest K of the benchmark shapes
    (1, 32, 4, 32, True),          # degenerate: one row, one group
]


@pytest.mark.parametrize("M,K,bits,group,hz", SMALL)
def test_small_shapes(oracle_lib, M, K, bits, group, hz):
    q, s, z, x = rand_case(7000 + M + K + bits, M, K, 1, bits, group, hz)
    shape = tman.Shape(M, K, bits, group, hz)
    blob = pack(shape, q, s, z)
    y = mpgemv_x(shape, blob, x)
    Y = oracle.matmul(q, s, z, x, bits, group)
    assert np.all(np.isfinite(y.astype(np.float32)))
    err = oracle.row_relative_error(y, Y)
    assert err.max() <= TOL, f"row-normalised error {err.max():.3e}"
    # the two-call path uses the same tables (same rounding) and lookups; only the order of the fp32
    # additions across K may differ (other segment lengths): at most the last bit of the fp16 result
    y2 = mpgemv(shape, blob, x).astype(np.float64)
    assert oracle.row_relative_error(y, y2).max() <= 1.0e-3


def test_unit_vectors_return_dequantized_columns(oracle_lib):
    """x = e_k picks column k of dequant(W): a wrong activation, table or pattern order fails."""
    M, K, bits, group = 64, 512, 4, 64
    q, s, z, _ = rand_case(31, M, K, 1, bits, group)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    for k in (0, 1, 2, 3, 4, 31, 32, 127, 128, 255, 256, 511):
        x = np.zeros((1, K), dtype=np.float16)
        x[0, k] = 1.0
        y = mpgemv_x(shape, blob, x)[0].astype(np.float64)
        col = (q[:, k].astype(np.float64) - z[:, k // group].astype(np.float64)) * s[:, k // group].astype(np.float64)
        assert np.all(np.abs(y - col) <= 1e-3 * np.abs(col).max()), k


def test_integer_case_is_exact(oracle_lib):
    M, K, bits, group = 96, 256, 2, 64
    q = synth.uniform_codes(41, M * K, bits).reshape(M, K)
    xi = (synth.uniform_codes(42, K, 2).astype(np.int64) - 1).reshape(1, K)  # in {-1,0,1,2}
    s = np.ones((M, K // group), dtype=np.float16)
    z = np.zeros((M, K // group), dtype=np.float16)
    shape = tman.Shape(M, K, bits, group)
    y = mpgemv_x(shape, pack(shape, q, s, z), xi.astype(np.float16))
    ref = xi @ q.astype(np.int64).T
    assert np.array_equal(y.astype(np.int64), ref)


def test_deterministic_and_workspace_reusable(oracle_lib):
    M, K, bits, group = 512, 11008, 2, 64  # three K segments: exercises the ticketed reduction
    q, s, z, x = rand_case(61, M, K, 1, bits, group)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    ws = gemv_workspace(shape, 1)
    y1 = mpgemv_x(shape, blob, x, ws)
    y2 = mpgemv_x(shape, blob, x, ws)
    y3 = mpgemv_x(shape, blob, x)
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
    assert np.array_equal(y1.view(np.uint16), y3.view(np.uint16))
    assert int(ws[: (M // 64) * 4].view(torch.int32).abs().sum().item()) == 0  # tickets back to zero
    assert oracle.row_relative_error(y1, oracle.matmul(q, s, z, x, bits, group)).max() <= TOL


def _embedded(values, poison, lead=1024, tail=8192):
    """A device tensor filled with `poison` that holds `values` (fp16, 1-D) at element `lead` (16-byte aligned);
    returns (whole tensor, the slice holding the values)."""
    big = torch.full((lead + values.numel() + tail,), poison, dtype=torch.float16, device=dev())
    big[lead:lead + values.numel()] = values
    return big, big[lead:lead + values.numel()]


@pytest.mark.parametrize("poison", [float("nan"), float("inf")])
@pytest.mark.parametrize("M,K,bits,group", [
    (64, 160, 4, 32),     # one segment; the second tile's tables past column 160 must read as zero
    (130, 4672, 4, 64),   # 37 tiles -> two segments of 19; the last tile of the LAST segment is half beyond K
    (70, 11040, 2, 32),   # 87 tiles -> four segments of 22; the last has 21 tiles, the last tile a quarter used
])
def test_activations_and_outputs_stay_inside_their_buffers(oracle_lib, poison, M, K, bits, group):
    """x and y are slices of larger tensors filled with NaN (Inf): whatever the kernel reads beyond x would
    reach the result (0 * NaN is NaN: the padded groups have zero scale and zero, which hides any finite
    value), and whatever it writes beyond y would overwrite the filler.  Single call and batch form."""
    q, s, z, x = rand_case(77 + K, M, K, 1, bits, group)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    Y = oracle.matmul(q, s, z, x, bits, group)
    xbig, xs = _embedded(to_dev(x)[0], poison)
    ybig, ys = _embedded(torch.zeros(M, dtype=torch.float16, device=dev()), poison, lead=64, tail=64)
    tman.tman_mpgemv_x(shape, blob, xs, ys, gemv_workspace(shape, 1))
    torch.cuda.synchronize()
    y = ys.cpu().numpy().reshape(1, M)
    assert np.all(np.isfinite(y.astype(np.float32)))
    assert oracle.row_relative_error(y, Y).max() <= TOL
    filler = torch.cat([ybig[:64], ybig[64 + M:]])
    assert bool(torch.isnan(filler).all() if poison != poison else torch.isinf(filler).all())
    # batch form: the same GEMV twice in one launch, sharing the activation slice
    y2 = [torch.zeros((1, M), dtype=torch.float16, device=dev()) for _ in range(2)]
    wss = [gemv_workspace(shape, 1) for _ in range(2)]
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(2), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_x_batch_prepare([shape, shape], [blob, blob], [xs, xs], y2, wss, desc)
    tman.tman_mpgemv_x_batch_run([shape, shape], desc)
    torch.cuda.synchronize()
    for yy in y2:
        assert np.array_equal(yy.cpu().numpy().view(np.uint16), y.view(np.uint16))


@pytest.mark.parametrize("name", ["7b_w2g64", "7b_w4g128", "3p8b_w2g64", "3p8b_w1g64"])
def test_batched_layer_set_full_size(oracle_lib, name):
    """The whole layer set in one launch (the configuration bench.py times): every output against the
    oracle, two runs bit-identical, layers fed by one activation share its buffer."""
    w = synth.WORKLOADS[name]
    shapes, blobs, xs, ys, wss, ref = [], [], [], [], [], []
    x_of_act = {}
    for li, spec in enumerate(w.layers):
        q, s, z = synth.layer_tensors(w, 1, li)
        x = synth.activation(w, 1, li, 1)
        if spec.act not in x_of_act:
            x_of_act[spec.act] = to_dev(x)
        shape = tman.Shape(spec.M, spec.K, w.bits, w.group, w.has_zero)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); xs.append(x_of_act[spec.act])
        ys.append(torch.full((1, spec.M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, 1)); ref.append((q, s, z, x))
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_x_batch_prepare(shapes, blobs, xs, ys, wss, desc)
    tman.tman_mpgemv_x_batch_run(shapes, desc)
    torch.cuda.synchronize()
    first = [y.cpu().numpy() for y in ys]
    for y in ys:
        y.fill_(float("nan"))
    tman.tman_mpgemv_x_batch_run(shapes, desc)
    torch.cuda.synchronize()
    for shape, y1, y, (q, s, z, x), ws in zip(shapes, first, ys, ref, wss):
        assert np.array_equal(y1.view(np.uint16), y.cpu().numpy().view(np.uint16))
        err = oracle.row_relative_error(y1, oracle.matmul(q, s, z, x, w.bits, w.group)).max()
        assert err <= TOL, f"{shape}: {err:.3e}"
        assert int(ws[: -(-shape.M // 64) * 4].view(torch.int32).abs().sum().item()) == 0


@pytest.mark.parametrize("name", ["7b_w2g64", "3p8b_w1g64"])
def test_numbered_and_plain_launch_give_the_same_bits(oracle_lib, name):
    """The workgroup numbering (tiling.decode_balance) only changes which compute unit runs which workgroup:
    the outputs of a numbered launch and of the plain grid are bit-identical."""
    w = synth.WORKLOADS[name]
    shapes, blobs, xs, ys, wss = [], [], [], [], []
    x_of_act = {}
    for li, spec in enumerate(w.layers):
        q, s, z = synth.layer_tensors(w, 5, li)
        if spec.act not in x_of_act:
            x_of_act[spec.act] = to_dev(synth.activation(w, 5, li, 1))
        shape = tman.Shape(spec.M, spec.K, w.bits, w.group, w.has_zero)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); xs.append(x_of_act[spec.act])
        ys.append(torch.full((1, spec.M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, 1))
    assert tman.tman_mpgemv_x_batch_order(shapes), "expected a numbered launch on this device"
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_x_batch_prepare(shapes, blobs, xs, ys, wss, desc)
    tman.tman_mpgemv_x_batch_run(shapes, desc)
    torch.cuda.synchronize()
    numbered = [y.cpu().numpy() for y in ys]
    saved = tman.tman_get_tiling()
    try:
        plain = tman.tman_get_tiling()
        plain.decode_balance = 0
        tman.tman_set_tiling(plain)
        assert tman.tman_mpgemv_x_batch_order(shapes) == []
        for y in ys:
            y.fill_(float("nan"))
        tman.tman_mpgemv_x_batch_prepare(shapes, blobs, xs, ys, wss, desc)
        tman.tman_mpgemv_x_batch_run(shapes, desc)
        torch.cuda.synchronize()
    finally:
        tman.tman_set_tiling(saved)
    for a, y in zip(numbered, ys):
        assert np.all(np.isfinite(a.astype(np.float32)))
        assert np.array_equal(a.view(np.uint16), y.cpu().numpy().view(np.uint16))


def test_batch_of_mixed_small_shapes(oracle_lib):
    bits, group = 4, 64
    dims = [(70, 192), (64, 4608), (130, 8320), (1, 64), (257, 4096)]
    shapes, blobs, xs, ys, wss, refs = [], [], [], [], [], []
    for i, (M, K) in enumerate(dims):
        q, s, z, x = rand_case(900 + i, M, K, 1, bits, group)
        shape = tman.Shape(M, K, bits, group)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); xs.append(to_dev(x))
        ys.append(torch.full((1, M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, 1)); refs.append((q, s, z, x))
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_x_batch_prepare(shapes, blobs, xs, ys, wss, desc)
    tman.tman_mpgemv_x_batch_run(shapes, desc)
    torch.cuda.synchronize()
    for shape, y, blob, (q, s, z, x) in zip(shapes, ys, blobs, refs):
        assert oracle.row_relative_error(y.cpu().numpy(), oracle.matmul(q, s, z, x, bits, group)).max() <= TOL
        assert np.array_equal(mpgemv_x(shape, blob, x).view(np.uint16), y.cpu().numpy().view(np.uint16))


def test_largest_batch(oracle_lib):
    """TMAN_MAX_BATCH = 256 GEMVs in one launch (more than one descriptor chunk, a grid of 256 rows of
    workgroups), small ragged shapes, every output checked."""
    bits, group, count = 2, 32, 256
    shapes, blobs, xs, ys, wss, refs = [], [], [], [], [], []
    for i in range(count):
        M, K = 40 + (i * 37) % 150, 32 * (1 + i % 9)  # enough rows for the row-normalised metric
        q, s, z, x = rand_case(12000 + i, M, K, 1, bits, group)
        shape = tman.Shape(M, K, bits, group)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); xs.append(to_dev(x))
        ys.append(torch.full((1, M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, 1)); refs.append((q, s, z, x))
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(count), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_x_batch_prepare(shapes, blobs, xs, ys, wss, desc)
    tman.tman_mpgemv_x_batch_run(shapes, desc)
    torch.cuda.synchronize()
    for y, (q, s, z, x) in zip(ys, refs):
        assert oracle.row_relative_error(y.cpu().numpy(), oracle.matmul(q, s, z, x, bits, group)).max() <= TOL
