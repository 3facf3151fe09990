"""tman_mpgemm with a handful of tokens (N <= 32: the kernel that streams tile blocks like the decoding kernels,
dequantizes them in registers and multiplies them with all tokens on the matrix cores) and its batch form,
against the fp64 definition oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
import synth
from gpu_helpers import TOL, dev, mpgemm, pack, rand_case, to_dev

pytestmark = pytest.mark.gpu


SMALL = [
    # M, K, bits, group, has_zero, N
    (256, 512, 4, 64, True, 4),
    (256, 512, 4, 64, True, 8),
    (70, 96, 4, 32, True, 5),        # ragged rows, K below one tile
    (33, 160, 2, 32, True, 2),       # K not a multiple of the 128-column tile
    (130, 2816, 2, 64, True, 17),    # 22 K tiles: the four waves get 6, 6, 6 and 4
    (96, 1024, 4, 128, True, 32),    # every token slot of the MFMA in use
    (64, 768, 1, 64, False, 8),      # sign plane
    (64, 512, 1, 128, True, 3),      # 1-bit affine
    (64, 256, 2, 32, True, 31),
    (64, 5632, 4, 64, True, 4),      # 44 K tiles: two segments
    (130, 8320, 4, 128, True, 8),    # three segments, ragged rows
    (100, 11008, 2, 64, True, 16),   # the longest K of the benchmark shapes
    (1, 32, 4, 32, True, 2),         # degenerate: one row, one group
    (200, 1056, 2, 32, True, 1),     # one token through this kernel, K = 8.25 tiles
]


@pytest.mark.parametrize("M,K,bits,group,hz,N", SMALL)
def test_small_shapes(oracle_lib, M, K, bits, group, hz, N):
    q, s, z, x = rand_case(9000 + M + K + bits + N, M, K, N, bits, group, hz)
    shape = tman.Shape(M, K, bits, group, hz)
    assert (tman.tman_mpgemm_workspace_bytes(shape, N) > 0) == (K > 43 * 128)  # a K segment is at most 43 tiles
    y = mpgemm(shape, pack(shape, q, s, z), x)
    assert np.all(np.isfinite(y.astype(np.float32)))
    err = oracle.row_relative_error(y, oracle.matmul(q, s, z, x, bits, group))
    assert err.max() <= TOL, f"row-normalised error {err.max():.3e}"


@pytest.mark.parametrize("bits,group", [(4, 64), (2, 32), (1, 128)])
def test_unit_vector_tokens_return_dequantized_columns(oracle_lib, bits, group):
    """Token n = e_k(n): output row n is column k(n) of dequant(W), as the fp16 table entry fp16((c - z) s) up to
    the one-step tolerance of the level-2 evaluation.  A wrong column, half-wave or token mapping fails."""
    M, K = 128, 384
    q, s, z, _ = rand_case(91 + bits, M, K, 1, bits, group)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    ks = [0, 1, 7, 8, 15, 16, 31, 32, 63, 64, 127, 128, 129, 200, 255, 256, 300, 383]
    x = np.zeros((len(ks), K), dtype=np.float16)
    for n, k in enumerate(ks):
        x[n, k] = 1.0
    y = mpgemm(shape, blob, x).astype(np.float64)
    Wd = (q.astype(np.float64) - np.repeat(z.astype(np.float64), group, axis=1)) * np.repeat(s.astype(np.float64), group, axis=1)
    for n, k in enumerate(ks):
        assert np.all(np.abs(y[n] - Wd[:, k]) <= 1.2e-3 * np.abs(Wd[:, k]).max()), (n, k)


def test_deterministic_and_workspace_reusable(oracle_lib):
    M, K, bits, group, N = 512, 11008, 2, 64, 8  # two K segments of 43 tiles: exercises the ticketed reduction
    q, s, z, x = rand_case(61, M, K, N, bits, group)
    shape = tman.Shape(M, K, bits, group)
    blob = pack(shape, q, s, z)
    ws = torch.zeros(tman.tman_mpgemm_workspace_bytes(shape, N), dtype=torch.uint8, device=dev())
    xd = to_dev(x)
    ys = []
    for _ in range(3):
        y = torch.full((N, M), float("nan"), dtype=torch.float16, device=dev())
        tman.tman_mpgemm(shape, blob, xd, N, y, ws)
        torch.cuda.synchronize()
        ys.append(y.cpu().numpy())
    assert np.array_equal(ys[0].view(np.uint16), ys[1].view(np.uint16))
    assert np.array_equal(ys[0].view(np.uint16), ys[2].view(np.uint16))
    assert int(ws[: (M // 64) * 4].view(torch.int32).abs().sum().item()) == 0  # tickets back to zero
    assert oracle.row_relative_error(ys[0], oracle.matmul(q, s, z, x, bits, group)).max() <= TOL
    with pytest.raises(tman.TmanError):
        tman.tman_mpgemm(shape, blob, xd, N, y, None)  # a long K needs the workspace


@pytest.mark.parametrize("N", [4, 8])
def test_batched_layer_set_full_size(oracle_lib, N):
    """BASELINE config 2 (7B layer set, uint4 g128, 1 % outlier channels x 20) at 4 and 8 tokens, the whole layer
    set in one launch as bench.py times it: every output against the oracle, two runs bit-identical."""
    w = synth.WORKLOADS["7b_w4g128"]
    shapes, blobs, xs, ys, wss, ref = [], [], [], [], [], []
    x_of_act = {}
    for li, spec in enumerate(w.layers):
        q, s, z = synth.layer_tensors(w, 1, li)
        x = synth.activation(w, 1, li, N)
        if spec.act not in x_of_act:
            x_of_act[spec.act] = to_dev(x)
        shape = tman.Shape(spec.M, spec.K, w.bits, w.group, w.has_zero)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); xs.append(x_of_act[spec.act])
        ys.append(torch.full((N, spec.M), float("nan"), dtype=torch.float16, device=dev()))
        need = tman.tman_mpgemm_workspace_bytes(shape, N)
        wss.append(torch.zeros(need, dtype=torch.uint8, device=dev()) if need else None)
        ref.append((q, s, z, x))
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev())
    tman.tman_mpgemm_batch_prepare(shapes, blobs, xs, N, ys, wss, desc)
    tman.tman_mpgemm_batch_run(shapes, N, desc)
    torch.cuda.synchronize()
    first = [y.cpu().numpy() for y in ys]
    for y in ys:
        y.fill_(float("nan"))
    tman.tman_mpgemm_batch_run(shapes, N, desc)
    torch.cuda.synchronize()
    assert tman.tman_device_status() == 0
    for shape, y1, y, (q, s, z, x) in zip(shapes, first, ys, ref):
        assert np.array_equal(y1.view(np.uint16), y.cpu().numpy().view(np.uint16))
        err = oracle.row_relative_error(y1, oracle.matmul(q, s, z, x, w.bits, w.group)).max()
        assert err <= TOL, f"{shape}: {err:.3e}"
    # the launch above numbers its workgroups for balance (tiling.decode_balance); the plain grid gives the same bits
    saved = tman.tman_get_tiling()
    try:
        plain = tman.tman_get_tiling()
        plain.decode_balance = 0
        tman.tman_set_tiling(plain)
        for y in ys:
            y.fill_(float("nan"))
        tman.tman_mpgemm_batch_prepare(shapes, blobs, xs, N, ys, wss, desc)
        tman.tman_mpgemm_batch_run(shapes, N, desc)
        torch.cuda.synchronize()
    finally:
        tman.tman_set_tiling(saved)
    for y1, y in zip(first, ys):
        assert np.array_equal(y1.view(np.uint16), y.cpu().numpy().view(np.uint16))


def test_batch_of_mixed_small_shapes_and_a_foreign_blob(oracle_lib):
    bits, group, N = 2, 64, 6
    dims = [(70, 192), (64, 5632), (130, 8320), (1, 64), (257, 4096)]
    shapes, blobs, xs, ys, wss, refs = [], [], [], [], [], []
    for i, (M, K) in enumerate(dims):
        q, s, z, x = rand_case(950 + i, M, K, N, bits, group)
        shape = tman.Shape(M, K, bits, group)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); xs.append(to_dev(x))
        ys.append(torch.full((N, M), float("nan"), dtype=torch.float16, device=dev()))
        need = tman.tman_mpgemm_workspace_bytes(shape, N)
        wss.append(torch.zeros(need, dtype=torch.uint8, device=dev()) if need else None)
        refs.append((q, s, z, x))
    shapes[4] = tman.Shape(200, 4096, bits, group)  # declared with fewer rows than its blob was packed for
    ys[4] = torch.full((N, 200), float("nan"), dtype=torch.float16, device=dev())
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev())
    tman.tman_mpgemm_batch_prepare(shapes, blobs, xs, N, ys, wss, desc)
    assert tman.tman_device_status() == -8
    tman.tman_mpgemm_batch_run(shapes, N, desc)
    torch.cuda.synchronize()
    assert bool(torch.isnan(ys[4]).all())
    for i in range(4):
        q, s, z, x = refs[i]
        y = ys[i].cpu().numpy()
        assert oracle.row_relative_error(y, oracle.matmul(q, s, z, x, bits, group)).max() <= TOL
        assert np.array_equal(mpgemm(shapes[i], blobs[i], x).view(np.uint16), y.view(np.uint16))
