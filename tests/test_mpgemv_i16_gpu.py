"""Integer activations / integer tables (tman_build_lut_i16, tman_mpgemv_i16) against the CPU oracle: the table
buffer bit for bit (integers), the outputs against the fp64 result for the dequantized integer activations.
Tolerance: the integer path has no table rounding at all; what is left is the fp32 sum across blocks and the
fp16 rounding of the output (half a unit in the last place = 4.9e-4 relative), so 1e-3 under the row-normalised
metric, half of what the fp16-table path is allowed."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
import synth
from gpu_helpers import dev, gemv_workspace, pack, rand_case, to_dev

pytestmark = pytest.mark.gpu
TOL_I16 = 1e-3


def _tables(x, group, poison=0x5A):
    xd = x if torch.is_tensor(x) else to_dev(x)
    N, K = xd.shape
    lut = torch.empty(tman.tman_lut_i16_bytes(N, K, group), dtype=torch.uint8, device=dev())
    lut.fill_(poison)
    tman.tman_build_lut_i16(xd, N, K, group, lut)
    return lut


def _decode_buffer(buf, N, K, group):
    """Documented layout: int16 entry (n, j, p) at element (j * 16 + p) * NP + n (tokens padded to NP = 1, 2, 4, 8,
    K to whole 128-column tiles), int32 block sums at element G * NP + n behind them, then int32 e[n]."""
    NP = 1 if N == 1 else 2 if N == 2 else 4 if N <= 4 else 8
    nkt = -(-K // 128)
    t_bytes = nkt * 1024 * NP
    T = buf[:t_bytes].view(np.int16).reshape(nkt * 32, 16, NP).transpose(2, 0, 1)
    gp = nkt * (128 // group)
    S = buf[t_bytes:t_bytes + gp * NP * 4].view(np.int32).reshape(gp, NP).T
    e = buf[t_bytes + gp * NP * 4:t_bytes + gp * NP * 4 + NP * 4].view(np.int32)
    return T, S, e, NP


@pytest.mark.parametrize("N,K,group,gain", [(1, 512, 64, 1.0), (3, 160, 32, 1.0), (8, 4096, 128, 1.0), (2, 384, 64, 300.0),
                                            (5, 1024, 128, 1e-3), (4, 11008, 64, 1.0)])
def test_integer_tables_are_exact(oracle_lib, N, K, group, gain):
    x = (synth.normal_fp16(500 + N + K, N * K).astype(np.float64) * gain).astype(np.float16).reshape(N, K)
    if N > 1:
        x[1, :] = 0  # a token of zeros
    buf = _tables(x, group).cpu().numpy()
    T, S, e, NP = _decode_buffer(buf, N, K, group)
    xq, eo = oracle.quantize_activations(x)
    assert np.array_equal(e[:N], eo) and not e[N:].any()
    # the oracle's tables: exact sums of the integer activations
    xq4 = xq.astype(np.int64).reshape(N, K // 4, 4)
    pat = ((np.arange(16)[:, None] >> np.arange(4)[None, :]) & 1).astype(np.int64)  # [p][t]
    Tq = np.einsum("njt,pt->njp", xq4, pat)
    assert np.array_equal(T[:N, : K // 4, :], Tq)
    assert not T[N:].any() and not T[:, K // 4:, :].any()  # padding tokens and columns are zero
    assert np.array_equal(S[:N, : K // group], xq.astype(np.int64).reshape(N, K // group, group).sum(axis=2))
    assert not S[N:].any() and not S[:, K // group:].any()


SMALL = [
    # M, K, bits, group, has_zero, N
    (256, 512, 4, 64, True, 1),
    (70, 96, 4, 32, True, 1),
    (33, 384, 2, 64, True, 2),
    (130, 2816, 2, 64, True, 3),
    (96, 1024, 4, 128, True, 4),
    (64, 768, 1, 64, False, 5),
    (64, 512, 1, 128, True, 8),
    (200, 1024, 4, 128, True, 8),
    (64, 4608, 4, 64, True, 1),      # two K segments
    (130, 8320, 2, 32, True, 4),     # several segments, ragged rows
    (1, 32, 4, 32, True, 1),
]


@pytest.mark.parametrize("M,K,bits,group,hz,N", SMALL)
def test_small_shapes(oracle_lib, M, K, bits, group, hz, N):
    q, s, z, x = rand_case(8000 + M + K + bits + N, M, K, N, bits, group, hz)
    shape = tman.Shape(M, K, bits, group, hz)
    blob = pack(shape, q, s, z)
    lut = _tables(x, group)
    y = torch.full((N, M), float("nan"), dtype=torch.float16, device=dev())
    tman.tman_mpgemv_i16(shape, blob, lut, N, y, gemv_workspace(shape, N))
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    assert np.all(np.isfinite(y.astype(np.float32)))
    xq, e = oracle.quantize_activations(x)
    Y = oracle.lut_matmul_i16(q, s, z, xq, e, bits, group)
    err = oracle.row_relative_error(y, Y)
    assert err.max() <= TOL_I16, f"row-normalised error {err.max():.3e}"


def test_integer_case_is_exact(oracle_lib):
    """scale = 1, zero = 0, integer activations with the largest in (4095, 8191] (step 1): the result is the
    integer product, exactly, where it is an fp16 number."""
    M, K, bits, group = 96, 256, 2, 64
    q = synth.uniform_codes(41, M * K, bits).reshape(M, K)
    xi = (synth.uniform_codes(42, K, 2).astype(np.int64) - 1).reshape(1, K)  # in {-1, 0, 1, 2}
    s = np.full((M, K // group), 2.0 ** -14, dtype=np.float16)  # keeps the outputs inside the fp16 integers
    z = np.zeros((M, K // group), dtype=np.float16)
    x = (xi * 4096).astype(np.float16)  # largest magnitude 8192 -> step 2: codes xi * 2048
    shape = tman.Shape(M, K, bits, group)
    y = torch.empty((1, M), dtype=torch.float16, device=dev())
    tman.tman_mpgemv_i16(shape, pack(shape, q, s, z), _tables(x, group), 1, y, gemv_workspace(shape, 1))
    torch.cuda.synchronize()
    ref = (xi @ q.astype(np.int64).T) * 4096 * 2.0 ** -14
    assert np.array_equal(y.cpu().numpy().astype(np.float64), ref.astype(np.float64))


@pytest.mark.parametrize("N", [1, 8])
def test_batched_layer_set_full_size(oracle_lib, N):
    """BASELINE config 2 (7B layer set, uint4 g128, outlier channels x 20) through integer tables, one table launch
    and one lookup launch for the layer set: every output against the oracle for the integer activations."""
    w = synth.WORKLOADS["7b_w4g128"]
    shapes, blobs, xs, luts, ys, wss, ref = [], [], [], [], [], [], []
    lut_of_act, x_of_act = {}, {}
    for li, spec in enumerate(w.layers):
        q, s, z = synth.layer_tensors(w, 2, li)
        x = synth.activation(w, 2, li, N)
        if spec.act not in lut_of_act:
            x_of_act[spec.act] = to_dev(x)
            lut_of_act[spec.act] = torch.empty(tman.tman_lut_i16_bytes(N, spec.K, w.group), dtype=torch.uint8, device=dev())
        shape = tman.Shape(spec.M, spec.K, w.bits, w.group, w.has_zero)
        shapes.append(shape); blobs.append(pack(shape, q, s, z)); luts.append(lut_of_act[spec.act])
        ys.append(torch.full((N, spec.M), float("nan"), dtype=torch.float16, device=dev()))
        wss.append(gemv_workspace(shape, N)); ref.append((q, s, z, x))
    acts = list(lut_of_act)
    Ks = [x_of_act[a].shape[1] for a in acts]
    tman.tman_build_lut_i16_batch([x_of_act[a] for a in acts], N, Ks, w.group, [lut_of_act[a] for a in acts])
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev())
    tman.tman_mpgemv_batch_prepare(shapes, blobs, luts, N, ys, wss, desc)
    tman.tman_mpgemv_i16_batch_run(shapes, N, desc)
    torch.cuda.synchronize()
    for shape, y, (q, s, z, x) in zip(shapes, ys, ref):
        xq, e = oracle.quantize_activations(x)
        err = oracle.row_relative_error(y.cpu().numpy(), oracle.lut_matmul_i16(q, s, z, xq, e, w.bits, w.group)).max()
        assert err <= TOL_I16, f"{shape}: {err:.3e}"
