"""tman_quantize_act_i8 / tman_mpgemm_i8 (weights with one scale and zero per row on the integer matrix cores)
against the CPU oracle: the integer activations and the integer accumulators bit for bit, the fp16 outputs
within 1e-3 (row-normalised) of the fp64 result for the same integers -- what is left after exact integer
accumulation is the fp32 scaling and the fp16 rounding of the output (4.9e-4 relative)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
import synth
from gpu_helpers import dev, pack, to_dev

pytestmark = pytest.mark.gpu
TOL_I8 = 1e-3
SIGMA = np.array([8 * (p & 3) + 4 * ((p >> 2) & 1) + (p >> 3) for p in range(32)])  # byte p of a group holds column SIGMA[p]


def _case(seed, M, K, N, bits, hz, group):
    q = synth.uniform_codes(seed, M * K, bits).reshape(M, K)
    rs = synth.uniform_fp16(seed + 1, M, 0.005, 0.02)
    rz = synth.uniform_fp16(seed + 2, M, 0.0, float((1 << bits) - 1)) if hz else None
    x = synth.normal_fp16(seed + 3, N * K).reshape(N, K)
    s = np.repeat(rs.reshape(M, 1), K // group, axis=1)
    z = None if rz is None else np.repeat(rz.reshape(M, 1), K // group, axis=1)
    return q, rs, rz, s, z, x


def _quantize(x, misalign=False):
    N, K = x.shape
    buf = torch.empty(tman.tman_act_i8_bytes(N, K), dtype=torch.uint8, device=dev())
    buf.fill_(0x5A)
    xd = to_dev(x)
    if misalign:  # the activations start 2 bytes past a 16-byte boundary: the kernel without wide loads
        big = torch.empty(N * K + 8, dtype=torch.float16, device=dev())
        big[1:1 + N * K] = xd.reshape(-1)
        xd = big[1:1 + N * K].view(N, K)
        assert xd.data_ptr() % 16 == 2
    tman.tman_quantize_act_i8(xd, N, K, buf)
    return buf


def _read_buffer(buf, N, K):
    b = buf.cpu().numpy()
    qb = (N * K + 255) // 256 * 256
    nb = (N * 4 + 255) // 256 * 256
    perm = b[: N * K].view(np.int8).reshape(N, K // 32, 32)
    xq = np.empty_like(perm)
    xq[:, :, SIGMA] = perm  # undo the per-group permutation
    return xq.reshape(N, K), b[qb:qb + N * 4].view(np.float32), b[qb + nb:qb + nb + N * 4].view(np.int32)


@pytest.mark.parametrize("misalign", [False, True])
@pytest.mark.parametrize("N,K,gain", [(1, 32, 1.0), (5, 2560, 1.0), (130, 6912, 1.0), (3, 96, 200.0), (4, 512, 1e-3),
                                      (3, 8192 + 96, 1.0)])  # more than 256 groups of 32 columns per token
def test_quantizer_matches_the_oracle_bit_for_bit(oracle_lib, N, K, gain, misalign):
    x = (synth.normal_fp16(40 + N + K, N * K).astype(np.float64) * gain).astype(np.float16).reshape(N, K)
    if N > 2:
        x[2, :] = 0
        x[1, :8] = [127, -63.5, 1.5, 2.5, 0.25, -127, 0.5, -0.5]  # exact ties when the token's largest is 127
        x[1, 8:] = np.clip(x[1, 8:], -100, 100)
    xq, mx, sums = _read_buffer(_quantize(x, misalign), N, K)
    xo, mo = oracle.quantize_activations_i8(x)
    assert np.array_equal(mx, mo)
    assert np.array_equal(xq, xo)
    assert np.array_equal(sums, xo.astype(np.int64).sum(axis=1))


SHAPES = [
    # M, K, bits, has_zero, group, N
    (2560, 2560, 2, True, 64, 128),     # BitNet-2B shapes (Sec. 6.1), ternary-like 2-bit
    (6912, 2560, 2, True, 64, 64),
    (2560, 6912, 2, True, 128, 200),    # ragged token tile
    (256, 512, 4, True, 64, 128),
    (70, 96, 4, True, 32, 37),          # ragged everywhere, K = 1.5 stages
    (130, 1056, 2, True, 32, 260),
    (64, 768, 1, False, 64, 5),         # sign plane
    (64, 512, 1, True, 128, 33),        # 1-bit affine
    (1, 32, 4, True, 32, 1),
]


@pytest.fixture
def restore_tiling():
    yield
    tman.tman_set_tiling(tman.tman_default_tiling())


def _force(blocks):
    t = tman.tman_default_tiling()
    t.i8_token_blocks = blocks
    tman.tman_set_tiling(t)


# 1: the kernel with 128 x 128 tiles; 3, 4, 7: the kernel that dequantizes in registers, 96 / 128 / 224 tokens per workgroup;
# 9: the kernel whose waves split K, 128 rows x 128 tokens per workgroup
@pytest.mark.parametrize("blocks", [1, 3, 4, 7, 9])
@pytest.mark.parametrize("M,K,bits,hz,group,N", SHAPES)
def test_accumulators_are_exact_and_outputs_close(oracle_lib, restore_tiling, M, K, bits, hz, group, N, blocks):
    _force(blocks)
    q, rs, rz, s, z, x = _case(600 + M + K + N, M, K, N, bits, hz, group)
    shape = tman.Shape(M, K, bits, group, hz)
    blob = pack(shape, q, s, z)
    xbuf = _quantize(x)
    y = torch.full((N, M), float("nan"), dtype=torch.float16, device=dev())
    acc = torch.full((N, M), -1, dtype=torch.int32, device=dev())
    tman.tman_mpgemm_i8(shape, blob, xbuf, N, y, acc)
    torch.cuda.synchronize()
    assert tman.tman_device_status() == 0
    xq, mx = oracle.quantize_activations_i8(x)
    acc_o, Y = oracle.matmul_i8(q, rs, rz, xq, mx, bits)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_o)
    yh = y.cpu().numpy()
    assert np.all(np.isfinite(yh.astype(np.float32)))
    err = oracle.row_relative_error(yh, Y)
    assert err.max() <= TOL_I8, f"row-normalised error {err.max():.3e}"
    # without the accumulator output the result is the same
    y2 = torch.full((N, M), float("nan"), dtype=torch.float16, device=dev())
    tman.tman_mpgemm_i8(shape, blob, xbuf, N, y2, None)
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy().view(np.uint16), yh.view(np.uint16))


def test_ternary_per_tensor_weights(oracle_lib):
    """BitNet-style: {-1, 0, 1} * s with ONE scale for the tensor, stored as 2-bit codes with zero 1."""
    M, K, N, group = 2560, 2560, 96, 64
    t = (synth.uniform_codes(5, M * K, 2).reshape(M, K) % 3).astype(np.uint8)
    x = synth.normal_fp16(6, N * K).reshape(N, K)
    sc = np.float16(0.037)
    s = np.full((M, K // group), sc, dtype=np.float16)
    z = np.ones((M, K // group), dtype=np.float16)
    shape = tman.Shape(M, K, 2, group, True)
    y = torch.empty((N, M), dtype=torch.float16, device=dev())
    tman.tman_mpgemm_i8(shape, pack(shape, t, s, z), _quantize(x), N, y, None)
    torch.cuda.synchronize()
    xq, mx = oracle.quantize_activations_i8(x)
    _, Y = oracle.matmul_i8(t, np.full(M, sc), np.ones(M, np.float16), xq, mx, 2)
    assert oracle.row_relative_error(y.cpu().numpy(), Y).max() <= TOL_I8
    # and the int8 activations keep the result close to the fp16-activation product (8-bit steps: about 1 %)
    Yf = oracle.matmul(t, s, z, x, 2, group)
    assert np.abs(Y - Yf).max() <= 0.05 * np.sqrt(np.mean(Yf * Yf))


def test_every_kernel_gives_the_same_bits_at_full_size(oracle_lib, restore_tiling):
    """11008 x 4096 uint4 with one scale and zero per row, N = 1000 (a ragged last token tile for every tile width):
    the kernel chosen for the call against the oracle on sampled whole tokens, and every other kernel against it
    bit for bit (the integer accumulators are exact and the epilogue is the same arithmetic)."""
    M, K, bits, group, N = 11008, 4096, 4, 64, 1000
    q, rs, rz, s, z, x = _case(77, M, K, N, bits, True, group)
    shape = tman.Shape(M, K, bits, group, True)
    blob = pack(shape, q, s, z)
    xbuf = _quantize(x)
    assert tman.tman_mpgemm_i8_token_blocks(shape, N) in (3, 4, 7)
    y = torch.full((N, M), float("nan"), dtype=torch.float16, device=dev())
    tman.tman_mpgemm_i8(shape, blob, xbuf, N, y, None)
    torch.cuda.synchronize()
    assert tman.tman_device_status() == 0
    yh = y.cpu().numpy()
    assert np.all(np.isfinite(yh.astype(np.float32)))
    tokens = sorted({0, 95, 96, 127, 128, 223, 224, 255, 256, 671, 672, 895, 896, 959, 960, 991, 992, 999})
    xq, mx = oracle.quantize_activations_i8(x[tokens])
    _, Y = oracle.matmul_i8(q, rs, rz, xq, mx, bits)
    err = oracle.row_relative_error(yh[tokens], Y)
    assert err.max() <= TOL_I8, f"row-normalised error {err.max():.3e}"
    for blocks in (1, 3, 4, 7, 9):
        _force(blocks)
        y2 = torch.full((N, M), float("nan"), dtype=torch.float16, device=dev())
        tman.tman_mpgemm_i8(shape, blob, xbuf, N, y2, None)
        torch.cuda.synchronize()
        assert np.array_equal(y2.cpu().numpy().view(np.uint16), yh.view(np.uint16)), blocks
