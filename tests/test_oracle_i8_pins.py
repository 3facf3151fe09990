"""CPU pins of the oracle's int8 routines (Sec. 6.1 / 6.2: per-tensor formats computed as W_INT8 x A_INT8): hand
values of the absmax quantizer including ties, its defining properties, the integer product against numpy's
integer matmul, and the scaled result against the (separately pinned) fp64 definition applied to the
dequantized integer activations."""
import numpy as np
import pytest

import oracle
import synth


def test_quantizer_hand_values(oracle_lib):
    x = np.array([[127, -63.5, 1.5, 2.5, 0.25, -127],      # largest 127: the numbers themselves; ties go to even
                  [0, 0, 0, 0, 0, 0],
                  [2, -1, 0.5, 0.0078125, 1, -2],           # largest 2: x * 63.5 -> 127, -63.5 (tie -> -64), 31.75 -> 32, 0.496 -> 0
                  [254, 1, -3, 5, 127, 253]], dtype=np.float16)  # largest 254: x / 2 -> 127, 0.5 (tie -> 0), -1.5 (tie -> -2), 2.5 -> 2, 63.5 -> 64, 126.5 -> 126
    xq, mx = oracle.quantize_activations_i8(x)
    assert mx.tolist() == [127.0, 0.0, 2.0, 254.0]
    assert xq[0].tolist() == [127, -64, 2, 2, 0, -127]
    assert xq[1].tolist() == [0] * 6
    assert xq[2].tolist() == [127, -64, 32, 0, 64, -127]
    assert xq[3].tolist() == [127, 0, -2, 2, 64, 126]


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_quantizer_properties(oracle_lib, seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((5, 384)) * rng.choice([1e-3, 1.0, 50.0], size=(5, 1))).astype(np.float16)
    xq, mx = oracle.quantize_activations_i8(x)
    xd = x.astype(np.float64)
    assert np.array_equal(mx.astype(np.float64), np.abs(xd).max(axis=1))
    assert np.abs(xq).max() <= 127 and np.all(np.abs(xq).max(axis=1) == 127)  # the largest activation maps to +-127
    t = xd * (127.0 / mx.astype(np.float64))[:, None]
    assert np.all(np.abs(xq - t) <= 0.5 + 1e-4)  # nearest integer, up to the binary32 evaluation of t
    assert np.all(np.sign(xq) * np.sign(xd) >= 0)


@pytest.mark.parametrize("M,K,N,bits,hz", [(24, 256, 5, 4, True), (17, 128, 3, 2, True), (9, 96, 2, 1, False), (40, 2560, 2, 2, True)])
def test_integer_product_and_scaling(oracle_lib, M, K, N, bits, hz):
    q = synth.uniform_codes(70 + M, M * K, bits).reshape(M, K)
    x = synth.normal_fp16(71 + M, N * K).reshape(N, K)
    rs = synth.uniform_fp16(72 + M, M, 0.005, 0.02)
    rz = synth.uniform_fp16(73 + M, M, 0.5, 9.0) if hz else None
    xq, mx = oracle.quantize_activations_i8(x)
    acc, Y = oracle.matmul_i8(q, rs, rz, xq, mx, bits)
    assert np.array_equal(acc, xq.astype(np.int64) @ q.astype(np.int64).T)
    # the same numbers through the definition oracle: per-row scale / zero repeated over the blocks, activations
    # dequantized to absmax / 127 * xq
    group = 32
    S = np.repeat(rs.reshape(M, 1), K // group, axis=1)
    Z = None if rz is None else np.repeat(rz.reshape(M, 1), K // group, axis=1)
    xhat = xq.astype(np.float64) * (mx.astype(np.float64) / 127.0)[:, None]
    Yd = oracle.matmul_real_x(q, S, Z, xhat, bits, group)
    assert np.all(np.abs(Y - Yd) <= 1e-12 * np.abs(Yd).max())


def test_ternary_weights_are_a_special_case(oracle_lib):
    """BitNet-style ternary weights {-1, 0, 1} * s: codes {0, 1, 2}, zero 1, one scale for the tensor."""
    M, K, N = 16, 128, 2
    t = synth.uniform_codes(5, M * K, 2).reshape(M, K) % 3
    x = synth.normal_fp16(6, N * K).reshape(N, K)
    s = np.float16(0.037)
    xq, mx = oracle.quantize_activations_i8(x)
    acc, Y = oracle.matmul_i8(t, np.full(M, s), np.full(M, np.float16(1.0)), xq, mx, 2)
    W = (t.astype(np.float64) - 1.0) * float(s)
    ref = (xq.astype(np.float64) * (mx.astype(np.float64) / 127.0)[:, None]) @ W.T
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-12)
