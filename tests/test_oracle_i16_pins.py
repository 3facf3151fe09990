"""CPU pins of the oracle's integer-activation routines (Sec. 6.1 A_INT16, Sec. 4.3 integer aggregation inside a
quantization block): hand values, the defining inequalities of the quantizer, the exact-integer identity between
the table-lookup route and a brute-force integer dot product, exact rationals on a tiny case."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth


def _case(seed, M, K, N, bits, group, hz=True):
    q = synth.uniform_codes(seed, M * K, bits).reshape(M, K)
    s = synth.uniform_fp16(seed + 1, M * (K // group), 0.005, 0.02).reshape(M, -1)
    z = synth.uniform_fp16(seed + 2, M * (K // group), 0.5, 9.0).reshape(M, -1) if hz else None
    x = synth.normal_fp16(seed + 3, N * K).reshape(N, K)
    return q, s, z, x


def test_quantizer_hand_values(oracle_lib):
    x = np.array([[1, -0.5, 3.75, 8188],      # largest 8188 <= 8191: step 1; -0.5 is a tie -> 0 (even), 3.75 -> 4
                  [0, 0, 0, 0],               # all zero: step 1
                  [1, 2, 3, 8192],            # 8192 > 8191: step 2; 0.5 -> 0, 1.5 -> 2 (ties to even)
                  [2.5, 1.5, -2.5, 4096],     # step 1: 2.5 -> 2, 1.5 -> 2, -2.5 -> -2
                  [0.25, -0.125, 0, 0.1875]], dtype=np.float16)  # largest 0.25 = 0.5 * 2^-1: step 2^(-1 - 13)
    xq, e = oracle.quantize_activations(x)
    assert e.tolist() == [0, 0, 1, 0, -14]
    assert xq[0].tolist() == [1, 0, 4, 8188]
    assert xq[1].tolist() == [0, 0, 0, 0]
    assert xq[2].tolist() == [0, 1, 2, 4096]
    assert xq[3].tolist() == [2, 2, -2, 4096]
    assert xq[4].tolist() == [4096, -2048, 0, 3072]  # 0.25 / 2^-14, -0.125 / 2^-14, 0.1875 / 2^-14


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_quantizer_defining_properties(oracle_lib, seed):
    """2^e is the smallest power of two with max|x| / 2^e <= 8191; xq is the nearest integer to x / 2^e."""
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((6, 512)) * rng.choice([1e-4, 0.03, 1.0, 40.0, 3000.0], size=(6, 1))).astype(np.float16)
    x[2, 7] = np.float16(65504.0)  # the largest fp16 number
    xq, e = oracle.quantize_activations(x)
    xd = x.astype(np.float64)
    for n in range(x.shape[0]):
        mx = np.abs(xd[n]).max()
        assert mx / 2.0 ** e[n] <= 8191 < mx / 2.0 ** (e[n] - 1)
        t = xd[n] / 2.0 ** e[n]
        assert np.abs(xq[n]).max() <= 8191
        assert np.all(np.abs(xq[n] - t) <= 0.5)
        ties = np.abs(np.abs(xq[n] - t) - 0.5) < 1e-12
        assert np.all(xq[n][ties] % 2 == 0)
    ints = rng.integers(-8191, 8192, size=(1, 64)).astype(np.float64)
    ints[0, 0] = 8000  # largest in (4095, 8191]: the integers themselves are the codes
    xi = ints.astype(np.float16)  # (integers above 2048 round to fp16 first)
    xq, e = oracle.quantize_activations(xi)
    assert e[0] == 0 and np.array_equal(xq[0], xi[0].astype(np.int64))


@pytest.mark.parametrize("M,K,N,bits,group,hz", [(24, 256, 3, 4, 64, True), (17, 128, 2, 2, 32, True),
                                                 (9, 384, 1, 1, 128, False), (5, 64, 4, 1, 32, True)])
def test_block_sums_are_the_integer_dot_products(oracle_lib, M, K, N, bits, group, hz):
    """Exact-integer identity of the table-lookup form: per (token, row, block)
    sum_i 2^i sum_j Tq[j][idx_i] == sum_k q[m][k] * xq[n][k], computed here by plain integer arithmetic."""
    q, s, z, x = _case(300 + M, M, K, N, bits, group, hz)
    xq, e = oracle.quantize_activations(x)
    Y, A = oracle.lut_matmul_i16(q, s, z, xq, e, bits, group, return_block_sums=True)
    G = K // group
    brute = np.einsum("mgk,ngk->nmg", q.astype(np.int64).reshape(M, G, group), xq.astype(np.int64).reshape(N, G, group))
    assert np.array_equal(A, brute)
    # and the scaled result is the definition applied to the dequantized activations
    xhat = xq.astype(np.float64) * (2.0 ** e.astype(np.float64))[:, None]
    Yd = oracle.matmul_real_x(q, s, z, xhat, bits, group)
    assert np.all(np.abs(Y - Yd) <= 1e-12 * np.abs(Yd).max())


def test_tiny_case_in_exact_rationals(oracle_lib):
    M, K, N, bits, group = 3, 32, 2, 4, 32
    q, s, z, x = _case(77, M, K, N, bits, group)
    xq, e = oracle.quantize_activations(x)
    Y = oracle.lut_matmul_i16(q, s, z, xq, e, bits, group)
    for n in range(N):
        for m in range(M):
            acc = Fraction(0)
            for k in range(K):
                w = (Fraction(int(q[m, k])) - Fraction(float(z[m, 0]))) * Fraction(float(s[m, 0]))
                acc += w * Fraction(int(xq[n, k])) * Fraction(2) ** int(e[n])
            assert abs(Y[n, m] - float(acc)) <= 1e-13 * max(1.0, abs(float(acc)))


def test_real_x_definition_agrees_with_the_fp16_definition(oracle_lib):
    """matmul_real_x is the same sum as matmul when the activations happen to be fp16 numbers."""
    q, s, z, x = _case(5, 33, 192, 3, 2, 64)
    assert np.array_equal(oracle.matmul_real_x(q, s, z, x.astype(np.float64), 2, 64), oracle.matmul(q, s, z, x, 2, 64))
    qs, ss, _, xs = _case(6, 12, 128, 2, 1, 64, hz=False)
    assert np.array_equal(oracle.matmul_real_x(qs, ss, None, xs.astype(np.float64), 1, 64), oracle.matmul(qs, ss, None, xs, 1, 64))


def test_integer_activations_stay_close_to_the_fp16_ones(oracle_lib):
    """14-bit steps relative to the token's largest activation: the result moves by a small fraction of its rms."""
    q, s, z, x = _case(9, 64, 1024, 2, 4, 128)
    xq, e = oracle.quantize_activations(x)
    Y16 = oracle.lut_matmul_i16(q, s, z, xq, e, 4, 128)
    Y = oracle.matmul(q, s, z, x, 4, 128)
    assert np.abs(Y16 - Y).max() <= 1e-3 * np.sqrt(np.mean(Y * Y))
