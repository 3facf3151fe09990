"""Pins for the CPU oracle: each oracle routine is checked against something other than itself --
exact rational brute force, closed forms, special cases that reduce to a library routine, and the
values the paper prints.  No GPU needed."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


def _frac_half(v) -> Fraction:
    return Fraction(float(np.float16(v)))  # float -> Fraction is exact


def _rand_case(seed, M, K, N, bits, group, has_zero=True, zlo=0.0, zhi=None):
    zhi = float((1 << bits) - 1) if zhi is None else zhi
    q = synth.uniform_codes(seed, M * K, bits).reshape(M, K)
    s = synth.uniform_fp16(seed + 1, M * (K // group), 0.005, 0.02).reshape(M, -1)
    z = synth.uniform_fp16(seed + 2, M * (K // group), zlo, zhi).reshape(M, -1) if has_zero else None
    x = synth.normal_fp16(seed + 3, N * K).reshape(N, K)
    return q, s, z, x


# ---------------------------------------------------------------- binary16 conversions

def test_half_to_double_all_patterns(oracle_lib):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)  # numpy's own conversion
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    both_nan = np.isnan(want) & np.isnan(got)
    assert np.all((want == got) | both_nan)
    assert np.all(np.signbit(want) == np.signbit(got))


def test_double_to_half_matches_numpy_rounding(oracle_lib):
    u = synth.uniform01(77, 0, 20000)
    vals = np.concatenate([
        (u[:5000] - 0.5) * 20.0,                 # ordinary magnitudes
        (u[5000:10000] - 0.5) * 2e-4,            # around the subnormal boundary 6.1e-5
        (u[10000:15000] - 0.5) * 1.4e5,          # up to and past overflow (65504)
        (u[15000:] - 0.5) * 1e-7,                # deep subnormals / underflow to zero
    ])
    ties = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2048.0 + 1.0, 2048.0 + 3.0, 65520.0, 65519.99,
                     2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -24, -0.0, 0.0, 1023.5 * 2.0 ** -24, 65504.0])
    vals = np.concatenate([vals, ties, -ties])
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(want, got)


# ---------------------------------------------------------------- the definition oracle

@pytest.mark.parametrize("bits", [1, 2, 4])
def test_matmul_brute_force_exact_rationals(oracle_lib, bits):
    """Tiny shape, every code value present, exact arithmetic with Python fractions."""
    M, K, N, group = 5, 32, 3, 16  # deliberately M != K != N so a transposed operand cannot pass
    q, s, z, x = _rand_case(1000 + bits, M, K, N, bits, group, has_zero=bits > 1)
    q[0, : 1 << bits] = np.arange(1 << bits)  # all codes occur
    Y = oracle.matmul(q, s, z, x, bits, group)
    for n in range(N):
        for m in range(M):
            acc = Fraction(0)
            for k in range(K):
                sc = _frac_half(s[m, k // group])
                if z is None:
                    w = (2 * int(q[m, k]) - 1) * sc
                else:
                    w = (int(q[m, k]) - _frac_half(z[m, k // group])) * sc
                acc += _frac_half(x[n, k]) * w
            ref = float(acc)
            assert abs(Y[n, m] - ref) <= 1e-13 * max(1.0, abs(ref))


def test_matmul_hand_values(oracle_lib):
    """Numbers worked by hand with fp16-exact inputs: catches a wrong sign or swapped scale/zero.
    row 0: codes 5,1 | zero 2.5, scale 0.5 -> weights 1.25, -0.75
    row 1: codes 0,3 | zero 1.0, scale 2.0 -> weights -2.0, 4.0
    x = (2, -1):  y0 = 2*1.25 + 0.75 = 3.25 ;  y1 = -4 - 4 = -8"""
    q = np.array([[5, 1], [0, 3]], dtype=np.uint8)
    s = np.array([[0.5], [2.0]], dtype=np.float16)
    z = np.array([[2.5], [1.0]], dtype=np.float16)
    x = np.array([[2.0, -1.0]], dtype=np.float16)
    Y = oracle.matmul(q, s, z, x, 4, 2)
    assert Y.shape == (1, 2)
    assert Y[0, 0] == 3.25 and Y[0, 1] == -8.0
    # two groups along K: k=0 uses group 0, k=1 uses group 1
    s2 = np.array([[0.5, 0.25], [2.0, 1.0]], dtype=np.float16)
    z2 = np.array([[2.5, 0.0], [1.0, 4.0]], dtype=np.float16)
    Y2 = oracle.matmul(q, s2, z2, x, 4, 1)
    # row0: (5-2.5)*0.5=1.25 ; (1-0)*0.25=0.25 -> 2*1.25 - 0.25 = 2.25
    # row1: (0-1)*2=-2 ; (3-4)*1=-1 -> -4 + 1 = -3
    assert Y2[0, 0] == 2.25 and Y2[0, 1] == -3.0


def test_matmul_unit_vectors_return_dequantized_columns(oracle_lib):
    M, K, group, bits = 7, 64, 32, 4
    q, s, z, _ = _rand_case(2000, M, K, 1, bits, group)
    for k in (0, 1, 31, 32, 63):
        x = np.zeros((1, K), dtype=np.float16)
        x[0, k] = 1.0
        Y = oracle.matmul(q, s, z, x, bits, group)
        col = (q[:, k].astype(np.float64) - z[:, k // group].astype(np.float64)) * s[:, k // group].astype(np.float64)
        assert np.array_equal(Y[0], col)


@pytest.mark.parametrize("bits", [2, 4])
def test_matmul_reduces_to_integer_matvec(oracle_lib, bits):
    """zero = 0, scale = 1, integer activations: the product is an integer matrix product (numpy int64)."""
    M, K, N, group = 33, 128, 4, 64
    q = synth.uniform_codes(3000 + bits, M * K, bits).reshape(M, K)
    xi = (synth.uniform_codes(3100 + bits, N * K, 4).astype(np.int64) - 8).reshape(N, K)
    s = np.ones((M, K // group), dtype=np.float16)
    z = np.zeros((M, K // group), dtype=np.float16)
    Y = oracle.matmul(q, s, z, xi.astype(np.float16), bits, group)
    assert np.array_equal(Y, (xi @ q.astype(np.int64).T).astype(np.float64))


def test_sign_mode_is_plus_minus_scale(oracle_lib):
    M, K, N, group = 9, 128, 2, 64
    q = synth.uniform_codes(3300, M * K, 1).reshape(M, K)
    xi = (synth.uniform_codes(3301, N * K, 3).astype(np.int64) - 4).reshape(N, K)
    s = np.full((M, K // group), 0.25, dtype=np.float16)
    Y = oracle.matmul(q, s, None, xi.astype(np.float16), 1, group)
    signs = 2 * q.astype(np.int64) - 1
    assert np.array_equal(Y, 0.25 * (xi @ signs.T))
    # and it equals the affine form with zero = 1/2 and a doubled scale
    Y2 = oracle.matmul(q, 2 * s, np.full_like(s, 0.5), xi.astype(np.float16), 1, group)
    assert np.array_equal(Y, Y2)


def test_matmul_thread_count_does_not_change_results(oracle_lib):
    q, s, z, x = _rand_case(3400, 40, 256, 3, 4, 64, zlo=6, zhi=9)
    Y1, used1 = oracle.matmul(q, s, z, x, 4, 64, threads=1, return_threads=True)
    Y4, used4 = oracle.matmul(q, s, z, x, 4, 64, threads=4, return_threads=True)
    assert used1 == 1 and used4 >= 1
    assert np.array_equal(Y1, Y4)


# ---------------------------------------------------------------- table-lookup form

def test_tables_closed_forms(oracle_lib):
    x = synth.normal_fp16(4000, 3 * 64).reshape(3, 64)
    T = oracle.build_tables(x, 4)
    assert T.shape == (3, 16, 16)
    xd = x.astype(np.float64).reshape(3, 16, 4)
    assert np.all(T[:, :, 0] == 0.0)
    for t in range(4):
        assert np.array_equal(T[:, :, 1 << t], xd[:, :, t])  # pattern bit t selects activation 4j+t
    for p in range(16):
        assert np.array_equal(T[:, :, p] + T[:, :, 15 - p], T[:, :, 15])  # complement patterns (exact in double)
    # brute force with exact rationals on one table
    for p in range(16):
        ref = sum((_frac_half(x[1, 20 + t]) for t in range(4) if (p >> t) & 1), Fraction(0))
        assert T[1, 5, p] == float(ref)


def test_lut_indices_paper_example(oracle_lib):
    """Sec. 4.1: the most significant bits of four INT4 weights pack to 0b0011 when weights 0 and 1
    have their MSB set; the repacking table entry for it is 0b0000 0000 1000 1000."""
    (row,) = _rows("repack_example.txt")
    i, p, entry = int(row[0]), int(row[1], 2), int(row[2], 2)
    q = np.array([[0b1000, 0b1010, 0b0111, 0b0001]], dtype=np.uint8)  # MSB set on weights 0 and 1 only
    idx = oracle.lut_indices(q, 4, 4)
    assert idx.shape == (4, 1, 1)
    assert idx[i, 0, 0] == p
    assert oracle.repack_entry(i, p) == entry
    # combining the entries of all four bit positions reconstructs the codes, field t = weight t
    word = 0
    for b in range(4):
        word |= oracle.repack_entry(b, int(idx[b, 0, 0]))
    assert [(word >> (4 * t)) & 15 for t in range(4)] == [int(c) for c in q[0]]


def test_repack_table_reconstructs_all_patterns(oracle_lib):
    for codes in ([0, 0, 0, 0], [15, 15, 15, 15], [1, 2, 4, 8], [9, 6, 3, 12], [5, 10, 0, 15]):
        q = np.array([codes], dtype=np.uint8)
        idx = oracle.lut_indices(q, 4, 4)
        word = 0
        for b in range(4):
            word |= oracle.repack_entry(b, int(idx[b, 0, 0]))
        assert word == sum(c << (4 * t) for t, c in enumerate(codes))


def test_vlut_table_pins_group_width_four():
    """One lookup stands for g multiply-adds; the printed table gives g = 4 for the 16-entry variant
    the paper selects, and 16 table registers <-> k-tile 256 gives 16-bit entries."""
    rows = _rows("vlut_throughput.txt")
    for r in rows:
        if r[0] == "VLUT16":
            assert int(r[5]) == 4 * int(r[4]) and int(r[1]) == 2 ** 4
        if r[0] == "VLUT32":
            assert int(r[5]) == 5 * int(r[4]) and int(r[1]) == 2 ** 5
        if r[0] == "REGS":
            regs, reg_bits, ktile = int(r[1]), int(r[2]), int(r[3])
            tables_per_reg = reg_bits // (16 * 16)  # 16 entries of 16 bits
            assert regs * tables_per_reg * 4 == ktile


@pytest.mark.parametrize("bits,group", [(1, 64), (2, 64), (4, 64), (4, 128), (2, 32)])
def test_lut_identity_bit_exact(oracle_lib, bits, group):
    """Group sums through tables == sum_k q*x per group, bit for bit (every term is a multiple of
    2^-24 and the sums stay far below 2^53 * 2^-24), and the full products agree to rounding."""
    M, K, N = 24, 512, 3
    has_zero = bits > 1
    q, s, z, x = _rand_case(5000 + bits + group, M, K, N, bits, group, has_zero=has_zero)
    Y_lut, A = oracle.lut_matmul(q, s, z, x, bits, group, return_group_sums=True)
    direct = np.einsum("nGk,mGk->nmG", x.astype(np.float64).reshape(N, K // group, group),
                       q.astype(np.float64).reshape(M, K // group, group))
    assert np.array_equal(A, direct)
    Y = oracle.matmul(q, s, z, x, bits, group)
    scale = np.sqrt(np.mean(Y * Y))
    assert np.max(np.abs(Y_lut - Y)) <= 1e-12 * scale


def test_lut_form_with_fp16_tables_stays_within_budget(oracle_lib):
    """The method's own rounding (16-bit table entries) on an LLM-sized reduction stays inside the
    2e-3 bound under the row-normalised metric; this is the floor the kernels are compared above."""
    M, K, bits, group = 96, 4096, 4, 64
    q, s, z, x = _rand_case(5100, M, K, 1, bits, group, zlo=6, zhi=9)
    Y = oracle.matmul(q, s, z, x, bits, group)
    Yr = oracle.lut_matmul(q, s, z, x, bits, group, round_tables=True)
    assert oracle.row_relative_error(Yr, Y).max() < 1e-3
    assert not np.array_equal(Yr, Y)  # the rounding really happened


# ---------------------------------------------------------------- table dequantization (prefill)

def test_dequant_table_entries(oracle_lib):
    for r in _rows("dequant_table_ops.txt"):
        bits, block, ops = int(r[0]), int(r[1]), int(r[2])
        D = oracle.dequant_table(int(np.float16(0.0125).view(np.uint16)), int(np.float16(1.5).view(np.uint16)), bits)
        assert D.shape == (ops,) == (2 ** bits,)
        assert Fraction(r[3]) == Fraction(ops, block)
    s, z = np.float16(0.0123), np.float16(7.31)
    D = oracle.dequant_table(int(s.view(np.uint16)), int(z.view(np.uint16)), 4)
    for c in range(16):
        exact = (Fraction(c) - _frac_half(z)) * _frac_half(s)
        lo, hi = np.nextafter(D[c], np.float16(-np.inf)), np.nextafter(D[c], np.float16(np.inf))
        # correctly rounded: no neighbouring fp16 value is closer to the exact product
        assert abs(Fraction(float(D[c])) - exact) <= abs(Fraction(float(lo)) - exact)
        assert abs(Fraction(float(D[c])) - exact) <= abs(Fraction(float(hi)) - exact)
    Ds = oracle.dequant_table(int(np.float16(0.25).view(np.uint16)), 0, 1, sign_mode=True)
    assert list(Ds) == [-0.25, 0.25]


def test_table_dequant_matmul_close_to_definition(oracle_lib):
    q, s, z, x = _rand_case(5200, 48, 1024, 2, 4, 64, zlo=6, zhi=9)
    Y = oracle.matmul(q, s, z, x, 4, 64)
    Yt = oracle.table_dequant_matmul(q, s, z, x, 4, 64)
    err = oracle.row_relative_error(Yt, Y).max()
    assert 0 < err < 1e-3
    # with scale = 1 and integer zero every table entry is exact, so the two must coincide
    s1 = np.ones_like(s)
    z1 = np.full_like(z, 7.0)
    assert np.array_equal(oracle.table_dequant_matmul(q, s1, z1, x, 4, 64), oracle.matmul(q, s1, z1, x, 4, 64))


# ---------------------------------------------------------------- error metric

def test_row_relative_error_hand_example():
    Y = np.array([[3.0, -4.0, 0.0, 0.0]])  # rms = sqrt(25/4) = 2.5
    yh = np.array([[3.03, -4.0, 0.05, 0.0]])
    e = oracle.row_relative_error(yh, Y)
    assert e.shape == (1,)
    assert abs(e[0] - 0.05 / 2.5) < 1e-12  # the small output is judged against the row rms, 0.03/3 is smaller
