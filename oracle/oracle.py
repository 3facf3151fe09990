"""ctypes front end of ``tman_oracle.c`` (plain C, double precision).  TEST INFRASTRUCTURE ONLY.

The C file states what each routine computes and which passage of the paper it follows; this module
only marshals numpy arrays.  ``build()`` compiles the C file with gcc into ``oracle/libtman_oracle.so``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tman_oracle.c")
_SO = os.path.join(_HERE, "libtman_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle (always when ``force``; otherwise only if missing or stale)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        global _lib
        _lib = None
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        u8p, u16p, f64p = C.POINTER(C.c_uint8), C.POINTER(C.c_uint16), C.POINTER(C.c_double)
        L.tman_oracle_half_to_double.restype = C.c_double
        L.tman_oracle_half_to_double.argtypes = [C.c_uint16]
        L.tman_oracle_double_to_half.restype = C.c_uint16
        L.tman_oracle_double_to_half.argtypes = [C.c_double]
        L.tman_oracle_matmul.restype = C.c_int
        L.tman_oracle_matmul.argtypes = [u8p, u16p, u16p, u16p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, f64p, C.c_int]
        L.tman_oracle_build_tables.restype = None
        L.tman_oracle_build_tables.argtypes = [u16p, C.c_int, C.c_int, C.c_int, f64p]
        L.tman_oracle_lut_indices.restype = None
        L.tman_oracle_lut_indices.argtypes = [u8p, C.c_int, C.c_int, C.c_int, C.c_int, u8p]
        L.tman_oracle_lut_matmul.restype = None
        L.tman_oracle_lut_matmul.argtypes = [u8p, u16p, u16p, u16p] + [C.c_int] * 8 + [f64p, f64p]
        L.tman_oracle_repack_entry.restype = C.c_uint16
        L.tman_oracle_repack_entry.argtypes = [C.c_int, C.c_int]
        L.tman_oracle_dequant_table.restype = None
        L.tman_oracle_dequant_table.argtypes = [C.c_uint16, C.c_uint16, C.c_int, C.c_int, u16p]
        L.tman_oracle_table_dequant_matmul.restype = None
        L.tman_oracle_table_dequant_matmul.argtypes = [u8p, u16p, u16p, u16p] + [C.c_int] * 6 + [f64p]
        i16p, i32p, i64p = C.POINTER(C.c_int16), C.POINTER(C.c_int32), C.POINTER(C.c_int64)
        L.tman_oracle_quantize_activations.restype = None
        L.tman_oracle_quantize_activations.argtypes = [u16p, C.c_int, C.c_int, i16p, i32p]
        L.tman_oracle_matmul_real_x.restype = None
        L.tman_oracle_matmul_real_x.argtypes = [u8p, u16p, u16p, f64p] + [C.c_int] * 5 + [f64p]
        L.tman_oracle_lut_matmul_i16.restype = C.c_int
        L.tman_oracle_lut_matmul_i16.argtypes = [u8p, u16p, u16p, i16p, i32p] + [C.c_int] * 6 + [f64p, i64p]
        i8p, f32p = C.POINTER(C.c_int8), C.POINTER(C.c_float)
        L.tman_oracle_quantize_activations_i8.restype = None
        L.tman_oracle_quantize_activations_i8.argtypes = [u16p, C.c_int, C.c_int, i8p, f32p]
        L.tman_oracle_matmul_i8.restype = None
        L.tman_oracle_matmul_i8.argtypes = [u8p, u16p, u16p, i8p, f32p] + [C.c_int] * 4 + [i64p, f64p]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray], ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _prep(q, scale, zero, x, bits, group):
    q = np.ascontiguousarray(q, dtype=np.uint8)
    M, K = q.shape
    assert K % group == 0
    assert int(q.max(initial=0)) < (1 << bits)
    s = np.ascontiguousarray(scale, dtype=np.float16).reshape(M, K // group).view(np.uint16)
    z = None if zero is None else np.ascontiguousarray(zero, dtype=np.float16).reshape(M, K // group).view(np.uint16)
    x = np.ascontiguousarray(x, dtype=np.float16)
    N = x.shape[0]
    assert x.shape == (N, K)
    return q, s, z, x.view(np.uint16), N, M, K


def matmul(q, scale, zero, x, bits: int, group: int, threads: int = 0, return_threads: bool = False):
    """Definition oracle: Y[n][m] = sum_k x[n][k] * (q[m][k] - zero) * scale in double, ascending k.
    ``zero=None`` selects the 1-bit sign form (2q - 1) * scale."""
    q, s, z, xb, N, M, K = _prep(q, scale, zero, x, bits, group)
    Y = np.empty((N, M), dtype=np.float64)
    used = lib().tman_oracle_matmul(_p(q, C.c_uint8), _p(s, C.c_uint16), _p(z, C.c_uint16), _p(xb, C.c_uint16),
                                    N, M, K, group, int(zero is None), _p(Y, C.c_double), threads)
    assert used >= 1
    return (Y, used) if return_threads else Y


def lut_matmul(q, scale, zero, x, bits: int, group: int, g: int = 4, round_tables: bool = False,
               return_group_sums: bool = False):
    """Bit-serial table-lookup form (Sec. 2.2) in double; optionally with fp16-rounded table entries."""
    q, s, z, xb, N, M, K = _prep(q, scale, zero, x, bits, group)
    assert group % g == 0
    Y = np.empty((N, M), dtype=np.float64)
    A = np.empty((N, M, K // group), dtype=np.float64) if return_group_sums else None
    lib().tman_oracle_lut_matmul(_p(q, C.c_uint8), _p(s, C.c_uint16), _p(z, C.c_uint16), _p(xb, C.c_uint16),
                                 N, M, K, bits, group, g, int(zero is None), int(round_tables),
                                 _p(Y, C.c_double), _p(A, C.c_double))
    return (Y, A) if return_group_sums else Y


def table_dequant_matmul(q, scale, zero, x, bits: int, group: int):
    """Prefill at the method's own precision: fp16 table-dequantized weights, exact accumulation."""
    q, s, z, xb, N, M, K = _prep(q, scale, zero, x, bits, group)
    Y = np.empty((N, M), dtype=np.float64)
    lib().tman_oracle_table_dequant_matmul(_p(q, C.c_uint8), _p(s, C.c_uint16), _p(z, C.c_uint16), _p(xb, C.c_uint16),
                                           N, M, K, bits, group, int(zero is None), _p(Y, C.c_double))
    return Y


def quantize_activations(x):
    """Integer activations of the A_INT16 reading: (xq int16 [N][K] with |xq| <= 8191, e int32 [N]) with
    xq = RNE(x / 2^e), 2^e the smallest power of two that brings every activation of the token within 8191."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    N, K = x.shape
    xq = np.empty((N, K), dtype=np.int16)
    e = np.empty(N, dtype=np.int32)
    lib().tman_oracle_quantize_activations(_p(x.view(np.uint16), C.c_uint16), N, K, _p(xq, C.c_int16), _p(e, C.c_int32))
    return xq, e


def matmul_real_x(q, scale, zero, xd, bits: int, group: int):
    """The definition for activations given as doubles [N][K] (e.g. dequantized integer activations)."""
    xd = np.ascontiguousarray(xd, dtype=np.float64)
    N, K = xd.shape
    q, s, z, _, _, M, K2 = _prep(q, scale, zero, np.zeros((1, K), np.float16), bits, group)
    assert K2 == K
    Y = np.empty((N, M), dtype=np.float64)
    lib().tman_oracle_matmul_real_x(_p(q, C.c_uint8), _p(s, C.c_uint16), _p(z, C.c_uint16), _p(xd, C.c_double), N, M, K,
                                    group, int(zero is None), _p(Y, C.c_double))
    return Y


def lut_matmul_i16(q, scale, zero, xq, e, bits: int, group: int, return_block_sums: bool = False):
    """Table-lookup form on integer activations: integer tables, integer sums inside a quantization block."""
    xq = np.ascontiguousarray(xq, dtype=np.int16)
    e = np.ascontiguousarray(e, dtype=np.int32)
    N, K = xq.shape
    q, s, z, _, _, M, K2 = _prep(q, scale, zero, np.zeros((1, K), np.float16), bits, group)
    assert K2 == K and e.shape == (N,)
    Y = np.empty((N, M), dtype=np.float64)
    A = np.empty((N, M, K // group), dtype=np.int64) if return_block_sums else None
    over = lib().tman_oracle_lut_matmul_i16(_p(q, C.c_uint8), _p(s, C.c_uint16), _p(z, C.c_uint16), _p(xq, C.c_int16),
                                            _p(e, C.c_int32), N, M, K, bits, group, int(zero is None), _p(Y, C.c_double),
                                            _p(A, C.c_int64))
    assert over == 0, "a table entry does not fit 16 bits"
    return (Y, A) if return_block_sums else Y


def quantize_activations_i8(x):
    """Per-token absmax quantizer to int8 (decision in binary32): (xq int8 [N][K], absmax float32 [N])."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    N, K = x.shape
    xq = np.empty((N, K), dtype=np.int8)
    mx = np.empty(N, dtype=np.float32)
    lib().tman_oracle_quantize_activations_i8(_p(x.view(np.uint16), C.c_uint16), N, K, _p(xq, C.c_int8), _p(mx, C.c_float))
    return xq, mx


def matmul_i8(q, row_scale, row_zero, xq, absmax, bits: int):
    """Integer product of codes and int8 activations with one scale / zero per row: (acc int64 [N][M], Y [N][M])."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    M, K = q.shape
    assert int(q.max(initial=0)) < (1 << bits)
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    N = xq.shape[0]
    assert xq.shape == (N, K)
    rs = np.ascontiguousarray(row_scale, dtype=np.float16).reshape(M).view(np.uint16)
    rz = None if row_zero is None else np.ascontiguousarray(row_zero, dtype=np.float16).reshape(M).view(np.uint16)
    mx = np.ascontiguousarray(absmax, dtype=np.float32)
    acc = np.empty((N, M), dtype=np.int64)
    Y = np.empty((N, M), dtype=np.float64)
    lib().tman_oracle_matmul_i8(_p(q, C.c_uint8), _p(rs, C.c_uint16), _p(rz, C.c_uint16), _p(xq, C.c_int8), _p(mx, C.c_float),
                                N, M, K, int(row_zero is None), _p(acc, C.c_int64), _p(Y, C.c_double))
    return acc, Y


def build_tables(x, g: int = 4) -> np.ndarray:
    """T[n][j][p] = sum_t bit_t(p) x[n][g j + t], double, exact."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    N, K = x.shape
    assert K % g == 0
    T = np.empty((N, K // g, 1 << g), dtype=np.float64)
    lib().tman_oracle_build_tables(_p(x.view(np.uint16), C.c_uint16), N, K, g, _p(T, C.c_double))
    return T


def lut_indices(q, bits: int, g: int = 4) -> np.ndarray:
    """idx[i][m][j]: g-bit pattern of plane i over weights g j .. g j + g - 1 (weight t in bit t)."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    M, K = q.shape
    idx = np.empty((bits, M, K // g), dtype=np.uint8)
    lib().tman_oracle_lut_indices(_p(q, C.c_uint8), M, K, bits, g, _p(idx, C.c_uint8))
    return idx


def repack_entry(i: int, p: int) -> int:
    return int(lib().tman_oracle_repack_entry(i, p))


def dequant_table(scale_bits: int, zero_bits: int, bits: int, sign_mode: bool = False) -> np.ndarray:
    D = np.empty(1 << bits, dtype=np.uint16)
    lib().tman_oracle_dequant_table(scale_bits, zero_bits, bits, int(sign_mode), _p(D, C.c_uint16))
    return D.view(np.float16)


def half_to_double(h: int) -> float:
    return float(lib().tman_oracle_half_to_double(h))


def double_to_half(d: float) -> int:
    return int(lib().tman_oracle_double_to_half(d))


def row_relative_error(y_hat: np.ndarray, Y: np.ndarray) -> np.ndarray:
    """Per token n: max_m |y_hat - Y| / max(|Y[n][m]|, rms_m Y[n][:]).

    Outputs are zero-mean sums, so a purely element-wise relative error is unbounded near zero
    crossings; the row's rms puts a floor under the denominator."""
    Y = np.asarray(Y, dtype=np.float64)
    d = np.abs(np.asarray(y_hat, dtype=np.float64) - Y)
    rms = np.sqrt(np.mean(Y * Y, axis=1, keepdims=True))
    den = np.maximum(np.abs(Y), np.maximum(rms, np.finfo(np.float64).tiny))
    return (d / den).max(axis=1)
