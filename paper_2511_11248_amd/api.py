"""ctypes binding of libtman.so.  Argument marshalling only -- no arithmetic happens in Python.

Tensors are ``torch`` tensors on the GPU (torch supplies device memory and the stream); anything with
a ``data_ptr()`` works.  Every call enqueues on ``stream`` (default: torch's current stream) and
returns without synchronising.  A missing library is an error: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtman.so")
_lib = None

TMAN_FLAG_HAS_ZERO = 1
TMAN_MAX_DECODE_TOKENS = 8


class TmanError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {tman_status_string(status)} (status {status})")


class Tiling(C.Structure):
    """Mirror of ``tman_tiling_t`` (see include/tman.h)."""
    _fields_ = [("decode_seg_tiles", C.c_int32), ("decode_seg_tiles_many", C.c_int32), ("decode_x_seg_tiles", C.c_int32),
                ("decode_x_long_seg_tiles", C.c_int32), ("decode_x_whole_bytes", C.c_int32), ("small_seg_tiles", C.c_int32),
                ("prefill_row_blocks", C.c_int32), ("decode_balance", C.c_int32), ("i8_token_blocks", C.c_int32), ("prefill_k_split", C.c_int32)]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class _CShape(C.Structure):
    _fields_ = [("M", C.c_int32), ("K", C.c_int32), ("bits", C.c_int32), ("group", C.c_int32), ("flags", C.c_int32)]


@dataclass(frozen=True)
class Shape:
    """Mirror of ``tman_shape_t``: W is (M, K), ``bits``-bit codes, quantization blocks of ``group``
    along K, with a per-block zero point unless ``has_zero`` is False (1-bit sign form)."""
    M: int
    K: int
    bits: int
    group: int
    has_zero: bool = True

    def c(self) -> _CShape:
        return _CShape(self.M, self.K, self.bits, self.group, TMAN_FLAG_HAS_ZERO if self.has_zero else 0)


def library_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2511_11248_amd.build` "
                "(there is no non-HIP fallback)")
        L = C.CDLL(_LIB_PATH)
        sp, vp = C.POINTER(_CShape), C.c_void_p
        L.tman_packed_bytes.restype = C.c_size_t
        L.tman_packed_bytes.argtypes = [sp]
        L.tman_lut_bytes.restype = C.c_size_t
        L.tman_lut_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.tman_mpgemv_workspace_bytes.restype = C.c_size_t
        L.tman_mpgemv_workspace_bytes.argtypes = [sp, C.c_int32]
        L.tman_mpgemm_workspace_bytes.restype = C.c_size_t
        L.tman_mpgemm_workspace_bytes.argtypes = [sp, C.c_int32]
        L.tman_pack_weights.restype = C.c_int
        L.tman_pack_weights.argtypes = [sp, vp, vp, vp, vp, vp]
        L.tman_unpack_weights.restype = C.c_int
        L.tman_unpack_weights.argtypes = [sp, vp, vp, vp, vp, vp]
        L.tman_build_lut.restype = C.c_int
        L.tman_build_lut.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, vp, vp]
        L.tman_build_lut_batch.restype = C.c_int
        L.tman_build_lut_batch.argtypes = [C.c_int32, vp, C.c_int32, vp, C.c_int32, vp, vp]
        L.tman_mpgemv.restype = C.c_int
        L.tman_mpgemv.argtypes = [sp, vp, vp, C.c_int32, vp, vp, C.c_size_t, vp]
        L.tman_lut_i16_bytes.restype = C.c_size_t
        L.tman_lut_i16_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.tman_build_lut_i16.restype = C.c_int
        L.tman_build_lut_i16.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, vp, vp]
        L.tman_build_lut_i16_batch.restype = C.c_int
        L.tman_build_lut_i16_batch.argtypes = [C.c_int32, vp, C.c_int32, vp, C.c_int32, vp, vp]
        L.tman_mpgemv_i16.restype = C.c_int
        L.tman_mpgemv_i16.argtypes = [sp, vp, vp, C.c_int32, vp, vp, C.c_size_t, vp]
        L.tman_mpgemv_i16_batch_run.restype = C.c_int
        L.tman_mpgemv_i16_batch_run.argtypes = [C.c_int32, sp, C.c_int32, vp, vp]
        L.tman_mpgemv_batch_desc_bytes.restype = C.c_size_t
        L.tman_mpgemv_batch_desc_bytes.argtypes = [C.c_int32]
        L.tman_mpgemv_batch_prepare.restype = C.c_int
        L.tman_mpgemv_batch_prepare.argtypes = [C.c_int32, sp, vp, vp, C.c_int32, vp, vp, vp, vp, vp]
        L.tman_mpgemv_batch_run.restype = C.c_int
        L.tman_mpgemv_batch_run.argtypes = [C.c_int32, sp, C.c_int32, vp, vp]
        L.tman_mpgemv_x.restype = C.c_int
        L.tman_mpgemv_x.argtypes = [sp, vp, vp, vp, vp, C.c_size_t, vp]
        L.tman_mpgemv_x_batch_order.restype = C.c_int
        L.tman_mpgemv_x_batch_order.argtypes = [C.c_int32, sp, C.c_int32, C.POINTER(C.c_uint16), C.c_int32,
                                                C.POINTER(C.c_int32)]
        L.tman_mpgemv_x_batch_prepare.restype = C.c_int
        L.tman_mpgemv_x_batch_prepare.argtypes = [C.c_int32, sp, vp, vp, vp, vp, vp, vp, vp]
        L.tman_mpgemv_x_batch_run.restype = C.c_int
        L.tman_mpgemv_x_batch_run.argtypes = [C.c_int32, sp, vp, vp]
        L.tman_mpgemm.restype = C.c_int
        L.tman_mpgemm.argtypes = [sp, vp, vp, C.c_int32, vp, vp, C.c_size_t, vp]
        L.tman_mpgemm_batch_prepare.restype = C.c_int
        L.tman_mpgemm_batch_prepare.argtypes = [C.c_int32, sp, vp, vp, C.c_int32, vp, vp, vp, vp, vp]
        L.tman_mpgemm_batch_run.restype = C.c_int
        L.tman_mpgemm_batch_run.argtypes = [C.c_int32, sp, C.c_int32, vp, vp]
        L.tman_act_i8_bytes.restype = C.c_size_t
        L.tman_act_i8_bytes.argtypes = [C.c_int32, C.c_int32]
        L.tman_quantize_act_i8.restype = C.c_int
        L.tman_quantize_act_i8.argtypes = [vp, C.c_int32, C.c_int32, vp, vp]
        L.tman_mpgemm_i8.restype = C.c_int
        L.tman_mpgemm_i8.argtypes = [sp, vp, vp, C.c_int32, vp, vp, vp]
        L.tman_mpgemm_tile_rows.restype = C.c_int32
        L.tman_mpgemm_tile_rows.argtypes = [sp, C.c_int32]
        L.tman_mpgemm_splits_k.restype = C.c_int32
        L.tman_mpgemm_splits_k.argtypes = [sp, C.c_int32]
        L.tman_mpgemm_i8_token_blocks.restype = C.c_int32
        L.tman_mpgemm_i8_token_blocks.argtypes = [sp, C.c_int32]
        L.tman_check_packed.restype = C.c_int
        L.tman_check_packed.argtypes = [sp, vp, vp]
        L.tman_device_status.restype = C.c_int
        L.tman_device_status.argtypes = [vp]
        L.tman_noalloc_init.restype = C.c_int
        L.tman_noalloc_init.argtypes = []
        L.tman_mpgemv_noalloc.restype = C.c_int
        L.tman_mpgemv_noalloc.argtypes = [sp, vp, vp, C.c_int32, vp, vp]
        for fn in (L.tman_default_tiling, L.tman_get_tiling, L.tman_set_tiling):
            fn.restype = C.c_int
            fn.argtypes = [C.POINTER(Tiling)]
        L.tman_status_string.restype = C.c_char_p
        L.tman_status_string.argtypes = [C.c_int]
        L.tman_layout_version.restype = C.c_int32
        L.tman_layout_version.argtypes = []
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise TmanError(status, where)


def tman_status_string(status: int) -> str:
    return _load().tman_status_string(status).decode()


def tman_layout_version() -> int:
    return int(_load().tman_layout_version())


def tman_packed_bytes(shape: Shape) -> int:
    return int(_load().tman_packed_bytes(C.byref(shape.c())))


def tman_lut_bytes(N: int, K: int, group: int) -> int:
    return int(_load().tman_lut_bytes(N, K, group))


def tman_mpgemv_workspace_bytes(shape: Shape, N: int) -> int:
    return int(_load().tman_mpgemv_workspace_bytes(C.byref(shape.c()), N))


def tman_mpgemm_workspace_bytes(shape: Shape, N: int) -> int:
    return int(_load().tman_mpgemm_workspace_bytes(C.byref(shape.c()), N))


def tman_mpgemm_tile_rows(shape: Shape, N: int) -> int:
    return int(_load().tman_mpgemm_tile_rows(C.byref(shape.c()), N))


def tman_mpgemm_splits_k(shape: Shape, N: int) -> int:
    return int(_load().tman_mpgemm_splits_k(C.byref(shape.c()), N))


def tman_mpgemm_i8_token_blocks(shape: Shape, N: int) -> int:
    return int(_load().tman_mpgemm_i8_token_blocks(C.byref(shape.c()), N))


def tman_pack_weights(shape: Shape, codes, scales, zeros, packed, stream=None) -> None:
    """codes u8 [M][K], scales/zeros fp16 [M][K/group] (zeros None for the sign form) -> packed (u8 blob)."""
    _check(_load().tman_pack_weights(C.byref(shape.c()), _ptr(codes), _ptr(scales), _ptr(zeros), _ptr(packed),
                                     _stream(stream)), "tman_pack_weights")


def tman_unpack_weights(shape: Shape, packed, codes, scales=None, zeros=None, stream=None) -> None:
    _check(_load().tman_unpack_weights(C.byref(shape.c()), _ptr(packed), _ptr(codes), _ptr(scales), _ptr(zeros),
                                       _stream(stream)), "tman_unpack_weights")


def tman_build_lut(x, N: int, K: int, group: int, lut, stream=None) -> None:
    """x fp16 [N][K] -> lut (u8 buffer of tman_lut_bytes(N, K, group))."""
    _check(_load().tman_build_lut(_ptr(x), N, K, group, _ptr(lut), _stream(stream)), "tman_build_lut")


def tman_lut_i16_bytes(N: int, K: int, group: int) -> int:
    return int(_load().tman_lut_i16_bytes(N, K, group))


def tman_build_lut_i16(x, N: int, K: int, group: int, lut, stream=None) -> None:
    """x fp16 [N][K] -> integer tables (u8 buffer of tman_lut_i16_bytes(N, K, group))."""
    _check(_load().tman_build_lut_i16(_ptr(x), N, K, group, _ptr(lut), _stream(stream)), "tman_build_lut_i16")


def tman_build_lut_i16_batch(xs, N: int, Ks, group: int, luts, stream=None) -> None:
    n = len(xs)
    vp = C.c_void_p * n
    _check(_load().tman_build_lut_i16_batch(n, vp(*[_ptr(t) for t in xs]), N, (C.c_int32 * n)(*Ks), group,
                                            vp(*[_ptr(t) for t in luts]), _stream(stream)), "tman_build_lut_i16_batch")


def tman_mpgemv_i16(shape: Shape, packed, lut, N: int, y, workspace, stream=None) -> None:
    """y fp16 [N][M] through lookups in integer tables (from tman_build_lut_i16)."""
    wb = 0 if workspace is None or isinstance(workspace, int) else _nbytes(workspace)
    _check(_load().tman_mpgemv_i16(C.byref(shape.c()), _ptr(packed), _ptr(lut), N, _ptr(y), _ptr(workspace), wb,
                                   _stream(stream)), "tman_mpgemv_i16")


def tman_mpgemv_i16_batch_run(shapes, N: int, desc, stream=None) -> None:
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    _check(_load().tman_mpgemv_i16_batch_run(n, cs, N, _ptr(desc), _stream(stream)), "tman_mpgemv_i16_batch_run")


def tman_mpgemv(shape: Shape, packed, lut, N: int, y, workspace, stream=None) -> None:
    """y fp16 [N][M] = x * dequant(W)^T through table lookup; workspace zero-filled once by the caller."""
    wb = 0 if workspace is None or isinstance(workspace, int) else _nbytes(workspace)
    _check(_load().tman_mpgemv(C.byref(shape.c()), _ptr(packed), _ptr(lut), N, _ptr(y), _ptr(workspace), wb,
                               _stream(stream)), "tman_mpgemv")


def tman_check_packed(shape: Shape, packed, stream=None) -> int:
    """Status of the host-side header check (0 or TMAN_ERR_HEADER = -8); waits for the stream."""
    return int(_load().tman_check_packed(C.byref(shape.c()), _ptr(packed), _stream(stream)))


def tman_device_status(stream=None) -> int:
    """Returns and clears the device status word (0, or -8 when a kernel met a blob with a foreign header)."""
    return int(_load().tman_device_status(_stream(stream)))


def tman_default_tiling() -> Tiling:
    t = Tiling()
    _check(_load().tman_default_tiling(C.byref(t)), "tman_default_tiling")
    return t


def tman_get_tiling() -> Tiling:
    t = Tiling()
    _check(_load().tman_get_tiling(C.byref(t)), "tman_get_tiling")
    return t


def tman_set_tiling(t: Tiling) -> None:
    _check(_load().tman_set_tiling(C.byref(t)), "tman_set_tiling")


def tman_noalloc_init() -> None:
    _check(_load().tman_noalloc_init(), "tman_noalloc_init")


def tman_mpgemv_noalloc(shape: Shape, packed, lut, N: int, y, stream=None) -> None:
    """tman_mpgemv with the library's own fixed scratch array as workspace (allocates nothing)."""
    _check(_load().tman_mpgemv_noalloc(C.byref(shape.c()), _ptr(packed), _ptr(lut), N, _ptr(y), _stream(stream)),
           "tman_mpgemv_noalloc")


def tman_mpgemm(shape: Shape, packed, x, N: int, y, workspace=None, stream=None) -> None:
    """y fp16 [N][M] = x fp16 [N][K] * dequant(W)^T, table dequantization feeding the matrix cores."""
    wb = 0 if workspace is None or isinstance(workspace, int) else _nbytes(workspace)
    _check(_load().tman_mpgemm(C.byref(shape.c()), _ptr(packed), _ptr(x), N, _ptr(y), _ptr(workspace), wb,
                               _stream(stream)), "tman_mpgemm")


def tman_act_i8_bytes(N: int, K: int) -> int:
    return int(_load().tman_act_i8_bytes(N, K))


def tman_quantize_act_i8(x, N: int, K: int, xq, stream=None) -> None:
    """x fp16 [N][K] -> int8 activations (permuted per 32 columns), per-token maxima and sums."""
    _check(_load().tman_quantize_act_i8(_ptr(x), N, K, _ptr(xq), _stream(stream)), "tman_quantize_act_i8")


def tman_mpgemm_i8(shape: Shape, packed, xq, N: int, y, acc=None, stream=None) -> None:
    """y fp16 [N][M] on the integer matrix cores for weights with one scale and zero per row."""
    _check(_load().tman_mpgemm_i8(C.byref(shape.c()), _ptr(packed), _ptr(xq), N, _ptr(y), _ptr(acc), _stream(stream)),
           "tman_mpgemm_i8")


def tman_mpgemm_batch_prepare(shapes, packed, xs, N: int, y, workspace, desc, stream=None) -> None:
    """Descriptor table for a batch of small-batch mpGEMMs (N <= 32); workspace entries may be None where the
    size query gives 0."""
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    vp = C.c_void_p * n
    wb = (C.c_size_t * n)(*[0 if t is None else _nbytes(t) for t in workspace])
    _check(_load().tman_mpgemm_batch_prepare(n, cs, vp(*[_ptr(t) for t in packed]), vp(*[_ptr(t) for t in xs]), N,
                                             vp(*[_ptr(t) for t in y]), vp(*[_ptr(t) for t in workspace]), wb,
                                             _ptr(desc), _stream(stream)), "tman_mpgemm_batch_prepare")


def tman_mpgemm_batch_run(shapes, N: int, desc, stream=None) -> None:
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    _check(_load().tman_mpgemm_batch_run(n, cs, N, _ptr(desc), _stream(stream)), "tman_mpgemm_batch_run")


def bound_mpgemm_batch_run(shapes, N: int, desc):
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    fn, args = _load().tman_mpgemm_batch_run, (n, cs, N, _ptr(desc))

    def call(stream_handle):
        _check(fn(*args, stream_handle), "tman_mpgemm_batch_run")

    return call


def tman_mpgemv_batch_desc_bytes(count: int) -> int:
    return int(_load().tman_mpgemv_batch_desc_bytes(count))


def _batch_arrays(shapes, packed, lut, y, workspace):
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    vp = C.c_void_p * n
    return (n, cs, vp(*[_ptr(t) for t in packed]), vp(*[_ptr(t) for t in lut]), vp(*[_ptr(t) for t in y]),
            vp(*[_ptr(t) for t in workspace]), (C.c_size_t * n)(*[_nbytes(t) for t in workspace]))


def tman_mpgemv_batch_prepare(shapes, packed, lut, N: int, y, workspace, desc, stream=None) -> None:
    """Write the device descriptor table for a batch of GEMVs (lists of equal length; lut entries may
    repeat).  The table is reusable for every step while the buffers stay in place."""
    n, cs, pk, lt, yy, ws, wb = _batch_arrays(shapes, packed, lut, y, workspace)
    _check(_load().tman_mpgemv_batch_prepare(n, cs, pk, lt, N, yy, ws, wb, _ptr(desc), _stream(stream)),
           "tman_mpgemv_batch_prepare")


def tman_mpgemv_batch_run(shapes, N: int, desc, stream=None) -> None:
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    _check(_load().tman_mpgemv_batch_run(n, cs, N, _ptr(desc), _stream(stream)), "tman_mpgemv_batch_run")


def tman_mpgemv_x(shape: Shape, packed, x, y, workspace, stream=None) -> None:
    """y fp16 [M] = x fp16 [K] * dequant(W)^T for one token; the lookup kernel builds its tables itself."""
    wb = 0 if workspace is None or isinstance(workspace, int) else _nbytes(workspace)
    _check(_load().tman_mpgemv_x(C.byref(shape.c()), _ptr(packed), _ptr(x), _ptr(y), _ptr(workspace), wb,
                                 _stream(stream)), "tman_mpgemv_x")


def tman_mpgemv_x_batch_order(shapes, n_units: int = 0):
    """The workgroup numbering of a one-token batch as (gemv, workgroup) pairs; empty for a plain grid."""
    cs = (_CShape * len(shapes))(*[s.c() for s in shapes])
    n = C.c_int32(0)
    _check(_load().tman_mpgemv_x_batch_order(len(shapes), cs, n_units, None, 0, C.byref(n)), "tman_mpgemv_x_batch_order")
    out = (C.c_uint16 * max(1, n.value))()
    _check(_load().tman_mpgemv_x_batch_order(len(shapes), cs, n_units, out, n.value, C.byref(n)),
           "tman_mpgemv_x_batch_order")
    return [(int(out[i]) >> 13, int(out[i]) & 0x1FFF) for i in range(n.value)]


def tman_mpgemv_x_batch_prepare(shapes, packed, xs, y, workspace, desc, stream=None) -> None:
    """Descriptor table for a batch of one-token GEMVs that build their own tables (xs entries may repeat)."""
    n, cs, pk, xx, yy, ws, wb = _batch_arrays(shapes, packed, xs, y, workspace)
    _check(_load().tman_mpgemv_x_batch_prepare(n, cs, pk, xx, yy, ws, wb, _ptr(desc), _stream(stream)),
           "tman_mpgemv_x_batch_prepare")


def tman_mpgemv_x_batch_run(shapes, desc, stream=None) -> None:
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    _check(_load().tman_mpgemv_x_batch_run(n, cs, _ptr(desc), _stream(stream)), "tman_mpgemv_x_batch_run")


def tman_build_lut_batch(xs, N: int, Ks, group: int, luts, stream=None) -> None:
    """Lookup tables for several activations (lists of equal length) in one launch."""
    n = len(xs)
    vp = C.c_void_p * n
    _check(_load().tman_build_lut_batch(n, vp(*[_ptr(t) for t in xs]), N, (C.c_int32 * n)(*Ks), group,
                                        vp(*[_ptr(t) for t in luts]), _stream(stream)), "tman_build_lut_batch")


# Calls that run every decode step with the same arguments can be marshalled once: the returned
# callables only hand the prebuilt ctypes arguments to the C entry point.
def bound_build_lut_batch(xs, N: int, Ks, group: int, luts):
    n = len(xs)
    vp = C.c_void_p * n
    fn, args = _load().tman_build_lut_batch, (n, vp(*[_ptr(t) for t in xs]), N, (C.c_int32 * n)(*Ks), group,
                                               vp(*[_ptr(t) for t in luts]))

    def call(stream_handle):
        _check(fn(*args, stream_handle), "tman_build_lut_batch")

    return call


def bound_build_lut_i16_batch(xs, N: int, Ks, group: int, luts):
    n = len(xs)
    vp = C.c_void_p * n
    fn, args = _load().tman_build_lut_i16_batch, (n, vp(*[_ptr(t) for t in xs]), N, (C.c_int32 * n)(*Ks), group,
                                                   vp(*[_ptr(t) for t in luts]))

    def call(stream_handle):
        _check(fn(*args, stream_handle), "tman_build_lut_i16_batch")

    return call


def bound_mpgemv_i16_batch_run(shapes, N: int, desc):
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    fn, args = _load().tman_mpgemv_i16_batch_run, (n, cs, N, _ptr(desc))

    def call(stream_handle):
        _check(fn(*args, stream_handle), "tman_mpgemv_i16_batch_run")

    return call


def bound_mpgemv_batch_run(shapes, N: int, desc):
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    fn, args = _load().tman_mpgemv_batch_run, (n, cs, N, _ptr(desc))

    def call(stream_handle):
        _check(fn(*args, stream_handle), "tman_mpgemv_batch_run")

    return call


def bound_mpgemv_x_batch_run(shapes, desc):
    n = len(shapes)
    cs = (_CShape * n)(*[s.c() for s in shapes])
    fn, args = _load().tman_mpgemv_x_batch_run, (n, cs, _ptr(desc))

    def call(stream_handle):
        _check(fn(*args, stream_handle), "tman_mpgemv_x_batch_run")

    return call
