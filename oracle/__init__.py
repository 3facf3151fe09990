"""CPU oracle for the T-MAN hot path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  It shares no code with ``paper_2511_11248_amd`` and neither imports the other.
"""
from .oracle import (  # noqa: F401
    build,
    lib,
    matmul,
    lut_matmul,
    quantize_activations,
    matmul_real_x,
    lut_matmul_i16,
    quantize_activations_i8,
    matmul_i8,
    table_dequant_matmul,
    build_tables,
    lut_indices,
    repack_entry,
    dequant_table,
    half_to_double,
    double_to_half,
    row_relative_error,
)
from .layout_ref import (  # noqa: F401
    PackedLayout,
    pack_reference,
    unpack_reference,
    lut_layout_decode,
)
