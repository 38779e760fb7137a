"""NestedFP CPU oracle -- TEST INFRASTRUCTURE, not part of the product path.

Thin ctypes/numpy access to ``nestedfp_oracle.c`` (plain C, fp64).  Only the
tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package; the HIP library and its Python binding never do, and
this package imports nothing from them.
"""
from .nestedfp_oracle import (  # noqa: F401
    build_oracle,
    fp16_value,
    e4m3_value,
    e4m3_encode,
    in_range,
    decompose,
    decompose_one,
    reconstruct,
    reconstruct_one,
    count_out_of_range,
    quantize_act,
    gemm_fp16,
    gemm_fp16_planes,
    gemm_fp8,
    dot_fp16,
    dot_fp8,
)
