"""CPU oracle for the ZipCCL exponent-coding format.  TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may import
this package.  It shares nothing with the HIP library.
"""
from .zipccl_oracle import (  # noqa: F401
    BF16, FP32, G_DEFAULT, build, build_table, pwin, xopt, slot_cap, chunk_bytes,
    slot_offsets, compress, decompress, decompress_reduce, OracleError,
)
