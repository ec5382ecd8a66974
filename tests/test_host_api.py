"""CPU-only checks of the C ABI: the library loads, exports what include/zipccl.h declares,
and its host logic (table builder, sizes, argument checking) agrees with the oracle."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import oracle
import paper_2604_27844_amd.binding as z

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "zipccl.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(zipccl_[a-z_]+)\s*\(", hdr))
    assert {"zipccl_build_table", "zipccl_max_compressed_size", "zipccl_compress", "zipccl_decompress"} <= declared
    lib = ctypes.CDLL(z.lib_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(z.EXPORTS)


def test_table_builder_matches_oracle_on_sigma_grid():
    sigmas = np.exp(np.linspace(math.log(1e-40), math.log(1e38), 997))
    for s in list(sigmas) + [0.02, 0.5, 1.0, 1e-4, 0.82335, 0.8233, 0.8234]:
        for dt in (z.BF16, z.FP32):
            assert list(bytes(z.zipccl_build_table(float(s), dt).dec)) == list(oracle.build_table(float(s)))
    for bad in (0.0, -3.0, float("nan"), float("inf")):
        with pytest.raises(z.ZipcclError) as ei:
            z.zipccl_build_table(bad)
        assert ei.value.code == 1
    with pytest.raises(z.ZipcclError) as ei:
        z.zipccl_build_table(1.0, 9)
    assert ei.value.code == 2


def test_sizes_and_offsets_match_oracle():
    rng = np.random.default_rng(0)
    for dt in (z.BF16, z.FP32):
        for _ in range(50):
            k = int(rng.integers(1, 40))
            ce = rng.integers(0, 70000, k).astype(np.uint64)
            ce[rng.integers(0, k)] = 0
            n = int(ce.sum())
            off = z.zipccl_chunk_slot_offsets(n, dt, k, ce)
            assert np.array_equal(off, oracle.slot_offsets(n, dt, k, ce))
            assert z.zipccl_max_compressed_size(n, dt, k, ce) == int(off[-1])
            assert np.all(off % 128 == 0)
        assert z.zipccl_max_compressed_size(1 << 20, dt, 8) == 8 * oracle.slot_cap(1 << 17, dt)
    # sizes near the per-chunk maximum must not overflow
    big = 0xFFFFFFFF
    assert z.zipccl_max_compressed_size(big, z.BF16, 1) == oracle.slot_cap(big, z.BF16)
    assert z.zipccl_max_compressed_size(3 * big, z.FP32, 3) == 3 * oracle.slot_cap(big, z.FP32)
    assert z.zipccl_max_compressed_size(big + 1, z.BF16, 1) == 0          # chunk too large
    assert z.zipccl_max_compressed_size(10, z.BF16, 3) == 0               # equal split must divide
    assert z.zipccl_max_compressed_size(10, z.BF16, 0) == 0
    assert z.zipccl_max_compressed_size(10, z.BF16, 2, [4, 5]) == 0       # must sum to n
    assert z.zipccl_max_compressed_size(10, 5, 1) == 0
    # header + (u32 count + u32 prefix) per tile, each array padded to 16 bytes
    # [+ stash: 1 byte per element + slack]
    assert z.zipccl_compress_min_workspace_size(8192 * 3 + 1, z.BF16, 1) == 256 + 16 + 16
    assert z.zipccl_compress_workspace_size(8192 * 3 + 1, z.BF16, 1) == 256 + 32 + (8192 * 3 + 1 + 64 + 15) // 16 * 16
    assert z.zipccl_compress_min_workspace_size(0, z.BF16, 2, [0, 0]) == 256 + 32
    assert z.zipccl_compress_min_workspace_size(8192 * 4096 * 2, z.BF16, 2) == 256 + 2 * 4 * 8192


def test_static_bytes_match_oracle_layout():
    # static part = everything but the zero-point list: chunk_bytes of a chunk without zero-points
    for dt in (z.BF16, z.FP32):
        ce = np.array([0, 1, 511, 512, 513, 8192, 100000], dtype=np.uint64)
        st = z.zipccl_chunk_static_bytes(int(ce.sum()), dt, len(ce), ce)
        assert [int(v) for v in st] == [oracle.chunk_bytes(int(n), 0, dt) for n in ce]
        assert np.all(st % 128 == 0)
    with pytest.raises(z.ZipcclError):
        z.zipccl_chunk_static_bytes(10, z.BF16, 3)


def test_argument_errors_return_before_any_launch():
    lib = z._lib
    t = z.zipccl_build_table(1.0)
    A = 1 << 20                      # a fake, aligned "device" address: never dereferenced on these paths
    cap = z.zipccl_max_compressed_size(1024, z.BF16, 1)
    ws = z.zipccl_compress_min_workspace_size(1024, z.BF16, 1)

    def comp(d_in=A, n=1024, dt=z.BF16, k=1, ce=None, table=t, out=A, ocap=cap, cb=A, w=A, wb=ws):
        tab = ctypes.byref(table) if table is not None else None
        return lib.zipccl_compress(d_in, n, dt, k, ce, tab, out, ocap, cb, w, wb, None)

    assert comp(dt=3) == 2
    assert comp(k=0) == 1
    assert comp(n=1025, k=2) == 1
    assert comp(table=None) == 1
    assert comp(out=None) == 1
    assert comp(w=None) == 1
    assert comp(d_in=None) == 1
    assert comp(d_in=A + 1) == 1
    assert comp(out=A + 64) == 1
    assert comp(w=A + 8) == 1
    assert comp(ocap=cap - 1) == 3
    assert comp(wb=ws - 1) == 3
    bad = z.zipccl_table_t()
    bad.dec[:] = [0, 120, 121, 122, 124, 125, 126, 127]
    assert comp(table=bad) == 1

    def decomp(comp_=A, ccap=cap, out=A, n=1024, dt=z.BF16, k=1, ce=None, st=A):
        return lib.zipccl_decompress(comp_, ccap, out, n, dt, k, ce, st, None)

    assert decomp(dt=7) == 2
    assert decomp(k=0) == 1
    assert decomp(comp_=None) == 1
    assert decomp(out=None) == 1
    assert decomp(comp_=A + 32) == 1
    assert decomp(out=A + 1) == 1
    assert decomp(ccap=128) == 3      # static part of the slot is not readable
    def sampled(stride, d_in=A, n=1 << 20, dt=z.BF16, k=4, tables=A, ws_=A, wsb=z.zipccl_estimate_chunk_tables_workspace_size(4)):
        return lib.zipccl_estimate_chunk_tables_sampled(d_in, n, dt, k, None, stride, tables, None, ws_, wsb, None)

    for stride in (0, 3, 24, 8192, 1 << 31):              # a power of two from 1 to 4096 is asked for
        assert sampled(stride) == 1, stride
    assert sampled(16, dt=5) == 2
    assert sampled(16, tables=None) == 1
    assert sampled(16, k=3) == 1                          # 2^20 values do not split into 3 equal chunks
    assert sampled(16, wsb=100) == 3
    assert z.zipccl_status_string(4) == "corrupt compressed data"
