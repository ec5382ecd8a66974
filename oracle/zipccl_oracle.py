"""ctypes front end of ``zipccl_oracle.c`` (plain scalar C, compiled with gcc -O2).

TEST INFRASTRUCTURE ONLY -- see the header of the C file.  Argument marshalling only;
all of the oracle's arithmetic lives in the C file so that it can be read against the
paper (section 4, section 4.1 Eq.2/Eq.5, section 4.2.1, section 4.2.3) in one place.
"""
import ctypes
import os
import subprocess

import numpy as np

BF16, FP32 = 0, 1
G_DEFAULT = 512
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zipccl_oracle.c")
_LIB = os.path.join(_HERE, "libzipccl_oracle.so")
_lib = None


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


def build(force=False):
    """Compile the oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, u32, i32, dbl, vp = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_double,
                                  ctypes.c_void_p)
        lib.zo_pwin.restype = dbl
        lib.zo_pwin.argtypes = [dbl, i32]
        lib.zo_xopt.restype = dbl
        lib.zo_xopt.argtypes = [dbl]
        lib.zo_build_table.restype = i32
        lib.zo_build_table.argtypes = [dbl, vp]
        lib.zo_slot_cap.restype = u64
        lib.zo_slot_cap.argtypes = [u64, i32, u32]
        lib.zo_chunk_bytes.restype = u64
        lib.zo_chunk_bytes.argtypes = [u64, u64, i32, u32]
        lib.zo_slot_offsets.restype = i32
        lib.zo_slot_offsets.argtypes = [u64, i32, u32, u32, vp, vp]
        lib.zo_compress.restype = i32
        lib.zo_compress.argtypes = [vp, u64, i32, u32, u32, vp, vp, vp, u64, vp]
        lib.zo_decompress.restype = i32
        lib.zo_decompress.argtypes = [vp, u64, vp, u64, i32, u32, vp]
        lib.zo_decompress_reduce.restype = i32
        lib.zo_decompress_reduce.argtypes = [vp, u64, vp, u64, i32, u32, i32, vp, vp]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chunks(chunk_elems):
    if chunk_elems is None:
        return None
    return np.ascontiguousarray(np.asarray(chunk_elems, dtype=np.uint64))


def _raw(x, dtype):
    """View the input as a flat byte array; bf16 data is carried as uint16 words."""
    x = np.ascontiguousarray(x)
    es = {BF16: 2, FP32: 4}.get(dtype)     # unknown codes go through to the C side, which rejects them
    if es is not None and x.dtype.itemsize != es:
        raise ValueError(f"dtype code {dtype} needs {es}-byte elements, got {x.dtype}")
    return x.reshape(-1).view(np.uint8), x.size


def pwin(sigma, x):
    return _load().zo_pwin(float(sigma), int(x))


def xopt(sigma):
    return _load().zo_xopt(float(sigma))


def build_table(sigma):
    dec = np.zeros(8, dtype=np.uint8)
    rc = _load().zo_build_table(float(sigma), _ptr(dec))
    if rc:
        raise OracleError(rc, "build_table")
    return dec


def slot_cap(n, dtype, G=G_DEFAULT):
    return int(_load().zo_slot_cap(int(n), dtype, G))


def chunk_bytes(n, n_esc, dtype, G=G_DEFAULT):
    return int(_load().zo_chunk_bytes(int(n), int(n_esc), dtype, G))


def slot_offsets(n_elems, dtype, n_chunks, chunk_elems=None, G=G_DEFAULT):
    ce = _chunks(chunk_elems)
    off = np.zeros(n_chunks + 1, dtype=np.uint64)
    rc = _load().zo_slot_offsets(int(n_elems), dtype, G, n_chunks, _ptr(ce), _ptr(off))
    if rc:
        raise OracleError(rc, "slot_offsets")
    return off


def compress(x, dtype, dec, n_chunks=1, chunk_elems=None, G=G_DEFAULT, out=None):
    """Returns (out_bytes uint8[capacity], chunk_bytes uint64[n_chunks], slot_off uint64[n_chunks+1])."""
    raw, n = _raw(x, dtype)
    ce = _chunks(chunk_elems)
    off = slot_offsets(n, dtype, n_chunks, ce, G)
    cap = int(off[-1])
    if out is None:
        out = np.full(cap, 0xA5, dtype=np.uint8)  # poison: unwritten bytes show up in comparisons
    dec = np.ascontiguousarray(np.asarray(dec, dtype=np.uint8))
    cb = np.zeros(n_chunks, dtype=np.uint64)
    rc = _load().zo_compress(_ptr(raw), n, dtype, G, n_chunks, _ptr(ce), _ptr(dec), _ptr(out), out.size,
                             _ptr(cb))
    if rc:
        raise OracleError(rc, "compress")
    return out, cb, off


def decompress(comp, n_elems, dtype, n_chunks=1, chunk_elems=None):
    """Returns the decoded tensor as uint16 (bf16 words) or uint32 (fp32 words)."""
    comp = np.ascontiguousarray(comp).view(np.uint8)
    ce = _chunks(chunk_elems)
    out = np.zeros(int(n_elems), dtype=np.uint16 if dtype == BF16 else np.uint32)
    rc = _load().zo_decompress(_ptr(comp), comp.size, _ptr(out), int(n_elems), dtype, n_chunks, _ptr(ce))
    if rc:
        raise OracleError(rc, "decompress")
    return out


def decompress_reduce(comp, n_elems, dtype, n_peers, out_dtype=FP32):
    """Decode n_peers back-to-back slots of n_elems values each and sum them in fp32, peers in order.
    Returns uint32 words of the fp32 sums (out_dtype FP32) or uint16 bf16 words (out_dtype BF16)."""
    comp = np.ascontiguousarray(comp).view(np.uint8)
    n = int(n_elems)
    out = np.zeros(n, dtype=np.uint32 if out_dtype == FP32 else np.uint16)
    scratch = np.zeros(n, dtype=np.uint16 if dtype == BF16 else np.uint32)
    acc = np.zeros(n, dtype=np.float32)
    rc = _load().zo_decompress_reduce(_ptr(comp), comp.size, _ptr(out), n, dtype, int(n_peers), out_dtype,
                                      _ptr(scratch), _ptr(acc))
    if rc:
        raise OracleError(rc, "decompress_reduce")
    return out
