"""ctypes binding of libzipccl.so: same names as include/zipccl.h, argument marshalling only.

Device buffers are torch tensors (PyTorch-ROCm owns memory and streams); every step of the
path runs in the library's HIP kernels.  There is no fallback: a missing library is an error.
"""
import ctypes
import os

import numpy as np

from . import build_lib

BF16, FP32 = 0, 1
GROUP = 512
_STATUS = {0: "ZIPCCL_OK", 1: "ZIPCCL_ERR_INVALID_ARG", 2: "ZIPCCL_ERR_UNSUPPORTED_DTYPE",
           3: "ZIPCCL_ERR_BUFFER_TOO_SMALL", 4: "ZIPCCL_ERR_CORRUPT", 5: "ZIPCCL_ERR_DEVICE"}


class ZipcclError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        super().__init__(f"{where}: {_STATUS.get(self.code, self.code)} ({zipccl_status_string(self.code)})")


class zipccl_table_t(ctypes.Structure):
    _fields_ = [("dec", ctypes.c_uint8 * 8)]


class zipccl_link_model_t(ctypes.Structure):
    _fields_ = [("alpha_rs", ctypes.c_double), ("beta_rs", ctypes.c_double),
                ("alpha_a2a", ctypes.c_double), ("beta_a2a", ctypes.c_double)]


def lib_path():
    return build_lib.LIB


def _load():
    path = lib_path()
    if not os.path.exists(path):
        # tests, smoke() and bench.py load what is built and build only if nothing is there
        build_lib.build(lib=path)
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run __graft_entry__.build() (hipcc, gfx950) first")
    lib = ctypes.CDLL(path)
    u64, u32, sz, vp, i32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int
    tp = ctypes.POINTER(zipccl_table_t)
    lib.zipccl_build_table.restype = i32
    lib.zipccl_build_table.argtypes = [ctypes.c_double, i32, tp]
    lib.zipccl_max_compressed_size.restype = sz
    lib.zipccl_max_compressed_size.argtypes = [sz, i32, u32, vp]
    lib.zipccl_chunk_slot_offsets.restype = i32
    lib.zipccl_chunk_slot_offsets.argtypes = [sz, i32, u32, vp, vp]
    lib.zipccl_chunk_static_bytes.restype = i32
    lib.zipccl_chunk_static_bytes.argtypes = [sz, i32, u32, vp, vp]
    lib.zipccl_compress_workspace_size.restype = sz
    lib.zipccl_compress_workspace_size.argtypes = [sz, i32, u32, vp]
    lib.zipccl_compress_min_workspace_size.restype = sz
    lib.zipccl_compress_min_workspace_size.argtypes = [sz, i32, u32, vp]
    lib.zipccl_compress.restype = i32
    lib.zipccl_compress.argtypes = [vp, sz, i32, u32, vp, tp, vp, sz, vp, vp, sz, vp]
    lib.zipccl_estimate_chunk_tables_workspace_size.restype = sz
    lib.zipccl_estimate_chunk_tables_workspace_size.argtypes = [u32]
    lib.zipccl_estimate_chunk_tables.restype = i32
    lib.zipccl_estimate_chunk_tables.argtypes = [vp, sz, i32, u32, vp, vp, vp, vp, sz, vp]
    lib.zipccl_estimate_chunk_tables_sampled.restype = i32
    lib.zipccl_estimate_chunk_tables_sampled.argtypes = [vp, sz, i32, u32, vp, u32, vp, vp, vp, sz, vp]
    lib.zipccl_compress_chunk_tables.restype = i32
    lib.zipccl_compress_chunk_tables.argtypes = [vp, sz, i32, u32, vp, vp, vp, sz, vp, vp, sz, vp]
    lib.zipccl_compress_static.restype = i32
    lib.zipccl_compress_static.argtypes = [vp, sz, i32, u32, vp, tp, vp, sz, vp, vp]
    lib.zipccl_compress_device_table.restype = i32
    lib.zipccl_compress_device_table.argtypes = [vp, sz, i32, u32, vp, vp, vp, sz, vp, vp, sz, vp]
    lib.zipccl_estimate_workspace_size.restype = sz
    lib.zipccl_estimate_workspace_size.argtypes = []
    lib.zipccl_estimate_table.restype = i32
    lib.zipccl_estimate_table.argtypes = [vp, sz, i32, vp, vp, vp, sz, vp]
    lib.zipccl_decompress.restype = i32
    lib.zipccl_decompress.argtypes = [vp, sz, vp, sz, i32, u32, vp, vp, vp]
    lib.zipccl_estimate_robust_workspace_size.restype = sz
    lib.zipccl_estimate_robust_workspace_size.argtypes = []
    lib.zipccl_estimate_table_robust.restype = i32
    lib.zipccl_estimate_table_robust.argtypes = [vp, sz, i32, vp, vp, vp, sz, vp]
    lib.zipccl_decompress_reduce.restype = i32
    lib.zipccl_decompress_reduce.argtypes = [vp, sz, vp, sz, i32, u32, i32, vp, vp]
    dp = ctypes.POINTER(ctypes.c_double)
    lib.zipccl_switch_prefers_zipped.restype = i32
    lib.zipccl_switch_prefers_zipped.argtypes = [ctypes.POINTER(zipccl_link_model_t), ctypes.c_double,
                                                 ctypes.c_double, ctypes.c_double, dp, dp]
    lib.zipccl_fit_link_model.restype = i32
    lib.zipccl_fit_link_model.argtypes = [dp, dp, sz, dp, dp]
    lib.zipccl_status_string.restype = ctypes.c_char_p
    lib.zipccl_status_string.argtypes = [i32]
    return lib


_lib = _load()
EXPORTS = ("zipccl_build_table", "zipccl_max_compressed_size", "zipccl_chunk_slot_offsets", "zipccl_chunk_static_bytes",
           "zipccl_compress_workspace_size", "zipccl_compress_min_workspace_size", "zipccl_compress", "zipccl_decompress", "zipccl_decompress_reduce", "zipccl_status_string",
           "zipccl_switch_prefers_zipped", "zipccl_fit_link_model",
           "zipccl_estimate_workspace_size", "zipccl_estimate_table", "zipccl_compress_device_table",
           "zipccl_estimate_robust_workspace_size", "zipccl_estimate_table_robust", "zipccl_compress_static",
           "zipccl_estimate_chunk_tables_workspace_size", "zipccl_estimate_chunk_tables", "zipccl_estimate_chunk_tables_sampled",
           "zipccl_compress_chunk_tables")


def _host_u64(chunk_elems):
    if chunk_elems is None:
        return None, None
    a = np.ascontiguousarray(np.asarray(chunk_elems, dtype=np.uint64))
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _dptr(t):
    """Device address of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device buffers must be contiguous tensors on the GPU")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def zipccl_status_string(code):
    return _lib.zipccl_status_string(int(code)).decode()


def zipccl_build_table(sigma, dt=BF16):
    t = zipccl_table_t()
    rc = _lib.zipccl_build_table(float(sigma), dt, ctypes.byref(t))
    if rc:
        raise ZipcclError(rc, "zipccl_build_table")
    return t


def zipccl_max_compressed_size(n_elems, dt, n_chunks=1, chunk_elems=None):
    _keep, p = _host_u64(chunk_elems)
    return int(_lib.zipccl_max_compressed_size(int(n_elems), dt, int(n_chunks), p))


def zipccl_chunk_slot_offsets(n_elems, dt, n_chunks=1, chunk_elems=None):
    _keep, p = _host_u64(chunk_elems)
    off = np.zeros(int(n_chunks) + 1, dtype=np.uint64)
    rc = _lib.zipccl_chunk_slot_offsets(int(n_elems), dt, int(n_chunks), p, off.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ZipcclError(rc, "zipccl_chunk_slot_offsets")
    return off


def zipccl_compress_workspace_size(n_elems, dt, n_chunks=1, chunk_elems=None):
    _keep, p = _host_u64(chunk_elems)
    return int(_lib.zipccl_compress_workspace_size(int(n_elems), dt, int(n_chunks), p))


def zipccl_compress_min_workspace_size(n_elems, dt, n_chunks=1, chunk_elems=None):
    _keep, p = _host_u64(chunk_elems)
    return int(_lib.zipccl_compress_min_workspace_size(int(n_elems), dt, int(n_chunks), p))


def zipccl_compress(d_in, n_elems, dt, n_chunks, chunk_elems, table, d_out, d_chunk_bytes, d_workspace,
                    stream=None, out_capacity=None, workspace_bytes=None):
    """d_in / d_out / d_chunk_bytes / d_workspace are torch GPU tensors (any dtype; raw bytes)."""
    _keep, p = _host_u64(chunk_elems)
    cap = d_out.numel() * d_out.element_size() if out_capacity is None else int(out_capacity)
    wsb = d_workspace.numel() * d_workspace.element_size() if workspace_bytes is None else int(workspace_bytes)
    rc = _lib.zipccl_compress(_dptr(d_in), int(n_elems), dt, int(n_chunks), p, ctypes.byref(table),
                              _dptr(d_out), cap, _dptr(d_chunk_bytes), _dptr(d_workspace), wsb, _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_compress")


def zipccl_compress_static(d_in, n_elems, dt, n_chunks, chunk_elems, table, d_out, d_chunk_bytes, stream=None,
                           out_capacity=None):
    """zipccl_compress with the library's own fixed workspace (no allocation, no workspace argument)."""
    _keep, p = _host_u64(chunk_elems)
    cap = d_out.numel() * d_out.element_size() if out_capacity is None else int(out_capacity)
    rc = _lib.zipccl_compress_static(_dptr(d_in), int(n_elems), dt, int(n_chunks), p, ctypes.byref(table),
                                     _dptr(d_out), cap, _dptr(d_chunk_bytes), _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_compress_static")


def zipccl_decompress(d_comp, d_out, n_elems, dt, n_chunks=1, chunk_elems=None, d_status=None, stream=None,
                      comp_capacity=None):
    _keep, p = _host_u64(chunk_elems)
    cap = d_comp.numel() * d_comp.element_size() if comp_capacity is None else int(comp_capacity)
    rc = _lib.zipccl_decompress(_dptr(d_comp), cap, _dptr(d_out), int(n_elems), dt, int(n_chunks), p,
                                _dptr(d_status), _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_decompress")


def zipccl_decompress_reduce(d_comp, d_out, n_elems, dt, n_peers, out_dt=FP32, d_status=None, stream=None,
                             comp_capacity=None):
    cap = d_comp.numel() * d_comp.element_size() if comp_capacity is None else int(comp_capacity)
    rc = _lib.zipccl_decompress_reduce(_dptr(d_comp), cap, _dptr(d_out), int(n_elems), dt, int(n_peers), out_dt,
                                       _dptr(d_status), _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_decompress_reduce")


def zipccl_switch_prefers_zipped(alpha_rs, beta_rs, alpha_a2a, beta_a2a, d_bytes, e, s):
    """Returns (decision, t_rs, t_a2a); decision is 1, 0 or -1 (bad arguments)."""
    m = zipccl_link_model_t(alpha_rs, beta_rs, alpha_a2a, beta_a2a)
    t_rs, t_a2a = ctypes.c_double(), ctypes.c_double()
    r = _lib.zipccl_switch_prefers_zipped(ctypes.byref(m), d_bytes, e, s, ctypes.byref(t_rs), ctypes.byref(t_a2a))
    return int(r), t_rs.value, t_a2a.value


def zipccl_fit_link_model(d_bytes, t_seconds):
    d = (ctypes.c_double * len(d_bytes))(*d_bytes)
    t = (ctypes.c_double * len(t_seconds))(*t_seconds)
    a, b = ctypes.c_double(), ctypes.c_double()
    rc = _lib.zipccl_fit_link_model(d, t, len(d_bytes), ctypes.byref(a), ctypes.byref(b))
    if rc:
        raise ZipcclError(rc, "zipccl_fit_link_model")
    return a.value, b.value


def zipccl_estimate_workspace_size():
    return int(_lib.zipccl_estimate_workspace_size())


def zipccl_estimate_table(d_in, n_elems, dt, d_table, d_sigma, d_workspace, stream=None):
    """d_table: 8-byte GPU tensor; d_sigma: float64 GPU tensor of one element or None."""
    wsb = d_workspace.numel() * d_workspace.element_size()
    rc = _lib.zipccl_estimate_table(_dptr(d_in), int(n_elems), dt, _dptr(d_table), _dptr(d_sigma),
                                    _dptr(d_workspace), wsb, _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_estimate_table")


def zipccl_estimate_robust_workspace_size():
    return int(_lib.zipccl_estimate_robust_workspace_size())


def zipccl_estimate_table_robust(d_in, n_elems, dt, d_table, d_sigma, d_workspace, stream=None):
    """As zipccl_estimate_table, with sigma = median of the magnitudes / Phi^-1(3/4)."""
    wsb = d_workspace.numel() * d_workspace.element_size()
    rc = _lib.zipccl_estimate_table_robust(_dptr(d_in), int(n_elems), dt, _dptr(d_table), _dptr(d_sigma),
                                           _dptr(d_workspace), wsb, _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_estimate_table_robust")


def zipccl_estimate_chunk_tables_workspace_size(n_chunks):
    return int(_lib.zipccl_estimate_chunk_tables_workspace_size(int(n_chunks)))


def zipccl_estimate_chunk_tables(d_in, n_elems, dt, n_chunks, chunk_elems, d_tables, d_sigmas, d_workspace, stream=None):
    """d_tables: 8 * n_chunks bytes on the GPU; d_sigmas: n_chunks float64 on the GPU or None."""
    _keep, p = _host_u64(chunk_elems)
    wsb = d_workspace.numel() * d_workspace.element_size()
    rc = _lib.zipccl_estimate_chunk_tables(_dptr(d_in), int(n_elems), dt, int(n_chunks), p, _dptr(d_tables),
                                           _dptr(d_sigmas), _dptr(d_workspace), wsb, _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_estimate_chunk_tables")


def zipccl_estimate_chunk_tables_sampled(d_in, n_elems, dt, n_chunks, chunk_elems, sample_stride, d_tables, d_sigmas,
                                         d_workspace, stream=None):
    """As zipccl_estimate_chunk_tables, from one group of 512 values per sample_stride groups of every chunk."""
    _keep, p = _host_u64(chunk_elems)
    wsb = d_workspace.numel() * d_workspace.element_size()
    rc = _lib.zipccl_estimate_chunk_tables_sampled(_dptr(d_in), int(n_elems), dt, int(n_chunks), p, int(sample_stride),
                                                   _dptr(d_tables), _dptr(d_sigmas), _dptr(d_workspace), wsb,
                                                   _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_estimate_chunk_tables_sampled")


def zipccl_compress_chunk_tables(d_in, n_elems, dt, n_chunks, chunk_elems, d_tables, d_out, d_chunk_bytes,
                                 d_workspace, stream=None, workspace_bytes=None):
    _keep, p = _host_u64(chunk_elems)
    cap = d_out.numel() * d_out.element_size()
    wsb = d_workspace.numel() * d_workspace.element_size() if workspace_bytes is None else int(workspace_bytes)
    rc = _lib.zipccl_compress_chunk_tables(_dptr(d_in), int(n_elems), dt, int(n_chunks), p, _dptr(d_tables),
                                           _dptr(d_out), cap, _dptr(d_chunk_bytes), _dptr(d_workspace), wsb,
                                           _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_compress_chunk_tables")


def zipccl_compress_device_table(d_in, n_elems, dt, n_chunks, chunk_elems, d_table, d_out, d_chunk_bytes,
                                 d_workspace, stream=None, workspace_bytes=None):
    _keep, p = _host_u64(chunk_elems)
    cap = d_out.numel() * d_out.element_size()
    wsb = d_workspace.numel() * d_workspace.element_size() if workspace_bytes is None else int(workspace_bytes)
    rc = _lib.zipccl_compress_device_table(_dptr(d_in), int(n_elems), dt, int(n_chunks), p, _dptr(d_table),
                                           _dptr(d_out), cap, _dptr(d_chunk_bytes), _dptr(d_workspace), wsb,
                                           _stream(stream))
    if rc:
        raise ZipcclError(rc, "zipccl_compress_device_table")


def zipccl_chunk_static_bytes(n_elems, dt, n_chunks=1, chunk_elems=None):
    _keep, p = _host_u64(chunk_elems)
    out = np.zeros(int(n_chunks), dtype=np.uint64)
    rc = _lib.zipccl_chunk_static_bytes(int(n_elems), dt, int(n_chunks), p, out.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ZipcclError(rc, "zipccl_chunk_static_bytes")
    return out
