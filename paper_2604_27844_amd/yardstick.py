"""ctypes binding of libzipccl_yardstick.so: the plain-copy kernel the benchmark and the counter runs measure
against (include/zipccl_yardstick.h).  A measurement aid; the codec library does not contain it."""
import ctypes
import os

from . import build_lib
from .binding import _dptr, _stream

_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(build_lib.YARDSTICK):
            build_lib.build(lib=build_lib.YARDSTICK)
        lib = ctypes.CDLL(build_lib.YARDSTICK)
        lib.zipccl_yardstick_copy.restype = ctypes.c_int
        lib.zipccl_yardstick_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        _lib = lib
    return _lib


def zipccl_yardstick_copy(d_dst, d_src, nbytes, stream=None):
    rc = _load().zipccl_yardstick_copy(_dptr(d_dst), _dptr(d_src), int(nbytes), _stream(stream))
    if rc:
        raise RuntimeError(f"zipccl_yardstick_copy failed with code {rc}")
