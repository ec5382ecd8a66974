"""MI355X-native ZipCCL exponent-coding codec (compress / decompress hot path).

The product is ``libzipccl.so`` (HIP kernels for gfx950 behind a C ABI, see
``include/zipccl.h``).  ``binding`` is a thin ctypes layer with the same names.
``workloads`` holds only seeded input generators.
"""

_BINDING_NAMES = (
    "zipccl_build_table", "zipccl_max_compressed_size", "zipccl_chunk_slot_offsets", "zipccl_chunk_static_bytes",
    "zipccl_compress_workspace_size", "zipccl_compress_min_workspace_size", "zipccl_compress", "zipccl_decompress", "zipccl_decompress_reduce",
    "zipccl_status_string", "zipccl_switch_prefers_zipped", "zipccl_fit_link_model", "zipccl_estimate_workspace_size", "zipccl_estimate_table",
    "zipccl_compress_device_table", "zipccl_estimate_robust_workspace_size", "zipccl_estimate_table_robust", "zipccl_compress_static", "zipccl_estimate_chunk_tables_workspace_size", "zipccl_estimate_chunk_tables", "zipccl_estimate_chunk_tables_sampled", "zipccl_compress_chunk_tables", "ZipcclError", "BF16", "FP32", "GROUP", "lib_path",
)


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        import importlib
        b = importlib.import_module(__name__ + ".binding")
        return b if name == "binding" else getattr(b, name)
    raise AttributeError(name)
