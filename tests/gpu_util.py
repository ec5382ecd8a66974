"""Helpers for the GPU parity tests: run the HIP path through the C ABI binding and compare
with the CPU oracle byte for byte over the transmitted range of every slot."""
import numpy as np
import torch

import oracle
import paper_2604_27844_amd.binding as z

DEV = "cuda:0"


def to_device_words(data):
    """uint16 / uint32 numpy words -> int16 / int32 torch tensor on the GPU (same bytes)."""
    signed = np.int16 if data.dtype == np.uint16 else np.int32
    return torch.from_numpy(np.ascontiguousarray(data).view(signed)).to(DEV)


def gpu_compress(data, dtype, sigma, n_chunks=1, chunk_elems=None, table=None, d_in=None, reread=False):
    """reread: hand zipccl_compress only its minimum workspace, which selects the form that reads the input
    twice (count, prefix, emit) instead of the single pass with a stash."""
    n = int(data.size)
    table = table if table is not None else z.zipccl_build_table(sigma, dtype)
    cap = z.zipccl_max_compressed_size(n, dtype, n_chunks, chunk_elems)
    assert cap > 0
    d_in = to_device_words(data) if d_in is None else d_in
    d_out = torch.full((cap,), 0xA5, dtype=torch.uint8, device=DEV)      # poison
    d_cb = torch.full((n_chunks,), -1, dtype=torch.int64, device=DEV)
    ws = z.zipccl_compress_workspace_size(n, dtype, n_chunks, chunk_elems)
    d_ws = torch.full((ws,), 0x5A, dtype=torch.uint8, device=DEV)
    wsb = z.zipccl_compress_min_workspace_size(n, dtype, n_chunks, chunk_elems) if reread else None
    z.zipccl_compress(d_in, n, dtype, n_chunks, chunk_elems, table, d_out, d_cb, d_ws, workspace_bytes=wsb)
    torch.cuda.synchronize()
    return d_out, d_cb, table


def gpu_decompress(d_comp, n, dtype, n_chunks=1, chunk_elems=None, comp_capacity=None):
    d_back = torch.full((n,), 0x5B5B if dtype == z.BF16 else 0x5B5B5B5B,
                        dtype=torch.int16 if dtype == z.BF16 else torch.int32, device=DEV)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    z.zipccl_decompress(d_comp, d_back, n, dtype, n_chunks, chunk_elems, d_st, comp_capacity=comp_capacity)
    torch.cuda.synchronize()
    words = np.uint16 if dtype == z.BF16 else np.uint32
    return d_back.cpu().numpy().view(words), int(d_st.item())


def check_parity(data, dtype, sigma, n_chunks=1, chunk_elems=None, label="", reread=False):
    """GPU compressed bytes, chunk sizes and decoded words must equal the oracle's."""
    n = int(data.size)
    dec = oracle.build_table(sigma)
    ref, ref_cb, off = oracle.compress(data, dtype, dec, n_chunks, chunk_elems)
    d_out, d_cb, table = gpu_compress(data, dtype, sigma, n_chunks, chunk_elems, reread=reread)
    assert list(bytes(table.dec)) == list(dec), f"{label}: table differs"
    got = d_out.cpu().numpy()
    got_cb = d_cb.cpu().numpy().astype(np.uint64)
    assert np.array_equal(got_cb, ref_cb), f"{label}: chunk_bytes differ {got_cb[:8]} vs {ref_cb[:8]}"
    assert got.size == int(off[-1])
    for c in range(n_chunks):
        s, e = int(off[c]), int(off[c]) + int(ref_cb[c])
        if not np.array_equal(got[s:e], ref[s:e]):
            bad = np.nonzero(got[s:e] != ref[s:e])[0]
            raise AssertionError(f"{label}: chunk {c} differs at {bad.size} bytes, first slot offsets {bad[:8]}, "
                                 f"got {got[s:e][bad[:8]]} want {ref[s:e][bad[:8]]}")
        # bytes of the slot past the transmitted range must be left untouched (still poison)
        assert np.all(got[e:int(off[c + 1])] == 0xA5), f"{label}: chunk {c} wrote past chunk_bytes"
    back, st = gpu_decompress(d_out, n, dtype, n_chunks, chunk_elems)
    assert st == 0, f"{label}: decompress status {st}"
    assert np.array_equal(back, data), f"{label}: GPU round trip differs"
    # the GPU decoder must also accept the oracle's stream (it is the same bytes, but from host)
    d_ref = torch.from_numpy(ref).to(DEV)
    back2, st2 = gpu_decompress(d_ref, n, dtype, n_chunks, chunk_elems)
    assert st2 == 0 and np.array_equal(back2, data), f"{label}: GPU decode of oracle stream differs"
    return got, got_cb, off
