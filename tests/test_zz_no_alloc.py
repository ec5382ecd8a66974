"""zipccl_compress_static (the entry point that allocates nothing: its workspace is a fixed array inside the
library's device code) against zipccl_compress, through the C ABI: the same bytes, on calls in a row that share the
array, each smaller or differently shaped than the one before."""
import numpy as np
import pytest
import torch

import paper_2604_27844_amd.binding as z
from paper_2604_27844_amd import workloads as W

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DEV, to_device_words

LIMIT = 32 << 20


def _both(data, dtype, sigma, n_chunks, chunk_elems, label):
    """Compress with the caller-workspace entry point and with the static one into poisoned buffers; everything
    must be equal: written bytes, untouched bytes, chunk_bytes."""
    n = int(data.size)
    print(f"[static] {label}: n={n} chunks={n_chunks}", flush=True)
    table = z.zipccl_build_table(sigma, dtype)
    cap = z.zipccl_max_compressed_size(n, dtype, n_chunks, chunk_elems)
    d_in = to_device_words(data)
    ws = z.zipccl_compress_workspace_size(n, dtype, n_chunks, chunk_elems)
    # the existing entry point in the form the static one will take: single pass if its workspace fits the array
    d_ws = torch.full((ws,), 0x5A, dtype=torch.uint8, device=DEV)
    wsb = None if ws <= LIMIT else z.zipccl_compress_min_workspace_size(n, dtype, n_chunks, chunk_elems)
    want = torch.full((cap,), 0xA5, dtype=torch.uint8, device=DEV)
    want_cb = torch.full((n_chunks,), -1, dtype=torch.int64, device=DEV)
    z.zipccl_compress(d_in, n, dtype, n_chunks, chunk_elems, table, want, want_cb, d_ws, workspace_bytes=wsb)
    got = torch.full((cap,), 0xA5, dtype=torch.uint8, device=DEV)
    got_cb = torch.full((n_chunks,), -1, dtype=torch.int64, device=DEV)
    z.zipccl_compress_static(d_in, n, dtype, n_chunks, chunk_elems, table, got, got_cb)
    torch.cuda.synchronize()
    assert torch.equal(got_cb, want_cb), label
    assert torch.equal(got, want), label
    # and it decodes to the input
    d_back = torch.zeros_like(d_in)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    z.zipccl_decompress(got, d_back, n, dtype, n_chunks, chunk_elems, d_st)
    torch.cuda.synchronize()
    assert int(d_st.item()) == 0 and torch.equal(d_back, d_in), label


def test_static_workspace_compress_equals_compress_on_calls_in_a_row():
    rng = np.random.default_rng(21)
    # 1: larger than the array holds a stash for (two reads of the input), 8 chunks
    big = W.f32_to_bf16_words(rng.standard_normal(40_000_000, dtype=np.float32) * np.float32(0.02))
    big[::3] = 0x7F80                                                  # many zero-points: a busy stash / list
    _both(big, z.BF16, 0.02, 8, None, "two-read form")
    # 2: smaller, ragged with an empty chunk, single read with a stash in the same array
    ce = np.array([100_000, 0, 8192 * 7 + 5, 1, 300_001], dtype=np.uint64)
    mid = W.f32_to_bf16_words(rng.standard_normal(int(ce.sum()), dtype=np.float32))
    _both(mid, z.BF16, 1.0, len(ce), ce, "ragged, smaller")
    # 3: smaller again, fp32, one chunk
    small = (rng.standard_normal(50_001, dtype=np.float32) * np.float32(0.5)).view(np.uint32).copy()
    _both(small, z.FP32, 0.5, 1, None, "fp32, smaller again")
    # 4: a workload shape, larger than the previous call
    w = W.make("c2", 1 / 8)
    _both(w.data, w.dtype, w.sigma, w.n_chunks, w.chunk_elems, w.name)
    # 5: nothing at all
    _both(np.zeros(0, dtype=np.uint16), z.BF16, 1.0, 1, None, "empty")


def test_static_workspace_compress_rejects_what_does_not_fit_and_bad_arguments():
    d_in = torch.zeros(16, dtype=torch.int16, device=DEV)
    d_out = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    table = z.zipccl_build_table(1.0, z.BF16)
    # 16 chunks of 2^31 values: 4 194 304 tiles need 32 MiB + 256 bytes of workspace.  Rejected before anything is
    # launched (the capacity given is only a number; no byte of it is touched).
    n = 16 << 31
    assert z.zipccl_compress_min_workspace_size(n, z.BF16, 16) > LIMIT
    with pytest.raises(z.ZipcclError) as ei:
        z.zipccl_compress_static(d_in, n, z.BF16, 16, None, table, d_out, None, out_capacity=1 << 62)
    assert ei.value.code == 3
    with pytest.raises(z.ZipcclError) as ei:                           # not a split
        z.zipccl_compress_static(d_in, 10, z.BF16, 3, None, table, d_out, None)
    assert ei.value.code == 1
    with pytest.raises(z.ZipcclError) as ei:                           # output too small
        z.zipccl_compress_static(d_in, 16, z.BF16, 1, None, table, d_out[:128], None)
    assert ei.value.code == 3
    torch.cuda.synchronize()


def test_static_workspace_compress_replays_inside_a_hip_graph():
    """What the entry point is for: captured once (after a first call outside the capture, which looks up the
    array's address), replayed on fresh input contents with the program's own eager work in between; every replay
    must equal zipccl_compress on the same input."""
    rng = np.random.default_rng(22)
    ce = np.array([8192 * 5 + 3, 0, 20000, 8192 * 2], dtype=np.uint64)
    n, C = int(ce.sum()), len(ce)
    table = z.zipccl_build_table(0.3, z.BF16)
    cap = z.zipccl_max_compressed_size(n, z.BF16, C, ce)
    d_in = torch.zeros(n, dtype=torch.int16, device=DEV)
    got = torch.empty(cap, dtype=torch.uint8, device=DEV)
    got_cb = torch.zeros(C, dtype=torch.int64, device=DEV)
    want = torch.empty(cap, dtype=torch.uint8, device=DEV)
    want_cb = torch.zeros(C, dtype=torch.int64, device=DEV)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(n, z.BF16, C, ce), dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                              # first call on this GPU: outside the capture
        z.zipccl_compress_static(d_in, n, z.BF16, C, ce, table, got, got_cb)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        z.zipccl_compress_static(d_in, n, z.BF16, C, ce, table, got, got_cb)
    for rep in range(3):
        x = W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32) * np.float32(0.3 * 5 ** rep))
        d_in.copy_(torch.from_numpy(x.view(np.int16)))         # eager work between replays
        got.fill_(0xA5)
        want.fill_(0xA5)
        z.zipccl_compress(d_in, n, z.BF16, C, ce, table, want, want_cb, d_ws)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(got_cb, want_cb) and torch.equal(got, want), rep
