"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, bit for bit.

Integer / byte work throughout, so the bar is exact equality of the compressed bytes over
the transmitted range of every slot, of chunk_bytes, and of the decoded words.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2604_27844_amd.binding as z
from paper_2604_27844_amd import workloads as W

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DEV, check_parity, gpu_compress, gpu_decompress, to_device_words


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(params=[False, True], ids=["stash", "reread"])
def compress_path(request):
    """False: full workspace (single pass with a stash); True: minimum workspace (the input is read twice).
    The workspace size alone selects the form, call by call."""
    return request.param


SMALL = [("c1", 1.0), ("c2", 1 / 8), ("c3", 1 / 32), ("c4", 1 / 64), ("c5", 1 / 64), ("c5_fp32", 1 / 32)]


@pytest.mark.parametrize("name,scale", SMALL)
def test_workload_parity_small(name, scale, compress_path):
    w = W.make(name, scale)
    _say(f"[parity] {w.name} n={w.n_elems} chunks={w.n_chunks} path={compress_path}")
    check_parity(w.data, w.dtype, w.sigma, w.n_chunks, w.chunk_elems, label=w.name, reread=compress_path)


EDGE_N = [0, 1, 7, 8, 9, 63, 64, 127, 128, 129, 511, 512, 513, 1023, 4095, 4096, 4097, 8191, 8192, 8193,
          16383, 16384, 16385, 16389, 32767, 32768, 32769, 40000]


@pytest.mark.parametrize("dtype", [z.BF16, z.FP32], ids=["bf16", "fp32"])
def test_edge_sizes_single_chunk(dtype, compress_path):
    rng = np.random.default_rng(100 + dtype)
    for n in EDGE_N:
        _say(f"[edge] dtype={dtype} n={n} path={compress_path}")
        f = rng.standard_normal(n, dtype=np.float32)
        data = W.f32_to_bf16_words(f) if dtype == z.BF16 else f.view(np.uint32).copy()
        check_parity(data, dtype, 1.0, 1, None, label=f"n={n}", reread=compress_path)


@pytest.mark.parametrize("dtype", [z.BF16, z.FP32], ids=["bf16", "fp32"])
def test_ragged_chunks_with_empty_and_unaligned_starts(dtype, compress_path):
    # odd chunk sizes make chunk starts 2/4-byte aligned only -> the element-wise path
    ce = np.array([0, 1, 8191, 8192, 3, 0, 20001, 513, 16384, 7, 0], dtype=np.uint64)
    n = int(ce.sum())
    rng = np.random.default_rng(7)
    f = rng.standard_normal(n, dtype=np.float32) * np.float32(0.5)
    data = W.f32_to_bf16_words(f) if dtype == z.BF16 else f.view(np.uint32).copy()
    _say(f"[ragged] dtype={dtype} n={n} chunks={len(ce)} path={compress_path}")
    check_parity(data, dtype, 0.5, len(ce), ce, label="ragged", reread=compress_path)


@pytest.mark.parametrize("dtype", [z.BF16, z.FP32], ids=["bf16", "fp32"])
def test_ragged_chunks_in_a_launch_of_more_than_64_mib(dtype):
    """zipccl_decompress picks its tile by the bytes a launch writes: from 64 MiB on it decodes in tiles of
    8 groups (4096 values), below in tiles of 16.  Same ragged shapes as the small case (empty chunks, chunks
    around one and two of the small tiles, odd starts), followed by large odd chunks that carry the launch
    past 64 MiB; element by element against the oracle, and a damaged index entry deep in a large chunk must
    be flagged."""
    es = 2 if dtype == z.BF16 else 4
    big = (66 << 20) // es // 4
    ce = np.array([0, 1, 4095, 4096, 4097, 3, 0, 8191, 8193, 12289, 513, 7, big + 1, big + 4095, 0, big + 4097, big - 511],
                  dtype=np.uint64)
    n = int(ce.sum())
    assert n * es >= 64 << 20
    rng = np.random.default_rng(11 + dtype)
    f = rng.standard_normal(n, dtype=np.float32) * np.float32(0.5)
    data = W.f32_to_bf16_words(f) if dtype == z.BF16 else f.view(np.uint32).copy()
    del f
    _say(f"[ragged-large] dtype={dtype} n={n} chunks={len(ce)}")
    got, got_cb, off = check_parity(data, dtype, 0.5, len(ce), ce, label="ragged-large")
    c = 13                                                   # big + 4095 values
    nc = int(ce[c])
    pad = lambda x: (x + 127) // 128 * 128
    lay_idx = 128 + pad(nc) + (pad(2 * nc) if dtype == z.FP32 else 0) + 3 * pad((nc + 7) // 8)
    g = (nc // 512) - 3
    bad = torch.from_numpy(got).to(DEV)
    pos = int(off[c]) + lay_idx + 4 * g
    bad[pos:pos + 4] = torch.tensor([0xFF, 0xFF, 0xFF, 0x7F], dtype=torch.uint8, device=DEV)
    _, st = gpu_decompress(bad, n, dtype, len(ce), ce)
    assert st == 4


@pytest.mark.parametrize("dtype", [z.BF16, z.FP32], ids=["bf16", "fp32"])
def test_chunk_starts_of_every_alignment_with_whole_tiles(dtype, compress_path):
    # chunk starts (in bf16 bytes) at 0, 4, 49168, 81936, 81944 and 114714: multiples of 16, of 8, of 4 and
    # of 2 only, each followed by whole tiles (the vector path takes any dword-aligned start, the
    # element-wise one the rest)
    ce = np.array([2, 24582, 16384, 4, 16385, 24576], dtype=np.uint64)
    n = int(ce.sum())
    rng = np.random.default_rng(8)
    f = rng.standard_normal(n, dtype=np.float32) * np.float32(0.5)
    f[rng.integers(0, n, 3000)] *= np.float32(1e6)          # zero-points everywhere
    data = W.f32_to_bf16_words(f) if dtype == z.BF16 else f.view(np.uint32).copy()
    _say(f"[alignments] dtype={dtype} n={n} path={compress_path}")
    check_parity(data, dtype, 0.5, len(ce), ce, label="alignments", reread=compress_path)


def test_more_chunks_than_one_launch_holds(compress_path):
    rng = np.random.default_rng(8)
    ce = rng.integers(0, 3000, 300).astype(np.uint64)
    ce[::17] = 0
    ce[5] = 30000
    n = int(ce.sum())
    data = W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32))
    _say(f"[batches] n={n} chunks=300 path={compress_path}")
    check_parity(data, z.BF16, 1.0, 300, ce, label="300 chunks", reread=compress_path)


def test_all_bf16_patterns_and_extreme_tables(compress_path):
    data = np.tile(np.arange(65536, dtype=np.uint16), 2)[:-5]
    for sigma in (1.0, 1e-45, 1e300, 0.02):
        _say(f"[patterns] sigma={sigma} path={compress_path}")
        check_parity(data, z.BF16, sigma, 1, None, label=f"patterns sigma={sigma}", reread=compress_path)


def test_fp32_random_bit_patterns(compress_path):
    rng = np.random.default_rng(9)
    data = rng.integers(0, 2 ** 32, 100_003, dtype=np.uint64).astype(np.uint32)
    data[:6] = [0, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00001, 0xFFFFFFFF]
    _say(f"[fp32 bits] path={compress_path}")
    check_parity(data, z.FP32, 1.0, 1, None, label="fp32 bits", reread=compress_path)


def test_all_zero_points_and_none(compress_path):
    n = 3 * 8192 + 77
    zeros = np.zeros(n, dtype=np.uint16)                     # every value a zero-point: ESC = n bytes
    ones = np.full(n, 0x3F80, dtype=np.uint16)               # no zero-point at all
    half = ones.copy()
    half[::2] = 0x7F80                                       # alternating +Inf
    for name, d in (("all-escape", zeros), ("no-escape", ones), ("alternating", half)):
        _say(f"[{name}] path={compress_path}")
        got, cb, off = check_parity(d, z.BF16, 1.0, 1, None, label=name, reread=compress_path)
    # worst case fills the slot exactly: chunk_bytes == capacity
    d_out, d_cb, _ = gpu_compress(np.zeros(8192, dtype=np.uint16), z.BF16, 1.0)
    assert int(d_cb.item()) == z.zipccl_max_compressed_size(8192, z.BF16, 1)


def test_peer_decodes_its_slice_alone_from_transmitted_bytes():
    w = W.make("c3", 1 / 64)
    d_out, d_cb, table = gpu_compress(w.data, w.dtype, w.sigma, w.n_chunks, w.chunk_elems)
    off = z.zipccl_chunk_slot_offsets(w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    cb = d_cb.cpu().numpy()
    start = 0
    for c in range(w.n_chunks):
        nc = int(w.chunk_elems[c])
        if c % 9 == 0:
            slice_ = d_out[int(off[c]):int(off[c]) + int(cb[c])].clone()     # exactly what would be sent
            back, st = gpu_decompress(slice_, nc, w.dtype, 1, None)
            assert st == 0 and np.array_equal(back, w.data[start:start + nc]), c
        start += nc


def test_small_workspace_takes_the_two_pass_form():
    w = W.make("c3", 1 / 64)
    table = z.zipccl_build_table(w.sigma, w.dtype)
    cap = z.zipccl_max_compressed_size(w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    d_in = to_device_words(w.data)
    ref, ref_cb, off = oracle.compress(w.data, w.dtype, oracle.build_table(w.sigma), w.n_chunks, w.chunk_elems)
    lo = z.zipccl_compress_min_workspace_size(w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    hi = z.zipccl_compress_workspace_size(w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    assert lo < hi
    for ws in (lo, hi - 16, hi):
        d_out = torch.full((cap,), 0xA5, dtype=torch.uint8, device=DEV)
        d_cb = torch.zeros(w.n_chunks, dtype=torch.int64, device=DEV)
        d_ws = torch.empty(ws, dtype=torch.uint8, device=DEV)
        z.zipccl_compress(d_in, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, table, d_out, d_cb, d_ws)
        torch.cuda.synchronize()
        got = d_out.cpu().numpy()
        assert np.array_equal(d_cb.cpu().numpy().astype(np.uint64), ref_cb)
        for c in range(w.n_chunks):
            s, e = int(off[c]), int(off[c]) + int(ref_cb[c])
            assert np.array_equal(got[s:e], ref[s:e]), (ws, c)
    with pytest.raises(z.ZipcclError) as ei:
        d_ws = torch.empty(lo - 16, dtype=torch.uint8, device=DEV)
        z.zipccl_compress(d_in, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, table, d_out, d_cb, d_ws)
    assert ei.value.code == 3


def test_compress_is_deterministic_and_reuses_workspace():
    w = W.make("c4", 1 / 64)
    table = z.zipccl_build_table(w.sigma, w.dtype)
    cap = z.zipccl_max_compressed_size(w.n_elems, w.dtype, w.n_chunks)
    d_in = to_device_words(w.data)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(w.n_elems, w.dtype, w.n_chunks), dtype=torch.uint8, device=DEV)
    outs = []
    for it in range(4):
        d_out = torch.full((cap,), 0x11 * (it + 1), dtype=torch.uint8, device=DEV)
        d_cb = torch.zeros(w.n_chunks, dtype=torch.int64, device=DEV)
        z.zipccl_compress(d_in, w.n_elems, w.dtype, w.n_chunks, None, table, d_out, d_cb, d_ws)
        torch.cuda.synchronize()
        outs.append((d_out.cpu().numpy(), d_cb.cpu().numpy()))
    off = z.zipccl_chunk_slot_offsets(w.n_elems, w.dtype, w.n_chunks)
    for o, cb in outs[1:]:
        assert np.array_equal(cb, outs[0][1])
        for c in range(w.n_chunks):
            s, e = int(off[c]), int(off[c]) + int(cb[c])
            assert np.array_equal(o[s:e], outs[0][0][s:e])


def test_decoder_flags_corrupt_streams_without_leaving_buffers():
    w = W.make("c1", 1 / 16)
    d_out, d_cb, _ = gpu_compress(w.data, w.dtype, w.sigma)
    n = w.n_elems
    cb = int(d_cb.item())
    good = d_out[:cb].clone()
    back, st = gpu_decompress(good, n, w.dtype)
    assert st == 0 and np.array_equal(back, w.data)
    lay_idx = 128 + n + 3 * (n // 8)                       # n is a multiple of 1024 here
    for pos, val in ((0, 0x00), (4, 2), (8, 1), (13, 1), (16, 1), (24, 0xFF), (40, 1), (41, 3), (47, 0)):
        bad = good.clone()
        bad[pos] = val
        _, st = gpu_decompress(bad, n, w.dtype)
        assert st == 4, pos
    bad = good.clone()                                       # the reserved header bytes are ignored when decoding
    bad[48:128] = 0xEE
    back, st = gpu_decompress(bad, n, w.dtype)
    assert st == 0 and np.array_equal(back, w.data)
    bad = good.clone()                                       # an index far outside the zero-point list
    bad[lay_idx + 4:lay_idx + 8] = torch.tensor([0xFF, 0xFF, 0xFF, 0x7F], dtype=torch.uint8, device=DEV)
    _, st = gpu_decompress(bad, n, w.dtype)
    assert st == 4
    # zero-point list cut off: the header promises more bytes than the buffer holds
    _, st = gpu_decompress(good, n, w.dtype, comp_capacity=cb - 128)
    assert st == 4
    with pytest.raises(z.ZipcclError) as ei:                 # static part not readable: host error
        gpu_decompress(good, n, w.dtype, comp_capacity=lay_idx)
    assert ei.value.code == 3


def test_runs_on_a_side_stream():
    w = W.make("c2", 1 / 16)
    s = torch.cuda.Stream()
    table = z.zipccl_build_table(w.sigma, w.dtype)
    cap = z.zipccl_max_compressed_size(w.n_elems, w.dtype, w.n_chunks)
    d_in = to_device_words(w.data)
    d_out = torch.empty(cap, dtype=torch.uint8, device=DEV)
    d_cb = torch.zeros(w.n_chunks, dtype=torch.int64, device=DEV)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(w.n_elems, w.dtype, w.n_chunks), dtype=torch.uint8, device=DEV)
    d_back = torch.zeros_like(d_in)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        z.zipccl_compress(d_in, w.n_elems, w.dtype, w.n_chunks, None, table, d_out, d_cb, d_ws, stream=s)
        z.zipccl_decompress(d_out, d_back, w.n_elems, w.dtype, w.n_chunks, None, None, stream=s)
    s.synchronize()
    assert np.array_equal(d_back.cpu().numpy().view(np.uint16), w.data)


def test_random_splits_and_contents_fuzz(compress_path):
    """Seeded fuzz: random chunk splits (empty, tiny, multi-tile, odd sizes), dtypes, tables and value
    mixes (Gaussian bulk, runs of zero-points, special values), each compared byte for byte."""
    rng = np.random.default_rng(1234)
    for case in range(12):
        dtype = int(rng.integers(0, 2))
        k = int(rng.integers(1, 12))
        ce = rng.choice([0, 1, 5, 8, 100, 511, 512, 513, 4096, 8191, 8192, 8200, 20000, 33000], size=k).astype(np.uint64)
        n = int(ce.sum())
        sigma = float(np.exp(rng.uniform(np.log(1e-6), np.log(1e3))))
        f = rng.standard_normal(n, dtype=np.float32) * np.float32(sigma)
        # runs of values far outside the window (dense zero-point stretches) and specials
        for _ in range(int(rng.integers(0, 4))):
            if n:
                s0 = int(rng.integers(0, n)); ln = int(rng.integers(1, 3000))
                f[s0:s0 + ln] *= np.float32(1e6)
        data = W.f32_to_bf16_words(f) if dtype == z.BF16 else f.view(np.uint32).copy()
        if n > 10:
            spec = np.array([0x0000, 0x8000, 0x7F80, 0xFF80, 0x7FC1, 0x0001], dtype=np.uint32)
            pos = rng.integers(0, n, spec.size)
            data[pos] = spec.astype(data.dtype) if dtype == z.BF16 else (spec << 16 | 0x1234).astype(np.uint32)
        _say(f"[fuzz {case}] dtype={dtype} chunks={list(ce)} sigma={sigma:.3g} path={compress_path}")
        check_parity(data, dtype, sigma, k, ce, label=f"fuzz{case}", reread=compress_path)


@pytest.mark.parametrize("tiles", [2500, 4500], ids=["scan_in_place_kernel", "scan_kernel"])
def test_one_chunk_spanning_several_scan_segments(compress_path, tiles):
    # many tiles in a single chunk: the per-chunk prefix of tile counts crosses scan segments (2500 tiles:
    # summed inside the placement kernel; 4500: by the scan kernel of its own), plus a second, shorter
    # chunk so that grids over unequal chunks are covered
    ce = np.array([tiles * 8192 + 123, 1030 * 8192], dtype=np.uint64)
    rng = np.random.default_rng(77)
    data = W.f32_to_bf16_words(rng.standard_normal(int(ce.sum()), dtype=np.float32) * np.float32(0.5))
    data[5_000_000:5_020_000] = 0x7F80                      # a dense stretch of zero-points
    _say(f"[segments] n={data.size} path={compress_path}")
    check_parity(data, z.BF16, 0.5, 2, ce, label="scan segments", reread=compress_path)


def test_static_then_dynamic_transfer_as_in_the_second_all_to_all_design():
    """Send the static parts of all slots first, then the sizes, then the dynamic parts (paper
    section 3.2, design 2): the receiver rebuilds every slot from the two ranges and decodes."""
    w = W.make("c3", 1 / 64)
    d_out, d_cb, _ = gpu_compress(w.data, w.dtype, w.sigma, w.n_chunks, w.chunk_elems)
    off = z.zipccl_chunk_slot_offsets(w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    st = z.zipccl_chunk_static_bytes(w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    recv = torch.full_like(d_out, 0xEE)
    for c in range(w.n_chunks):                               # phase 1: static parts, sizes known a priori
        a = int(off[c])
        recv[a:a + int(st[c])] = d_out[a:a + int(st[c])]
    cb = d_cb.cpu().numpy()                                   # phase 2: the size exchange (one u64 per peer)
    assert np.all(cb.astype(np.uint64) >= st)
    for c in range(w.n_chunks):                               # phase 3: dynamic parts
        a, b = int(off[c]) + int(st[c]), int(off[c]) + int(cb[c])
        recv[a:b] = d_out[a:b]
    back, status = gpu_decompress(recv, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems)
    assert status == 0 and np.array_equal(back, w.data)


def test_compress_and_decompress_replay_inside_a_hip_graph():
    """The calls only launch kernels (no allocation, memset or synchronisation), so they can be
    captured; every replay, on fresh input contents, must equal the oracle."""
    w0 = W.make("c2", 1 / 16)
    n, dt, k = w0.n_elems, w0.dtype, w0.n_chunks
    table = z.zipccl_build_table(w0.sigma, dt)
    cap = z.zipccl_max_compressed_size(n, dt, k)
    d_in = to_device_words(w0.data)
    d_out = torch.empty(cap, dtype=torch.uint8, device=DEV)
    d_cb = torch.zeros(k, dtype=torch.int64, device=DEV)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(n, dt, k), dtype=torch.uint8, device=DEV)
    d_back = torch.zeros_like(d_in)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                              # warm-up outside the capture
        z.zipccl_compress(d_in, n, dt, k, None, table, d_out, d_cb, d_ws)
        z.zipccl_decompress(d_out, d_back, n, dt, k, None, d_st)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        z.zipccl_compress(d_in, n, dt, k, None, table, d_out, d_cb, d_ws)
        z.zipccl_decompress(d_out, d_back, n, dt, k, None, d_st)
    rng = np.random.default_rng(5)
    for rep in range(3):
        data = W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32) * np.float32(1.0 + rep))
        d_in.copy_(to_device_words(data))                      # eager work between replays
        d_out.fill_(0xA5)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ref, ref_cb, off = oracle.compress(data, dt, oracle.build_table(w0.sigma), k)
        got = d_out.cpu().numpy()
        assert np.array_equal(d_cb.cpu().numpy().astype(np.uint64), ref_cb), rep
        for c in range(k):
            a, b = int(off[c]), int(off[c]) + int(ref_cb[c])
            assert np.array_equal(got[a:b], ref[a:b]), (rep, c)
        assert int(d_st.item()) == 0
        assert np.array_equal(d_back.cpu().numpy().view(np.uint16), data), rep
