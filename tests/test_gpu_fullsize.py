"""GPU parity at the benchmark's full sizes and launch configuration (the >=256 MB workloads
plus the two small ones), element by element against the oracle, which needs a few seconds
per workload at these sizes."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2604_27844_amd.binding as z
from paper_2604_27844_amd import workloads as W

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DEV, gpu_compress, to_device_words


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5", "c5_fp32"])
def test_fullsize_parity(name):
    print(f"[full] generating {name}", flush=True)
    w = W.make(name, 1.0)
    print(f"[full] {w.name} n={w.n_elems} ({w.nbytes / 2**20:.0f} MiB) chunks={w.n_chunks}", flush=True)
    d_in = to_device_words(w.data)
    d_out, d_cb, table = gpu_compress(w.data, w.dtype, w.sigma, w.n_chunks, w.chunk_elems, d_in=d_in)
    words = torch.int16 if w.dtype == z.BF16 else torch.int32
    d_back = torch.zeros(w.n_elems, dtype=words, device=DEV)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    z.zipccl_decompress(d_out, d_back, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems, d_st)
    torch.cuda.synchronize()
    assert int(d_st.item()) == 0
    assert torch.equal(d_back, d_in), "GPU round trip differs"
    print("[full] oracle compress", flush=True)
    ref, ref_cb, off = oracle.compress(w.data, w.dtype, oracle.build_table(w.sigma), w.n_chunks, w.chunk_elems)
    got_cb = d_cb.cpu().numpy().astype(np.uint64)
    assert np.array_equal(got_cb, ref_cb)
    got = d_out.cpu().numpy()
    for c in range(w.n_chunks):
        s, e = int(off[c]), int(off[c]) + int(ref_cb[c])
        assert np.array_equal(got[s:e], ref[s:e]), f"chunk {c} differs"
    ratio = w.nbytes / float(ref_cb.sum())
    print(f"[full] {w.name} ratio {ratio:.4f}", flush=True)
    del ref, got
    # the robust sigma at this size, in the launch configuration the benchmark times: the median it found must
    # have the rank the definition gives it (lower median of the nonzero finite magnitudes of the high 16-bit
    # words; counted here with plain comparisons, no sort), and the window must be the nominal sigma's
    d_tab = torch.zeros(8, dtype=torch.uint8, device=DEV)
    d_sig = torch.zeros(1, dtype=torch.float64, device=DEV)
    d_ews = torch.full((z.zipccl_estimate_robust_workspace_size(),), 0x77, dtype=torch.uint8, device=DEV)
    z.zipccl_estimate_table_robust(d_in, w.n_elems, w.dtype, d_tab, d_sig, d_ews)
    torch.cuda.synchronize()
    med = np.float32(float(d_sig.item()) * 0.6744897501960817)          # sigma = median / Phi^-1(3/4); the median is a bf16 value
    med_word = int(np.array([med], dtype=np.float32).view(np.uint32)[0])
    assert med_word & 0xFFFF == 0, hex(med_word)
    med_bits = med_word >> 16
    mag = (w.data if w.dtype == z.BF16 else (w.data >> np.uint32(16)).astype(np.uint16)) & np.uint16(0x7FFF)
    counted = (mag != 0) & (mag < 0x7F80)
    K = int(np.count_nonzero(counted))
    below = int(np.count_nonzero(counted & (mag < med_bits)))
    upto = int(np.count_nonzero(counted & (mag <= med_bits)))
    assert below <= (K - 1) // 2 < upto, (name, K, below, upto, med_bits)
    assert list(d_tab.cpu().numpy()) == list(oracle.build_table(w.sigma)), name
    print(f"[full] {w.name} robust sigma {float(d_sig.item()):.6g}", flush=True)


@pytest.mark.parametrize("name", ["c3", "c4", "c5", "c5_fp32"])
def test_fullsize_reduce_parity(name):
    """The fused reduce in the configuration the benchmark times: the workload cut into 8 peer slices of one
    shard, compressed as 8 slots, decoded and summed; every sum against the oracle's, all bits, for both output
    types.  c3's shard is not a whole number of tiles (whole tiles and the rest in one launch, two groups per
    wave), c4 and c5 fill the chip a whole number of times (four), c5_fp32 takes one group per wave."""
    P = 8
    w = W.make(name, 1.0)
    assert w.n_elems % P == 0
    n = w.n_elems // P
    print(f"[full-reduce] {w.name}: {P} peers x {n} values ({n / 8192:.2f} tiles)", flush=True)
    d_in = to_device_words(w.data)
    table = z.zipccl_build_table(w.sigma, w.dtype)
    cap = z.zipccl_max_compressed_size(w.n_elems, w.dtype, P)
    assert cap == P * z.zipccl_max_compressed_size(n, w.dtype, 1)
    d_comp = torch.full((cap,), 0xA5, dtype=torch.uint8, device=DEV)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(w.n_elems, w.dtype, P), dtype=torch.uint8, device=DEV)
    z.zipccl_compress(d_in, w.n_elems, w.dtype, P, None, table, d_comp, None, d_ws)
    torch.cuda.synchronize()
    comp = d_comp.cpu().numpy()
    del d_in, d_ws
    for out_dt in (z.FP32, z.BF16):
        print(f"[full-reduce] {w.name}: out dtype {out_dt}", flush=True)
        d_out = torch.full((n,), 0x3C3C if out_dt == z.BF16 else 0x3C3C3C3C,
                           dtype=torch.int16 if out_dt == z.BF16 else torch.int32, device=DEV)
        d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
        z.zipccl_decompress_reduce(d_comp, d_out, n, w.dtype, P, out_dt, d_st)
        torch.cuda.synchronize()
        assert int(d_st.item()) == 0
        got = d_out.cpu().numpy().view(np.uint16 if out_dt == z.BF16 else np.uint32)
        want = oracle.decompress_reduce(comp, n, w.dtype, P, out_dt)
        bad = np.nonzero(got != want)[0]
        assert bad.size == 0, f"{name}: {bad.size} sums differ, first at {bad[:5]}"
        del d_out, got, want


@pytest.mark.parametrize("dtype,n,sigma", [(z.BF16, 2 ** 32 - 1, 0.02), (z.FP32, 2 ** 31 + 4097, 0.5)],
                         ids=["bf16_max_chunk", "fp32_sections_past_4GiB"])
def test_one_chunk_of_the_largest_sizes(dtype, n, sigma):
    """A single chunk of ZIPCCL_MAX_CHUNK_ELEMS bf16 values (524288 tiles, 2^23 IDX entries, > 2^27 zero-points)
    and an fp32 chunk whose sections start past 4 GiB inside the slot: 64-bit offsets everywhere.  The input
    repeats a random block (generating 2^32 samples would take minutes); both compress paths."""
    rng = np.random.default_rng(123 + dtype)
    if dtype == z.BF16:
        blk = W.f32_to_bf16_words(rng.standard_normal(2 ** 26, dtype=np.float32) * np.float32(sigma))
        blk[::1000] = 0x7F80
    else:
        blk = (rng.standard_normal(2 ** 25, dtype=np.float32) * np.float32(sigma)).view(np.uint32).copy()
        blk[::777] = 0x7F800000
    data = np.tile(blk, n // blk.size + 1)[:n].copy()
    data[-5:] = [0x0000, 0x8000, 0x7FC1, 0x3F80, 0xFF80] if dtype == z.BF16 else [0, 1 << 31, 0x7FC00001, 0x3F800000, 0xFF800000]
    print(f"[huge] dtype={dtype} n={n}: oracle compress", flush=True)
    ref, ref_cb, off = oracle.compress(data, dtype, oracle.build_table(sigma), 1, None)
    cb = int(ref_cb[0])
    d_in = to_device_words(data)
    cap = z.zipccl_max_compressed_size(n, dtype, 1)
    assert cap == int(off[-1])
    d_out = torch.empty(cap, dtype=torch.uint8, device=DEV)
    d_cb = torch.zeros(1, dtype=torch.int64, device=DEV)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(n, dtype, 1), dtype=torch.uint8, device=DEV)
    d_back = torch.empty_like(d_in)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    # the robust sigma over 2^32 - 1 (2^31 + 4097) values: bin counts beyond 2^27, 64-bit sums in the finish kernel.
    # The input is a block repeated, so its magnitude histogram is the block's times the repetitions plus the rest's;
    # the median found must have the rank the definition gives it.
    d_tab = torch.zeros(8, dtype=torch.uint8, device=DEV)
    d_sig = torch.zeros(1, dtype=torch.float64, device=DEV)
    d_ews = torch.full((z.zipccl_estimate_robust_workspace_size(),), 0x77, dtype=torch.uint8, device=DEV)
    z.zipccl_estimate_table_robust(d_in, n, dtype, d_tab, d_sig, d_ews)
    torch.cuda.synchronize()
    mags = lambda a: ((a if dtype == z.BF16 else (a >> np.uint32(16))) & 0x7FFF).astype(np.int64)
    reps = n // blk.size
    hist = reps * np.bincount(mags(blk), minlength=32768) + np.bincount(mags(data[reps * blk.size:]), minlength=32768)
    hist[0] = 0
    hist[0x7F80:] = 0
    K, cum = int(hist.sum()), np.cumsum(hist)
    med_word = int(np.array([np.float32(float(d_sig.item()) * 0.6744897501960817)], dtype=np.float32).view(np.uint32)[0])
    assert med_word & 0xFFFF == 0
    b = med_word >> 16
    assert int(cum[b - 1]) <= (K - 1) // 2 < int(cum[b]), (K, b)
    assert list(d_tab.cpu().numpy()) == list(oracle.build_table(sigma))
    print(f"[huge] robust sigma {float(d_sig.item()):.6g} over {K} magnitudes", flush=True)
    # full workspace: single pass with a stash; minimum workspace: the input is read twice
    for wsb in (None, z.zipccl_compress_min_workspace_size(n, dtype, 1)):
        print(f"[huge] GPU compress, workspace bytes {wsb}", flush=True)
        d_out.fill_(0xA5)
        z.zipccl_compress(d_in, n, dtype, 1, None, z.zipccl_build_table(sigma, dtype), d_out, d_cb, d_ws,
                          workspace_bytes=wsb)
        torch.cuda.synchronize()
        assert int(d_cb.item()) == cb
        for a in range(0, cb, 1 << 30):
            b = min(cb, a + (1 << 30))
            assert np.array_equal(d_out[a:b].cpu().numpy(), ref[a:b]), f"compressed bytes differ in [{a}, {b})"
        d_back.fill_(0)
        z.zipccl_decompress(d_out, d_back, n, dtype, 1, None, d_st)
        torch.cuda.synchronize()
        assert int(d_st.item()) == 0
        assert torch.equal(d_back, d_in), "GPU round trip differs"
