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
