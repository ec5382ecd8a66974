"""GPU parity of zipccl_decompress_reduce against the oracle: FP32 sums in peer order are
reproducible, so the bar is bit equality, NaN sums included (both sides store the one quiet NaN 0x7FC00000)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_27844_amd.binding as z
from paper_2604_27844_amd import workloads as W

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DEV


def _peers(rng, P, n, dtype, sigmas):
    out = []
    for p in range(P):
        f = rng.standard_normal(n, dtype=np.float32) * np.float32(sigmas[p % len(sigmas)])
        out.append(W.f32_to_bf16_words(f) if dtype == z.BF16 else f.view(np.uint32).copy())
    return out


def _receive_buffer(peers, dtype, sigmas):
    """Each peer compresses its slice with its own table (on the GPU); slots end up back to back."""
    n = peers[0].size
    cap1 = z.zipccl_max_compressed_size(n, dtype, 1)
    buf = torch.full((cap1 * len(peers),), 0xA5, dtype=torch.uint8, device=DEV)
    ws = torch.empty(z.zipccl_compress_workspace_size(n, dtype, 1), dtype=torch.uint8, device=DEV)
    for p, x in enumerate(peers):
        signed = np.int16 if dtype == z.BF16 else np.int32
        d_in = torch.from_numpy(x.view(signed)).to(DEV)
        z.zipccl_compress(d_in, n, dtype, 1, None, z.zipccl_build_table(sigmas[p % len(sigmas)], dtype),
                          buf[p * cap1:(p + 1) * cap1], None, ws)
        torch.cuda.synchronize()
    return buf


def _check(peers, dtype, sigmas, out_dt, label):
    n, P = peers[0].size, len(peers)
    buf = _receive_buffer(peers, dtype, sigmas)
    want = oracle.decompress_reduce(buf.cpu().numpy(), n, dtype, P, out_dt)
    d_out = torch.full((n,), 0x3C3C if out_dt == z.BF16 else 0x3C3C3C3C,
                       dtype=torch.int16 if out_dt == z.BF16 else torch.int32, device=DEV)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    z.zipccl_decompress_reduce(buf, d_out, n, dtype, P, out_dt, d_st)
    torch.cuda.synchronize()
    assert int(d_st.item()) == 0, label
    got = d_out.cpu().numpy().view(np.uint16 if out_dt == z.BF16 else np.uint32)
    ok = got == want                                         # all bits: a NaN sum is 0x7FC00000 / 0x7FC0 on both sides
    assert ok.all(), (f"{label}: {np.count_nonzero(~ok)} sums differ, first at {np.nonzero(~ok)[0][:5]}: "
                      f"got {got[~ok][:5]} want {want[~ok][:5]}")


@pytest.mark.parametrize("dtype", [z.BF16, z.FP32], ids=["bf16", "fp32"])
@pytest.mark.parametrize("out_dt", [z.FP32, z.BF16], ids=["out_fp32", "out_bf16"])
def test_reduce_parity(dtype, out_dt):
    rng = np.random.default_rng(40 + dtype)
    for P, n in ((1, 5000), (2, 8192), (3, 8193), (8, 3 * 8192 + 700), (5, 1), (4, 511), (16, 40000)):
        print(f"[reduce] dtype={dtype} out={out_dt} P={P} n={n}", flush=True)
        sig = [0.02, 0.02, 0.05, 1e-3]
        _check(_peers(rng, P, n, dtype, sig), dtype, sig, out_dt, f"P={P} n={n}")


def test_single_slot_is_widened_exactly_for_every_bf16_pattern():
    x = np.arange(65536, dtype=np.uint16)
    for out_dt in (z.FP32, z.BF16):
        _check([x], z.BF16, [1.0], out_dt, "all patterns, one slot")
    _check([x, np.full(65536, 0x8000, dtype=np.uint16)], z.BF16, [1.0], z.FP32, "all patterns + (-0)")


@pytest.mark.parametrize("dtype,n", [(z.BF16, 2048 * 8192 + 5000), (z.BF16, 700 * 8192 + 4 * 2048 + 1500),
                                     (z.FP32, 2600 * 8192 + 2048 + 77)], ids=["bf16_four", "bf16_two", "fp32_two"])
def test_reduce_large_shards_take_several_groups_per_wave(dtype, n):
    """Past a size that depends on the dtype a workgroup takes two groups per wave, and four for bf16 shards of a
    multiple of 2048 whole tiles; the rest behind the whole tiles runs in the same launch."""
    rng = np.random.default_rng(44)
    sig = [0.02, 0.03]
    _check(_peers(rng, 2, n, dtype, sig), dtype, sig, z.FP32, "large shard")


def test_reduce_order_specials_and_cancellation():
    n = 8192 + 37
    big = np.full(n, W.f32_to_bf16_words(np.array([2.0 ** 30], dtype=np.float32))[0], dtype=np.uint16)
    neg = big | np.uint16(0x8000)
    one = np.full(n, 0x3F80, dtype=np.uint16)
    for order in ([big, neg, one], [one, big, neg]):
        _check(order, z.BF16, [1.0], z.FP32, "order")
    rng = np.random.default_rng(3)
    peers = [rng.integers(0, 65536, n, dtype=np.uint16, endpoint=False) for _ in range(4)]   # Inf, NaN, subnormals
    _check(peers, z.BF16, [1.0], z.FP32, "specials")
    _check(peers, z.BF16, [1.0], z.BF16, "specials bf16 out")
    words = [rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32) for _ in range(3)]
    _check(words, z.FP32, [1.0], z.FP32, "fp32 specials")


def test_reduce_flags_a_corrupt_slot_and_checks_arguments():
    rng = np.random.default_rng(5)
    n, P = 10000, 3
    peers = _peers(rng, P, n, z.BF16, [0.02])
    buf = _receive_buffer(peers, z.BF16, [0.02])
    cap1 = z.zipccl_max_compressed_size(n, z.BF16, 1)
    bad = buf.clone()
    bad[cap1 + 1] = 0x00                                      # magic of peer 1
    d_out = torch.zeros(n, dtype=torch.int32, device=DEV)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    z.zipccl_decompress_reduce(bad, d_out, n, z.BF16, P, z.FP32, d_st)
    torch.cuda.synchronize()
    assert int(d_st.item()) == 4
    with pytest.raises(z.ZipcclError) as ei:
        z.zipccl_decompress_reduce(buf, d_out, n, z.BF16, P + 1, z.FP32, d_st)   # a fourth slot is not there
    assert ei.value.code == 3
    with pytest.raises(z.ZipcclError) as ei:
        z.zipccl_decompress_reduce(buf, d_out, n, z.BF16, 0, z.FP32, d_st)
    assert ei.value.code == 1


def test_reduce_flags_index_and_plane_damage_inside_a_slot():
    """Damage behind a valid header: an index entry far outside the zero-point list, one that makes a group's slice
    longer than a group, and plane bytes that disagree with the index about a group's count.  Each is flagged
    (the sums of the damaged groups are unspecified), in the whole-tile kernel and in the general one, and no
    access leaves the buffers (the clamps are the kernel's own)."""
    rng = np.random.default_rng(8)
    P = 3
    for n in (6 * 2048 + 100, 700):
        peers = _peers(rng, P, n, z.BF16, [0.02])
        buf = _receive_buffer(peers, z.BF16, [0.02])
        cap1 = z.zipccl_max_compressed_size(n, z.BF16, 1)
        pad = lambda x: (x + 127) // 128 * 128
        p0 = 128 + pad(n)                                     # first plane of a slot
        idx = p0 + 3 * pad((n + 7) // 8)                      # its index
        ng = (n + 511) // 512
        pb = pad((n + 7) // 8)                                # bytes of one plane
        zeros = [0x00, 0x00, 0x00, 0x00]
        damage = {"index entry beyond the list": [(idx + 4 * (ng - 1), [0xFF, 0xFF, 0xFF, 0x7F])],
                  "a slice longer than a group": [(idx + 4, [600 & 0xFF, 600 >> 8, 0x00, 0x00])],
                  # code 0 for values 24..55 of group 0: 32 zero-points the index knows nothing of
                  "plane bytes against the index": [(p0 + 3, zeros), (p0 + pb + 3, zeros), (p0 + 2 * pb + 3, zeros)]}
        for label, edits in damage.items():
            print(f"[reduce] n={n} damage: {label}", flush=True)
            bad = buf.clone()
            for at, val in edits:
                bad[cap1 + at:cap1 + at + 4] = torch.tensor(val, dtype=torch.uint8, device=DEV)  # in slot 1
            d_out = torch.full((n,), 0x3C3C3C3C, dtype=torch.int32, device=DEV)
            d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
            z.zipccl_decompress_reduce(bad, d_out, n, z.BF16, P, z.FP32, d_st)
            torch.cuda.synchronize()
            assert int(d_st.item()) == 4, (n, label)
            z.zipccl_decompress_reduce(buf, d_out, n, z.BF16, P, z.FP32, d_st)          # the intact buffer still sums
            torch.cuda.synchronize()
            assert np.array_equal(d_out.cpu().numpy().view(np.uint32),
                                  oracle.decompress_reduce(buf.cpu().numpy(), n, z.BF16, P, z.FP32))


def test_reduce_leaves_rejected_slots_out_of_the_sum():
    """A slot whose header is rejected is flagged and skipped; the others are summed in order
    (first slot rejected: the sum starts at the second).  Sizes cover the bounds-check-free
    kernel (whole tiles) and the general one (ragged tail)."""
    rng = np.random.default_rng(6)
    P = 4
    for n in (4 * 2048 + 300, 1500):
        peers = _peers(rng, P, n, z.BF16, [0.02])
        buf = _receive_buffer(peers, z.BF16, [0.02])
        cap1 = z.zipccl_max_compressed_size(n, z.BF16, 1)
        for victim in (0, 2, 3):
            print(f"[reduce] rejected slot {victim} n={n}", flush=True)
            bad = buf.clone()
            bad[victim * cap1 + 2] = 0x00                     # magic of that slot
            rest = [peers[p] for p in range(P) if p != victim]
            want = oracle.decompress_reduce(_receive_buffer(rest, z.BF16, [0.02]).cpu().numpy(), n, z.BF16, P - 1, z.FP32)
            d_out = torch.full((n,), 0x3C3C3C3C, dtype=torch.int32, device=DEV)
            d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
            z.zipccl_decompress_reduce(bad, d_out, n, z.BF16, P, z.FP32, d_st)
            torch.cuda.synchronize()
            assert int(d_st.item()) == 4
            assert np.array_equal(d_out.cpu().numpy().view(np.uint32), want)


def test_reduce_into_an_output_that_is_only_element_aligned_and_empty_input():
    rng = np.random.default_rng(7)
    n, P = 3 * 2048 + 17, 3
    peers = _peers(rng, P, n, z.BF16, [0.02])
    buf = _receive_buffer(peers, z.BF16, [0.02])
    for out_dt, tdt, udt in ((z.BF16, torch.int16, np.uint16), (z.FP32, torch.int32, np.uint32)):
        want = oracle.decompress_reduce(buf.cpu().numpy(), n, z.BF16, P, out_dt)
        backing = torch.zeros(n + 8, dtype=tdt, device=DEV)
        d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
        z.zipccl_decompress_reduce(buf, backing[1:n + 1], n, z.BF16, P, out_dt, d_st)
        torch.cuda.synchronize()
        got = backing.cpu().numpy().view(udt)
        assert int(d_st.item()) == 0
        assert np.array_equal(got[1:n + 1], want) and got[0] == 0 and not got[n + 1:].any()
    # no values: only the headers are checked
    cap0 = z.zipccl_max_compressed_size(0, z.BF16, 1)
    empty = torch.zeros(cap0 * 2, dtype=torch.uint8, device=DEV)
    ws = torch.empty(z.zipccl_compress_workspace_size(0, z.BF16, 1), dtype=torch.uint8, device=DEV)
    d_in = torch.zeros(1, dtype=torch.int16, device=DEV)
    for p in range(2):
        z.zipccl_compress(d_in, 0, z.BF16, 1, None, z.zipccl_build_table(0.02, z.BF16), empty[p * cap0:(p + 1) * cap0], None, ws)
    d_out = torch.zeros(4, dtype=torch.int32, device=DEV)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    z.zipccl_decompress_reduce(empty, d_out, 0, z.BF16, 2, z.FP32, d_st)
    torch.cuda.synchronize()
    assert int(d_st.item()) == 0 and not d_out.cpu().numpy().any()


def test_estimate_compress_reduce_chain_replays_inside_a_hip_graph():
    """Table estimate -> compress with the device table -> fused reduce only launch kernels (no allocation,
    memset or synchronisation), so the chain can be captured; every replay, on fresh input contents and with
    the program's own eager work in between, must equal the oracle's chain."""
    from oracle import sigma as osg
    P, n = 4, 5 * 8192 + 300                                  # P peer slices = P equal chunks of one tensor
    d_in = torch.zeros(P * n, dtype=torch.int16, device=DEV)
    cap = z.zipccl_max_compressed_size(P * n, z.BF16, P)
    d_comp = torch.empty(cap, dtype=torch.uint8, device=DEV)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(P * n, z.BF16, P), dtype=torch.uint8, device=DEV)
    d_ews = torch.empty(z.zipccl_estimate_workspace_size(), dtype=torch.uint8, device=DEV)
    d_tab = torch.zeros(8, dtype=torch.uint8, device=DEV)
    d_sum = torch.zeros(n, dtype=torch.int32, device=DEV)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)

    def chain():
        z.zipccl_estimate_table(d_in, P * n, z.BF16, d_tab, None, d_ews)
        z.zipccl_compress_device_table(d_in, P * n, z.BF16, P, None, d_tab, d_comp, None, d_ws)
        z.zipccl_decompress_reduce(d_comp, d_sum, n, z.BF16, P, z.FP32, d_st)

    rng = np.random.default_rng(11)
    first = W.f32_to_bf16_words(rng.standard_normal(P * n, dtype=np.float32) * np.float32(0.3))
    d_in.copy_(torch.from_numpy(first.view(np.int16)))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                              # warm-up outside the capture
        chain()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        chain()
    for rep in range(3):
        data = W.f32_to_bf16_words(rng.standard_normal(P * n, dtype=np.float32) * np.float32(0.01 * 7 ** rep))
        d_in.copy_(torch.from_numpy(data.view(np.int16)))      # eager work between replays
        d_comp.fill_(0xA5)
        d_sum.fill_(0x3C3C3C3C)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        dec, _ = osg.estimate_table(data, z.BF16)
        assert list(d_tab.cpu().numpy()) == list(dec), rep
        ref, ref_cb, off = oracle.compress(data, z.BF16, dec, P)
        want = oracle.decompress_reduce(ref, n, z.BF16, P, z.FP32)
        assert int(d_st.item()) == 0
        assert np.array_equal(d_sum.cpu().numpy().view(np.uint32), want), rep


@pytest.mark.parametrize("stride", [1, 4], ids=["every_value", "sampled"])
def test_chunk_table_estimate_and_compress_chain_replays_inside_a_hip_graph(stride):
    """Per-chunk robust tables (from every value, or from a sample) -> compress with them -> fused reduce, captured
    and replayed: the histogram state is zeroed by a kernel of the chain itself, so every replay starts clean."""
    from oracle import sigma as osg
    P, n = 3, 4 * 8192 + 77
    d_in = torch.zeros(P * n, dtype=torch.int16, device=DEV)
    cap = z.zipccl_max_compressed_size(P * n, z.BF16, P)
    d_comp = torch.empty(cap, dtype=torch.uint8, device=DEV)
    d_ws = torch.empty(z.zipccl_compress_workspace_size(P * n, z.BF16, P), dtype=torch.uint8, device=DEV)
    d_ews = torch.empty(z.zipccl_estimate_chunk_tables_workspace_size(P), dtype=torch.uint8, device=DEV)
    d_tabs = torch.zeros(8 * P, dtype=torch.uint8, device=DEV)
    d_sum = torch.zeros(n, dtype=torch.int32, device=DEV)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)

    def chain():
        if stride == 1:
            z.zipccl_estimate_chunk_tables(d_in, P * n, z.BF16, P, None, d_tabs, None, d_ews)
        else:
            z.zipccl_estimate_chunk_tables_sampled(d_in, P * n, z.BF16, P, None, stride, d_tabs, None, d_ews)
        z.zipccl_compress_chunk_tables(d_in, P * n, z.BF16, P, None, d_tabs, d_comp, None, d_ws)
        z.zipccl_decompress_reduce(d_comp, d_sum, n, z.BF16, P, z.FP32, d_st)

    rng = np.random.default_rng(13)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        chain()
    for rep in range(3):
        scales = [0.01 * 9 ** rep, 3.0, 1e-3 * 2 ** rep]        # every peer's slice at its own scale
        data = np.concatenate([W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32) * np.float32(s)) for s in scales])
        d_in.copy_(torch.from_numpy(data.view(np.int16)))
        d_comp.fill_(0xA5)
        d_sum.fill_(0x3C3C3C3C)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        decs, _ = osg.robust_chunk_tables_sampled(data, z.BF16, P, stride=stride)
        assert np.array_equal(d_tabs.cpu().numpy().reshape(P, 8), decs), rep
        slots = [oracle.compress(data[p * n:(p + 1) * n], z.BF16, decs[p])[0] for p in range(P)]
        want = oracle.decompress_reduce(np.concatenate(slots), n, z.BF16, P, z.FP32)
        assert int(d_st.item()) == 0
        assert np.array_equal(d_sum.cpu().numpy().view(np.uint32), want), rep


def test_reduce_of_the_largest_peer_count_with_rejected_slots_in_every_round():
    """1024 slots (the limit): headers are checked 256 at a time, the accepted ones listed in slot order;
    a rejected slot in each of those rounds (and two side by side) must only drop out of the sum."""
    rng = np.random.default_rng(12)
    P, n = 1024, 700
    peers = _peers(rng, P, n, z.BF16, [0.02, 0.3])
    buf = _receive_buffer(peers, z.BF16, [0.02, 0.3])
    cap1 = z.zipccl_max_compressed_size(n, z.BF16, 1)
    want_all = oracle.decompress_reduce(buf.cpu().numpy(), n, z.BF16, P, z.FP32)
    d_out = torch.full((n,), 0x3C3C3C3C, dtype=torch.int32, device=DEV)
    d_st = torch.zeros(1, dtype=torch.int32, device=DEV)
    z.zipccl_decompress_reduce(buf, d_out, n, z.BF16, P, z.FP32, d_st)
    torch.cuda.synchronize()
    assert int(d_st.item()) == 0
    assert np.array_equal(d_out.cpu().numpy().view(np.uint32), want_all)
    victims = [0, 255, 256, 257, 600, 1023]
    bad = buf.clone()
    for v in victims:
        bad[v * cap1 + 2] = 0x00                              # magic of that slot
    rest = [peers[p] for p in range(P) if p not in victims]
    sig = [[0.02, 0.3][p % 2] for p in range(P) if p not in victims]
    # the remaining slices, each with the table it had, as the oracle sees them
    cbuf = torch.full((cap1 * len(rest),), 0xA5, dtype=torch.uint8, device=DEV)
    ws = torch.empty(z.zipccl_compress_workspace_size(n, z.BF16, 1), dtype=torch.uint8, device=DEV)
    for k, x in enumerate(rest):
        z.zipccl_compress(torch.from_numpy(x.view(np.int16)).to(DEV), n, z.BF16, 1, None,
                          z.zipccl_build_table(sig[k], z.BF16), cbuf[k * cap1:(k + 1) * cap1], None, ws)
        torch.cuda.synchronize()
    want = oracle.decompress_reduce(cbuf.cpu().numpy(), n, z.BF16, len(rest), z.FP32)
    d_st.zero_()
    z.zipccl_decompress_reduce(bad, d_out, n, z.BF16, P, z.FP32, d_st)
    torch.cuda.synchronize()
    assert int(d_st.item()) == 4
    assert np.array_equal(d_out.cpu().numpy().view(np.uint32), want)
