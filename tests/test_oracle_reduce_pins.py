"""Pins for the oracle's decode-and-reduce (paper section 3.3 / 5.2: local FP32 reduction of the
slices a rank receives in the zipped Reduce-Scatter)."""
import numpy as np
import pytest

import oracle
from oracle import BF16, FP32
from paper_2604_27844_amd import workloads as W


def _pack(peers, dtype, sigma=1.0):
    """Compress every peer's slice as its own chunk: the receive-buffer layout (slots back to back)."""
    x = np.concatenate(peers)
    out, cb, off = oracle.compress(x, dtype, oracle.build_table(sigma), n_chunks=len(peers))
    return out


def _bf16(vals):
    return W.f32_to_bf16_words(np.asarray(vals, dtype=np.float32))


def test_single_peer_is_exact_widening_including_signed_zero():
    """Every bf16 pattern that is not a NaN comes back widened bit for bit (-0 stays -0, subnormals and
    infinities survive: -0 is the identity of the FP32 addition); every NaN comes back as 0x7FC00000."""
    x = np.arange(65536, dtype=np.uint16)
    got = oracle.decompress_reduce(_pack([x], BF16), x.size, BF16, 1)
    nan = (((x >> 7) & 0xFF) == 0xFF) & ((x & 0x7F) != 0)
    assert nan.sum() == 254
    assert np.array_equal(got[~nan], x[~nan].astype(np.uint32) << 16)
    assert np.all(got[nan] == 0x7FC00000)
    got16 = oracle.decompress_reduce(_pack([x], BF16), x.size, BF16, 1, BF16)
    assert np.array_equal(got16[~nan], x[~nan]) and np.all(got16[nan] == 0x7FC0)


def test_nan_sums_are_the_canonical_quiet_nan_whatever_produced_them():
    """Hand values.  A signalling NaN (0x7F800001) alone, a negative quiet NaN with payload, Inf - Inf, and a
    NaN met after finite terms all give 0x7FC00000 (bf16 output: 0x7FC0); signed zeros follow IEEE 754:
    (-0) + (-0) = -0, (+0) + (-0) = +0."""
    inf, ninf = 0x7F800000, 0xFF800000
    cases = [([0x7F800001], 0x7FC00000), ([0xFFC12345], 0x7FC00000), ([inf, ninf], 0x7FC00000),
             ([0x3F800000, 0x40000000, 0xFFFFFFFF], 0x7FC00000), ([0x7FC00001, 0x3F800000], 0x7FC00000),
             ([inf, inf], inf), ([0x80000000, 0x80000000], 0x80000000), ([0x00000000, 0x80000000], 0x00000000),
             ([0x80000000], 0x80000000), ([0x00000001, 0x00000001], 0x00000002)]
    for words, want in cases:
        peers = [np.array([w], dtype=np.uint32) for w in words]
        got = oracle.decompress_reduce(_pack(peers, FP32), 1, FP32, len(peers))
        assert got[0] == want, (words, hex(int(got[0])))
        got16 = oracle.decompress_reduce(_pack(peers, FP32), 1, FP32, len(peers), BF16)
        assert got16[0] == want >> 16, (words, hex(int(got16[0])))      # each sum is a bf16 value or rounds to zero


def test_small_integers_sum_exactly():
    rng = np.random.default_rng(0)
    peers = [_bf16(rng.integers(-100, 101, 5000)) for _ in range(7)]
    want = sum((p.astype(np.uint32) << 16).view(np.float32).astype(np.float64) for p in peers)
    got = oracle.decompress_reduce(_pack(peers, BF16), 5000, BF16, 7).view(np.float32)
    assert np.array_equal(got.astype(np.float64), want)


def test_sum_is_sequential_in_peer_order_and_in_fp32():
    big, one = 2.0 ** 30, 1.0
    a = oracle.decompress_reduce(_pack([_bf16([big]), _bf16([-big]), _bf16([one])], BF16), 1, BF16, 3).view(np.float32)
    b = oracle.decompress_reduce(_pack([_bf16([one]), _bf16([big]), _bf16([-big])], BF16), 1, BF16, 3).view(np.float32)
    assert a[0] == 1.0       # (2^30 - 2^30) + 1
    assert b[0] == 0.0       # (1 + 2^30) - 2^30: the 1 is lost in FP32 (it would survive in FP64)


@pytest.mark.parametrize("dtype", [BF16, FP32])
def test_error_bound_against_fp64(dtype):
    rng = np.random.default_rng(1)
    P, n = 8, 20000
    f = [rng.standard_normal(n, dtype=np.float32) * np.float32(0.02) for _ in range(P)]
    peers = [W.f32_to_bf16_words(v) if dtype == BF16 else v.view(np.uint32) for v in f]
    exact = [((p.astype(np.uint32) << 16) if dtype == BF16 else p).view(np.float32).astype(np.float64) for p in peers]
    got = oracle.decompress_reduce(_pack(peers, dtype, 0.02), n, dtype, P).view(np.float32).astype(np.float64)
    s, sabs = sum(exact), sum(np.abs(e) for e in exact)
    assert np.all(np.abs(got - s) <= (P - 1) * 2.0 ** -24 * sabs * 1.01)
    assert np.any(got != s)                                  # it really is FP32 arithmetic


def test_bf16_output_is_round_to_nearest_even_of_the_fp32_sum():
    rng = np.random.default_rng(2)
    P, n = 4, 30000
    peers = [W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32)) for _ in range(P)]
    comp = _pack(peers, BF16)
    f32 = oracle.decompress_reduce(comp, n, BF16, P, FP32)
    b16 = oracle.decompress_reduce(comp, n, BF16, P, BF16)
    x = f32.view(np.float32).astype(np.float64)
    lo = ((f32 >> 16) << 16).view(np.float32).astype(np.float64)                  # truncation toward zero
    hi = ((((f32 >> 16) + 1) << 16).astype(np.uint32)).view(np.float32).astype(np.float64)  # next bf16 away from zero
    r = (b16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.all((r == lo) | (r == hi))
    dl, dh = np.abs(x - lo), np.abs(hi - x)
    assert np.all(np.where(dl < dh, r == lo, True)) and np.all(np.where(dh < dl, r == hi, True))
    tie = dl == dh
    assert np.all((b16[tie] & 1) == 0)                        # ties go to the even bf16
    # exact ties do occur in sums of bf16 values; make sure some were exercised
    assert tie.sum() > 0


def test_reduce_rejects_corrupt_and_bad_arguments():
    peers = [_bf16(np.ones(100)), _bf16(np.ones(100))]
    comp = _pack(peers, BF16)
    bad = comp.copy()
    bad[oracle.slot_cap(100, BF16)] ^= 1                      # second slot's magic
    with pytest.raises(oracle.OracleError):
        oracle.decompress_reduce(bad, 100, BF16, 2)
    with pytest.raises(oracle.OracleError):
        oracle.decompress_reduce(comp, 100, BF16, 3)          # third slot is not there
    with pytest.raises(oracle.OracleError):
        oracle.decompress_reduce(comp, 100, BF16, 0)
