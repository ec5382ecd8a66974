"""Pins for the sigma-estimate oracle (paper section 4.1: sigma via torch.std)."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import sigma as osg
from oracle import BF16, FP32
from paper_2604_27844_amd import workloads as W


def test_textbook_values():
    x = np.array([1.0, 2.0, 3.0, 4.0], dtype=np.float32).view(np.uint32)
    assert osg.estimate_sigma(x, FP32) == pytest.approx(math.sqrt(5.0 / 3.0), rel=1e-15)     # ddof = 1
    two = np.array([3.0, 5.0], dtype=np.float32).view(np.uint32)
    assert osg.estimate_sigma(two, FP32) == pytest.approx(math.sqrt(2.0), rel=1e-15)
    assert math.isnan(osg.estimate_sigma(two[:1], FP32))


def test_matches_torch_std_the_routine_the_paper_names():
    rng = np.random.default_rng(0)
    f = rng.standard_normal(100_000, dtype=np.float32) * np.float32(0.02) + np.float32(0.003)
    w = W.f32_to_bf16_words(f)
    t = torch.from_numpy((w.astype(np.uint32) << 16).view(np.float32).copy()).double()
    assert osg.estimate_sigma(w, BF16) == pytest.approx(float(torch.std(t)), rel=1e-12)
    assert osg.estimate_sigma(f.view(np.uint32), FP32) == pytest.approx(float(torch.std(torch.from_numpy(f).double())), rel=1e-12)


def test_scale_equivariance_and_sampling():
    rng = np.random.default_rng(1)
    f = rng.standard_normal(1 << 18, dtype=np.float32)
    s1 = osg.estimate_sigma(f.view(np.uint32), FP32)
    assert abs(s1 - 1.0) < 5 / math.sqrt(2 * f.size)          # sampling error of a std estimate
    for k in (-20, -3, 7):
        g = (f * np.float32(2.0 ** k))                         # exact scaling
        assert osg.estimate_sigma(g.view(np.uint32), FP32) == pytest.approx(s1 * 2.0 ** k, rel=1e-14)


def test_table_from_estimate_and_fallbacks():
    rng = np.random.default_rng(2)
    for sigma, e0 in ((1.0, 122), (0.02, 116), (1e-4, 108)):
        w = W.f32_to_bf16_words(rng.standard_normal(1 << 16, dtype=np.float32) * np.float32(sigma))
        dec, s = osg.estimate_table(w, BF16)
        assert list(dec[1:]) == list(range(e0, e0 + 7)) and abs(s / sigma - 1) < 0.02
    for bad in (np.zeros(100, dtype=np.uint16), np.array([0x3F80], dtype=np.uint16),
                np.array([0x3F80, 0x7F80, 0x3F80], dtype=np.uint16), np.array([0x7FC0, 0, 0], dtype=np.uint16)):
        dec, s = osg.estimate_table(bad, BF16)
        assert list(dec) == [0, 1, 2, 3, 4, 5, 6, 7]


# ---- robust sigma: median of the magnitudes / Phi^-1(3/4) ----

def _f32w(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def test_robust_constant_is_the_normal_quartile():
    from scipy.special import ndtri, erf
    assert osg.PHI_INV_3_4 == pytest.approx(float(ndtri(0.75)), rel=1e-15)
    assert float(erf(osg.PHI_INV_3_4 / math.sqrt(2.0))) == pytest.approx(0.5, abs=1e-15)   # P(|w| < c sigma) = 1/2


def test_robust_hand_values_and_rank():
    c = osg.PHI_INV_3_4
    # lower median: rank (K - 1) // 2 of the sorted magnitudes; sign is ignored; every value here is a bf16 value
    assert osg.robust_sigma(_f32w([3.0, -1.0, 2.0, 4.0]), FP32) == 2.0 / c
    assert osg.robust_sigma(_f32w([3.0, -1.0, 2.0, 4.0, 8.0]), FP32) == 3.0 / c
    assert osg.robust_sigma(_f32w([-5.0]), FP32) == 5.0 / c
    assert osg.robust_sigma(W.f32_to_bf16_words(np.array([3.0, -1.0, 2.0, 4.0], dtype=np.float32)), BF16) == 2.0 / c
    # zeros, infinities and NaN are left out: [0, -0, 1, 2, 3, inf, nan] -> median of [1, 2, 3]
    x = np.array([0x0000, 0x8000, 0x3F80, 0x4000, 0x4040, 0x7F80, 0xFFC1], dtype=np.uint16)
    assert osg.robust_sigma(x, BF16) == 2.0 / c
    # an fp32 value counts with its bf16 prefix (truncated, not rounded): 1.99999 -> 1.9921875
    assert osg.robust_sigma(_f32w([1.99999]), FP32) == 1.9921875 / c
    # subnormals take part
    assert osg.robust_sigma(np.array([0x0001, 0x0002, 0x0003], dtype=np.uint16), BF16) == 2 * 2.0 ** -133 / c
    for nothing in (np.zeros(0, np.uint16), np.zeros(9, np.uint16), np.array([0x7F80, 0xFF80, 0x7FC0], np.uint16)):
        assert math.isnan(osg.robust_sigma(nothing, BF16))
        assert list(osg.robust_table(nothing, BF16)[0]) == [0, 1, 2, 3, 4, 5, 6, 7]


def test_robust_median_agrees_with_numpy_median_for_odd_counts():
    rng = np.random.default_rng(5)
    for n in (1, 3, 101, 4097):
        w = W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32) * np.float32(0.3))
        w = w[(w & 0x7FFF) != 0]
        if w.size % 2 == 0:
            w = w[1:]
        mags = ((w & 0x7FFF).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        assert osg.robust_sigma(w, BF16) == float(np.median(mags)) / osg.PHI_INV_3_4


def test_robust_on_clean_gaussians_is_sigma_within_sampling_error_and_scales_exactly():
    rng = np.random.default_rng(6)
    n = 1 << 18
    f = rng.standard_normal(n, dtype=np.float32)
    s1 = osg.robust_sigma(f.view(np.uint32), FP32)
    # asymptotic sd of the median-based sigma: 1 / (2 f(q) sqrt(n)) / q with f the half-normal density at the
    # quartile q, = 1.166 / sqrt(n); plus up to 2^-7 of truncation to the bf16 prefix
    assert -2.0 ** -7 - 5 * 1.166 / math.sqrt(n) < s1 - 1.0 < 5 * 1.166 / math.sqrt(n)
    for k in (-20, -3, 7):
        assert osg.robust_sigma((f * np.float32(2.0 ** k)).view(np.uint32), FP32) == s1 * 2.0 ** k     # bit for bit
    b = W.f32_to_bf16_words(f * np.float32(0.02))
    assert abs(osg.robust_sigma(b, BF16) / 0.02 - 1.0) < 2.0 ** -8 + 5 * 1.166 / math.sqrt(n)


def test_robust_ignores_what_poisons_the_sample_standard_deviation():
    """The two workloads on which the sample standard deviation picks a worse window: the estimate must stay
    within 10 % of the bulk sigma and choose the window of the nominal sigma."""
    from scipy.special import ndtri
    c5 = W.make("c5", 1 / 64)
    s = osg.robust_sigma(c5.data, c5.dtype)
    # closed form for the mixture: 5 % of the magnitudes sit near 1, so the median of all is the
    # 0.5 / 0.95 quantile of the bulk's magnitudes
    expect = 0.02 * float(ndtri(0.5 + 0.25 / 0.95)) / osg.PHI_INV_3_4
    assert s == pytest.approx(expect, rel=0.01) and abs(s / 0.02 - 1) < 0.10
    assert osg.estimate_sigma(c5.data, c5.dtype) > 0.2                      # ten times the bulk sigma
    assert list(osg.robust_table(c5.data, c5.dtype)[0]) == list(oracle.build_table(0.02))
    c2 = W.make("c2", 1 / 8)
    s = osg.robust_sigma(c2.data, c2.dtype)
    assert abs(s - 1.0) < 0.10 and osg.estimate_sigma(c2.data, c2.dtype) > 2.0
    assert list(osg.robust_table(c2.data, c2.dtype)[0]) == list(oracle.build_table(1.0))
    c5f = W.make("c5_fp32", 1 / 32)
    assert list(osg.robust_table(c5f.data, c5f.dtype)[0]) == list(oracle.build_table(0.02))
    # ratio with the estimated table within 1 % of the ratio with the nominal one
    for w in (c5, c2, c5f):
        nominal = oracle.compress(w.data, w.dtype, oracle.build_table(w.sigma), w.n_chunks, w.chunk_elems)[1].sum()
        robust = oracle.compress(w.data, w.dtype, osg.robust_table(w.data, w.dtype)[0], w.n_chunks, w.chunk_elems)[1].sum()
        assert abs(float(robust) / float(nominal) - 1.0) < 0.01


def test_robust_table_on_every_workload_is_the_nominal_one_or_better():
    for name, scale in (("c1", 1.0), ("c3", 1 / 32), ("c4", 1 / 64)):
        w = W.make(name, scale)
        dec, s = osg.robust_table(w.data, w.dtype)
        nominal = oracle.compress(w.data, w.dtype, oracle.build_table(w.sigma), w.n_chunks, w.chunk_elems)[1].sum()
        robust = oracle.compress(w.data, w.dtype, dec, w.n_chunks, w.chunk_elems)[1].sum()
        assert float(robust) <= float(nominal) * 1.01, (name, s, list(dec))


def test_robust_chunk_tables_follow_each_chunks_own_scale():
    """Chunks whose scales differ by orders of magnitude each get the window of their own sigma; with one table
    for all of them most chunks would be coded as zero-points only."""
    rng = np.random.default_rng(7)
    sigmas = [1e-4, 0.02, 1.0, 37.0]
    ce = [30000, 8192, 50001, 12345]
    x = np.concatenate([W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32) * np.float32(s)) for n, s in zip(ce, sigmas)])
    decs, est = osg.robust_chunk_tables(x, BF16, 4, ce)
    for c, s in enumerate(sigmas):
        assert list(decs[c]) == list(oracle.build_table(s)) and abs(est[c] / s - 1) < 0.05
    # an empty chunk and a chunk of zeros fall back to the lowest window
    decs, est = osg.robust_chunk_tables(np.concatenate([x[:100], np.zeros(50, np.uint16)]), BF16, 3, [100, 0, 50])
    assert list(decs[1]) == [0, 1, 2, 3, 4, 5, 6, 7] and list(decs[2]) == [0, 1, 2, 3, 4, 5, 6, 7] and math.isnan(est[1])
    # coded chunk by chunk with its own table, every chunk reaches the ratio of a Gaussian; with one table it cannot
    sizes = []
    start = 0
    for c, n in enumerate(ce):
        sizes.append(int(oracle.compress(x[start:start + n], BF16, osg.robust_chunk_tables(x, BF16, 4, ce)[0][c])[1][0]))
        start += n
    one = int(oracle.compress(x, BF16, osg.robust_table(x, BF16)[0], 4, ce)[1].sum())
    assert x.nbytes / sum(sizes) > 1.38 and x.nbytes / one < 1.1


# --- the robust estimate from a stratified sample of whole groups ---------------------------------------------

def test_sample_with_stride_one_is_everything():
    rng = np.random.default_rng(21)
    for n in (0, 1, 511, 512, 513, 5000):
        x = W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32))
        assert np.array_equal(osg.sample_of(x, 1), x)
        a, b = osg.robust_sigma_sampled(x, BF16, 1), osg.robust_sigma(x, BF16)
        assert a == b or (math.isnan(a) and math.isnan(b))


def test_sampled_groups_hand_values_and_stratification():
    # positions from Knuth's constant by plain integer arithmetic: ((k * 2654435761) mod 2^32) >> 16, mod S
    assert list(osg.sampled_groups(8 * 16 * 512, 16)) == [0, 23, 46, 54, 77, 85, 108, 116]
    assert list(osg.sampled_groups(8 * 4 * 512, 4)) == [0, 7, 10, 14, 17, 21, 24, 28]
    for n, s in ((1_000_000, 16), (777_777, 8), (512 * 64 + 1, 64), (100, 4), (0, 4)):
        g = osg.sampled_groups(n, s)
        ng = -(-n // 512)
        assert np.all(np.diff(g) > 0) and np.all(g < ng)
        assert np.array_equal(np.unique(g // s), g // s)                       # one group per block at most
        full_blocks = ng // s
        assert np.array_equal((g // s)[:full_blocks], np.arange(full_blocks))  # and every full block has one
        assert g.size in (full_blocks, -(-ng // s))
    # a last group that is cut short gives the values it has; one that lies past the end gives nothing
    x = np.arange(512 * 23 + 100, dtype=np.uint16)                             # groups 0..23, the last one of 100 values
    s = osg.sample_of(x, 16)                                                   # takes groups 0 and 23
    assert s.size == 512 + 100 and s[0] == 0 and s[512] == 512 * 23 and s[-1] == x[-1]
    assert osg.sample_of(x[:512 * 23], 16).size == 512                         # group 23 is past the end now


def test_sample_positions_do_not_alias_with_power_of_two_periods():
    """A row of 4096 values is 8 groups, one of 8192 values 16: the position of the sampled group inside such a
    period must take every value about equally often (a fixed stride of 16 groups would always give 0)."""
    for s in (4, 16, 64):
        g = osg.sampled_groups(512 * s * 8192, s)
        assert g.size == 8192
        assert set(g % s) == set(range(s))
        for period in (8, 16, 32):
            counts = np.bincount(g % period, minlength=period)
            assert counts.min() > 0.8 * g.size / period and counts.max() < 1.2 * g.size / period, (s, period, counts)


def test_sampled_estimate_finds_the_same_window_as_the_full_one():
    rng = np.random.default_rng(22)
    x = W.f32_to_bf16_words(rng.standard_normal(1 << 22, dtype=np.float32) * np.float32(0.02))
    full = osg.robust_sigma(x, BF16)
    for s in (4, 16, 64):
        est = osg.robust_sigma_sampled(x, BF16, s)
        assert abs(est / full - 1) < 0.01, (s, est, full)
    # structure the sample must not trip over: outlier columns (c2) and gain rows among weights (c5)
    for name, scale in (("c2", 1 / 4), ("c5", 1 / 64), ("c4", 1 / 32), ("c5_fp32", 1 / 32)):
        w = W.make(name, scale)
        want = list(osg.robust_table(w.data, w.dtype)[0])
        for s in (8, 16):
            d, sig = osg.robust_table(osg.sample_of(w.data, s), w.dtype)
            assert list(d) == want, (name, s, sig)


def test_sampled_chunk_tables_number_the_groups_from_each_chunks_start():
    rng = np.random.default_rng(23)
    ce = [512 * 40 + 7, 0, 300, 512 * 16 * 3]
    sig = [1e-3, 1.0, 5.0, 0.3]
    x = np.concatenate([W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32) * np.float32(s)) for n, s in zip(ce, sig)])
    decs, est = osg.robust_chunk_tables_sampled(x, BF16, 4, ce, stride=16)
    start = 0
    for c, n in enumerate(ce):
        d, s = osg.robust_table(osg.sample_of(x[start:start + n], 16), BF16)
        assert list(decs[c]) == list(d) and (est[c] == s or (math.isnan(est[c]) and math.isnan(s)))
        start += n
    assert list(decs[0]) == list(oracle.build_table(1e-3)) and list(decs[3]) == list(oracle.build_table(0.3))
    assert list(decs[1]) == [0, 1, 2, 3, 4, 5, 6, 7]
