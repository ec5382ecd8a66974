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
