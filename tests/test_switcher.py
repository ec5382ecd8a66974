"""Adaptive Reduce-Scatter switcher (paper section 5.2, Eq.6-7): oracle pins and library-vs-oracle checks."""
import math

import numpy as np
import pytest

from oracle import switcher as osw
import paper_2604_27844_amd.binding as z


def test_oracle_crossover_closed_form():
    # T_A2A < T_RS  <=>  d > (alpha_a2a - alpha_rs) / (beta_rs - beta_a2a e s) when the zipped slope is smaller
    a_rs, b_rs, a_a2a, b_a2a, e, s = 20e-6, 1 / 20e9, 60e-6, 1 / 25e9, 1 / 1.4, 1.0
    d_star = (a_a2a - a_rs) / (b_rs - b_a2a * e * s)
    assert d_star > 0
    assert not osw.prefers_zipped(a_rs, b_rs, a_a2a, b_a2a, e, s, d_star * 0.999)
    assert osw.prefers_zipped(a_rs, b_rs, a_a2a, b_a2a, e, s, d_star * 1.001)
    # no compression, same link, larger start-up: never switch
    assert not any(osw.prefers_zipped(a_rs, b_rs, a_a2a, b_rs, 1.0, 1.0, d) for d in (1e3, 1e6, 1e9, 1e12))
    # the paper's s: native collective in a format twice as wide halves the zipped volume
    assert osw.t_a2a(0.0, 1e-9, 0.7, 0.5, 1e6) == pytest.approx(0.35e-3)
    assert osw.t_rs(1e-5, 1e-9, 1e6) == pytest.approx(1e-5 + 1e-3)


def test_oracle_fit_recovers_a_line_and_matches_polyfit():
    ds = [2.0 ** k for k in range(10, 28, 2)]
    ts = [30e-6 + d / 18e9 for d in ds]
    a, b = osw.fit_linear(ds, ts)
    assert a == pytest.approx(30e-6, rel=1e-9) and b == pytest.approx(1 / 18e9, rel=1e-9)
    rng = np.random.default_rng(0)
    noisy = [t * (1 + 0.05 * rng.standard_normal()) for t in ts]
    a, b = osw.fit_linear(ds, noisy)
    pb, pa = np.polyfit(ds, noisy, 1)
    assert a == pytest.approx(pa, rel=1e-6) and b == pytest.approx(pb, rel=1e-9)


def test_library_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(2000):
        a_rs, a_a2a = rng.uniform(1e-6, 1e-4, 2)
        b_rs, b_a2a = 1 / rng.uniform(5e9, 200e9, 2)
        e, s = rng.uniform(0.5, 1.1), rng.choice([0.5, 1.0, 2.0])
        d = float(np.exp(rng.uniform(math.log(1e3), math.log(1e10))))
        dec, t_rs, t_a2a = z.zipccl_switch_prefers_zipped(a_rs, b_rs, a_a2a, b_a2a, d, e, s)
        assert t_rs == osw.t_rs(a_rs, b_rs, d) and t_a2a == osw.t_a2a(a_a2a, b_a2a, e, s, d)   # same fp64 expression
        assert dec == int(osw.prefers_zipped(a_rs, b_rs, a_a2a, b_a2a, e, s, d))
    ds = [1e4, 1e5, 1e6, 1e7, 3e7]
    ts = [1e-5 + 2e-10 * d * (1 + 0.01 * math.sin(i)) for i, d in enumerate(ds)]
    a, b = z.zipccl_fit_link_model(ds, ts)
    oa, ob = osw.fit_linear(ds, ts)
    assert a == pytest.approx(oa, rel=1e-12) and b == pytest.approx(ob, rel=1e-12)


def test_library_rejects_bad_arguments():
    assert z.zipccl_switch_prefers_zipped(-1.0, 1e-9, 1e-5, 1e-9, 1e6, 0.7, 1.0)[0] == -1
    assert z.zipccl_switch_prefers_zipped(1e-5, 1e-9, 1e-5, 1e-9, float("nan"), 0.7, 1.0)[0] == -1
    assert z._lib.zipccl_switch_prefers_zipped(None, 1.0, 1.0, 1.0, None, None) == -1
    with pytest.raises(z.ZipcclError):
        z.zipccl_fit_link_model([1e6, 1e6], [1e-3, 2e-3])           # a single size: no slope
    with pytest.raises(z.ZipcclError):
        z.zipccl_fit_link_model([1e6], [1e-3])
