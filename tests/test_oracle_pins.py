"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without the GPU.

Each test names the passage it pins.  None of the expected values comes from the HIP path.
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy import integrate, stats

import oracle
from oracle import BF16, FP32
from paper_2604_27844_amd import workloads as W

import format_witness as fw

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_kv(path):
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, *v = line.split()
            out[k] = v
    return out


def _pwin_quadrature(sigma, x):
    """Eq.1 evaluated by numerical integration of the Gaussian density (no erf involved)."""
    f = lambda t: math.exp(-t * t / (2 * sigma * sigma)) / math.sqrt(2 * math.pi * sigma * sigma)
    a, b = 2.0 ** x, 2.0 ** (x + 7)
    pts = [a * 2 ** k for k in range(1, 7)]
    val, _ = integrate.quad(f, a, b, points=pts, epsabs=1e-13, epsrel=1e-12, limit=400)
    return 2 * val


# ---------------------------------------------------------------- section 4.1: Eq.1-5
def test_eq4_eq5_constants_as_printed():
    g = _read_kv(os.path.join(GOLD, "section4_constants.txt"))
    c = oracle.xopt(1.0)                                   # Eq.5 at sigma = 1
    assert abs(c - float(g["xopt_minus_log2sigma"][0])) <= float(g["xopt_minus_log2sigma"][1])
    assert abs(c - (-5.36066)) < 1e-5                      # the exact expression
    u = 2.0 ** c / math.sqrt(2.0)                          # definition of u(x) at sigma = 1
    assert abs(u - float(g["u_opt"][0])) <= float(g["u_opt"][1])
    # Eq.4 is the root of the optimality condition 128 exp(-(128u)^2) = exp(-u^2)
    assert abs(128 * math.exp(-(128 * u) ** 2) - math.exp(-u * u)) < 1e-12
    for s in (1e-4, 0.02, 0.5, 3.0, 1000.0):               # Eq.5 is log2(sigma) + const
        assert abs(oracle.xopt(s) - (math.log2(s) + c)) < 1e-12


@pytest.mark.parametrize("sigma", [1e-4, 0.02, 0.5, 1.0, 7.3])
def test_eq2_equals_eq1_by_quadrature(sigma):
    x0 = round(oracle.xopt(sigma))
    for x in range(x0 - 3, x0 + 4):
        assert abs(oracle.pwin(sigma, x) - _pwin_quadrature(sigma, x)) < 1e-9


def test_eq5_is_the_continuous_maximiser_of_eq2():
    # scan a fine grid of real x around Eq.5's optimum with an independent cdf
    for sigma in (0.02, 1.0):
        xo = oracle.xopt(sigma)
        xs = np.linspace(xo - 2, xo + 2, 4001)
        p = 2 * (stats.norm.cdf(2.0 ** (xs + 7), scale=sigma) - stats.norm.cdf(2.0 ** xs, scale=sigma))
        assert abs(xs[np.argmax(p)] - xo) < 2e-3


def test_table_for_named_sigmas():
    # sigma -> first exponent of the window (biased); window is 7 consecutive exponents
    for sigma, e0 in ((1.0, 122), (0.5, 121), (0.02, 116), (1e-4, 108)):
        dec = oracle.build_table(sigma)
        assert dec[0] == 0 and list(dec[1:]) == list(range(e0, e0 + 7))
    assert abs(oracle.pwin(1.0, -5) - 0.97501) < 1e-5
    assert abs(oracle.pwin(0.02, 116 - 127) - 0.97874) < 1e-5


def test_table_is_integer_argmax_of_eq2_by_brute_force():
    # every integer base, independent cdf; includes the band where round(x_opt) is NOT the argmax
    sigmas = np.concatenate([np.exp(np.linspace(math.log(1e-6), math.log(1e4), 173)),
                             0.82335 * 2.0 ** np.arange(-3, 4) * 1.001, 0.82335 * 2.0 ** np.arange(-3, 4) * 0.999])
    xs = np.arange(-126, 122)
    differs_from_round = 0
    for sigma in sigmas:
        p = 2 * (stats.norm.cdf(2.0 ** (xs + 7.0), scale=sigma) - stats.norm.cdf(2.0 ** (xs + 0.0), scale=sigma))
        best = int(xs[np.argmax(p)])
        dec = oracle.build_table(float(sigma))
        assert int(dec[1]) - 127 == best, sigma
        differs_from_round += best != round(oracle.xopt(float(sigma)))
    assert differs_from_round > 0      # the grid did exercise the floor/ceil decision


def test_table_clamps_and_rejects_bad_sigma():
    assert list(oracle.build_table(1e-45)[1:]) == list(range(1, 8))
    assert list(oracle.build_table(1e300)[1:]) == list(range(248, 255))
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(oracle.OracleError):
            oracle.build_table(bad)


@pytest.mark.parametrize("sigma", [1e-4, 0.02, 0.5, 1.0])
def test_window_equals_empirical_top7(sigma):
    # section 4.1's claim: the 7 most frequent exponents of Gaussian data are the window
    rng = np.random.default_rng(11)
    w = W.f32_to_bf16_words(rng.standard_normal(1 << 21, dtype=np.float32) * np.float32(sigma))
    hist = np.bincount((w >> 7) & 0xFF, minlength=256)
    top7 = sorted(int(e) for e in np.argsort(hist)[-7:])
    assert top7 == list(oracle.build_table(sigma)[1:])


# ---------------------------------------------------------------- Table 1 and code length
def _codes_of(slot):
    hd = fw.read_header(slot)
    off = fw.section_offsets(hd["n"], hd["dtype"], hd["G"])
    nb = -(-hd["n"] // 8)
    code = np.zeros(hd["n"], dtype=np.uint8)
    for k in range(3):
        code |= np.unpackbits(slot[off[f"P{k}"]:off[f"P{k}"] + nb], bitorder="little")[:hd["n"]] << k
    return code


def test_table1_coverage_from_oracle_codes():
    rows = [l.split() for l in open(os.path.join(GOLD, "table1_topk_coverage.txt")) if l[0].isdigit()]
    paper = [float(r[1]) for r in rows]
    rng = np.random.default_rng(5)
    x = W.f32_to_bf16_words(rng.standard_normal(1 << 22, dtype=np.float32))
    out, cb, off = oracle.compress(x, BF16, oracle.build_table(1.0))
    freq = np.bincount(_codes_of(out), minlength=8)[1:] / x.size     # codes 1..7 = window exponents
    cum = 100 * np.cumsum(np.sort(freq)[::-1])
    assert np.all(np.abs(cum - np.array(paper)) < 0.15), cum        # paper prints 1 decimal


@pytest.mark.parametrize("sigma,dtype", [(0.02, BF16), (1.0, BF16), (0.5, BF16), (0.02, FP32)])
def test_ratio_matches_closed_form_code_length(sigma, dtype):
    # section 4: 8 verbatim bits + 3 code bits (+16 raw low bits for fp32) + 8 bits per zero-point,
    # plus this layout's 32/G index bits; zero-point probability from Eq.2 with an independent cdf.
    n, G = 1 << 20, 512
    rng = np.random.default_rng(17)
    f = rng.standard_normal(n, dtype=np.float32) * np.float32(sigma)
    x = W.f32_to_bf16_words(f) if dtype == BF16 else f.view(np.uint32)
    dec = oracle.build_table(sigma)
    xlo = int(dec[1]) - 127
    p_in = 2 * (stats.norm.cdf(2.0 ** (xlo + 7), scale=sigma) - stats.norm.cdf(2.0 ** xlo, scale=sigma))
    p_esc = 1 - p_in
    out, cb, _ = oracle.compress(x, dtype, dec)
    n_esc = fw.read_header(out)["n_esc"]
    sd = math.sqrt(n * p_esc * (1 - p_esc))
    assert abs(n_esc - n * p_esc) < 5 * sd + 1e-4 * n       # binomial spread + bf16 rounding at the edges
    bits = (16 if dtype == BF16 else 32)
    closed = bits / ((bits - 5) + 8 * p_esc + 32 / G)
    ratio = x.nbytes / float(cb.sum())
    assert abs(ratio / closed - 1) < 2e-3                    # header + padding + sampling noise
    assert ratio < bits / (bits - 5)                         # "up to 31%": 16/11 is the ceiling


def test_code_length_constants():
    g = _read_kv(os.path.join(GOLD, "section4_constants.txt"))
    # a chunk with no zero-points costs exactly 8+3 bits per value + index + header
    n, G = 1 << 16, 512
    x = np.full(n, 0x3F80, dtype=np.uint16)                 # all 1.0, inside the sigma=1 window
    out, cb, _ = oracle.compress(x, BF16, oracle.build_table(1.0))
    assert int(cb[0]) == 128 + n + 3 * n // 8 + 4 * n // G
    assert (n + 3 * n // 8) * 8 / n == float(g["bits_per_bf16_value"][0])
    assert abs(100 * (1 - 11 / 16) - float(g["max_saving_percent"][0])) <= float(g["max_saving_percent"][1])


# ---------------------------------------------------------------- layout: hand example, sizes
def test_hand_example_stream():
    g = _read_kv(os.path.join(GOLD, "hand_example_sigma1.txt"))
    x = np.array([int(v, 16) for v in g["input"]], dtype=np.uint16)
    out, cb, off = oracle.compress(x, BF16, oracle.build_table(1.0))
    assert int(cb[0]) == int(g["chunk_bytes"][0]) and list(off) == [0, 896]
    exp = np.zeros(896, dtype=np.uint8)
    hdr = b"ZPCL" + (1).to_bytes(4, "little") + (0).to_bytes(4, "little") + (512).to_bytes(4, "little") + \
        (4).to_bytes(8, "little") + int(g["n_esc"][0]).to_bytes(8, "little") + (896).to_bytes(8, "little") + \
        bytes([0, 122, 123, 124, 125, 126, 127, 128])
    exp[:len(hdr)] = np.frombuffer(hdr, dtype=np.uint8)
    exp[128:132] = [int(v, 16) for v in g["sm"]]
    exp[256] = int(g["p0"][0], 16)
    exp[384] = int(g["p1"][0], 16)
    exp[512] = int(g["p2"][0], 16)
    exp[640:644] = [int(g["idx"][0]), 0, 0, 0]
    exp[768] = int(g["esc"][0], 16)
    assert np.array_equal(out[:896], exp)
    assert np.array_equal(oracle.decompress(out, 4, BF16), x)


@pytest.mark.parametrize("dtype", [BF16, FP32])
def test_static_size_is_input_independent_and_aligned(dtype):
    # section 4: only the zero-point list has a data-dependent size; section 4.2.1: 128 B alignment
    rng = np.random.default_rng(3)
    ce = np.array([0, 1, 7, 8, 511, 512, 513, 4096, 5000, 127, 128, 129], dtype=np.uint64)
    n = int(ce.sum())
    off = oracle.slot_offsets(n, dtype, len(ce), ce)
    assert np.all(off % 128 == 0)
    for c, nc in enumerate(int(v) for v in ce):
        so = fw.section_offsets(nc, dtype, 512)
        assert all(v % 128 == 0 for v in so.values())
        assert so["CAP"] == int(off[c + 1] - off[c]) == oracle.slot_cap(nc, dtype)
    words = np.uint16 if dtype == BF16 else np.uint32
    a = rng.integers(0, np.iinfo(words).max, n, dtype=words, endpoint=True)
    b = np.zeros(n, dtype=words)
    dec = oracle.build_table(1.0)
    oa, cba, _ = oracle.compress(a, dtype, dec, len(ce), ce)
    ob, cbb, _ = oracle.compress(b, dtype, dec, len(ce), ce)
    for c, nc in enumerate(int(v) for v in ce):
        ha, hb = fw.read_header(oa[int(off[c]):]), fw.read_header(ob[int(off[c]):])
        static = fw.section_offsets(nc, dtype, 512)["ESC"]
        assert int(cba[c]) == static + -(-ha["n_esc"] // 128) * 128 == ha["chunk_bytes"]
        assert int(cbb[c]) == static + -(-hb["n_esc"] // 128) * 128 and hb["n_esc"] == nc   # zeros all escape
        assert int(cba[c]) == oracle.chunk_bytes(nc, ha["n_esc"], dtype)


def test_padding_and_tail_bits_are_zero():
    rng = np.random.default_rng(9)
    n = 1000                                                # not a multiple of 8, 128 or G
    x = W.f32_to_bf16_words(rng.standard_normal(n, dtype=np.float32))
    out, cb, _ = oracle.compress(x, BF16, oracle.build_table(1.0))
    so = fw.section_offsets(n, BF16, 512)
    hd = fw.read_header(out)
    assert hd["rest"] == bytes(80)
    assert not out[so["SM"] + n:so["P0"]].any()
    for k in range(3):
        sec = out[so[f"P{k}"]:so[f"P{k}"] + 128]
        assert not (sec[n // 8] >> (n % 8)) and not sec[n // 8 + 1:].any()
    assert not out[so["IDX"] + 8:so["ESC"]].any()
    assert not out[so["ESC"] + hd["n_esc"]:int(cb[0])].any()


# ---------------------------------------------------------------- losslessness
def test_roundtrip_all_bf16_patterns():
    x = np.arange(65536, dtype=np.uint16)
    for sigma in (1.0, 0.02, 1e-45, 1e300):
        dec = oracle.build_table(sigma)
        out, cb, _ = oracle.compress(x, BF16, dec)
        assert np.array_equal(oracle.decompress(out[:int(cb[0])], x.size, BF16), x)
        assert np.array_equal(fw.decode_slot(out), x)
    dec = oracle.build_table(1.0)
    for v in range(0, 65536, 7):                            # singly, too
        one = np.array([v], dtype=np.uint16)
        out, cb, _ = oracle.compress(one, BF16, dec)
        assert oracle.decompress(out, 1, BF16)[0] == v


def test_roundtrip_fp32_bit_patterns_with_specials():
    rng = np.random.default_rng(21)
    x = rng.integers(0, 2 ** 32, 200_003, dtype=np.uint64).astype(np.uint32)   # random words: NaNs, subnormals
    x[:8] = [0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00001, 0xFFFFFFFF, 0x00000001, 0x807FFFFF]
    ce = np.array([100_000, 0, 3, 100_000], dtype=np.uint64)
    out, cb, off = oracle.compress(x, FP32, oracle.build_table(0.02), 4, ce)
    assert np.array_equal(oracle.decompress(out, x.size, FP32, 4, ce), x)
    got = np.concatenate([fw.decode_slot(out[int(off[c]):int(off[c + 1])]) for c in range(4)])
    assert np.array_equal(got.astype(np.uint32), x)


@pytest.mark.parametrize("name,scale", [("c1", 1.0), ("c2", 1 / 16), ("c3", 1 / 64), ("c4", 1 / 128),
                                        ("c5", 1 / 256), ("c5_fp32", 1 / 64)])
def test_roundtrip_and_independent_decoder_on_workloads(name, scale):
    w = W.make(name, scale)
    dec = oracle.build_table(w.sigma)
    out, cb, off = oracle.compress(w.data, w.dtype, dec, w.n_chunks, w.chunk_elems)
    assert np.array_equal(oracle.decompress(out, w.n_elems, w.dtype, w.n_chunks, w.chunk_elems), w.data)
    ce = w.chunk_elems if w.chunk_elems is not None else np.full(w.n_chunks, w.n_elems // w.n_chunks)
    start = 0
    for c in range(w.n_chunks):
        nc = int(ce[c])
        slot = out[int(off[c]):int(off[c]) + int(cb[c])]    # only the transmitted bytes
        # a peer decodes its slice alone (n_chunks = 1), with both decoders
        assert np.array_equal(oracle.decompress(slot, nc, w.dtype), w.data[start:start + nc])
        if c % 16 == 0:
            assert np.array_equal(fw.decode_slot(slot), w.data[start:start + nc])
        start += nc


def test_chunked_equals_per_chunk_calls():
    # per-peer independence: compressing a slice alone gives exactly that slot's bytes
    w = W.make("c2", 1 / 64)
    dec = oracle.build_table(w.sigma)
    out, cb, off = oracle.compress(w.data, w.dtype, dec, w.n_chunks)
    nc = w.n_elems // w.n_chunks
    for c in range(w.n_chunks):
        o1, cb1, _ = oracle.compress(w.data[c * nc:(c + 1) * nc], w.dtype, dec)
        assert cb1[0] == cb[c]
        assert np.array_equal(o1[:int(cb1[0])], out[int(off[c]):int(off[c]) + int(cb[c])])


# ---------------------------------------------------------------- encoder is canonical (brute force)
def test_encoder_is_unique_shortest_by_brute_force():
    e0 = 122
    dec = oracle.build_table(1.0)
    alphabet = [0, e0 - 1, e0, e0 + 6, e0 + 7, 255]
    checked = 0
    for n in (1, 2, 3):
        for exps in itertools.product(alphabet, repeat=n):
            words = [((i & 1) << 15) | (e << 7) | (0x55 ^ i) & 0x7F for i, e in enumerate(exps)]
            x = np.array(words, dtype=np.uint16)
            enc_out, cb, _ = oracle.compress(x, BF16, dec)
            accepted = []
            for codes in itertools.product(range(8), repeat=n):
                n0 = sum(c == 0 for c in codes)
                for esc in itertools.product(alphabet, repeat=n0):
                    slot, used = fw.write_slot(words, BF16, 512, list(dec), list(codes), list(esc))
                    try:
                        y = oracle.decompress(slot[:used], n, BF16)
                    except oracle.OracleError:
                        continue
                    if np.array_equal(y, x):
                        accepted.append((used, n0, codes, esc, slot))
            assert accepted
            fewest = min(a[1] for a in accepted)
            best = [a for a in accepted if a[1] == fewest]
            assert len(best) == 1                         # unique stream with the fewest zero-points
            assert np.array_equal(best[0][4][:best[0][0]], enc_out[:int(cb[0])])
            # and there are as many accepted streams as ways to demote in-window exponents
            assert len(accepted) == 2 ** sum(e0 <= e <= e0 + 6 for e in exps)
            checked += 1
    assert checked == 6 + 36 + 216


def test_group_index_crosses_groups_with_small_G():
    # zero-point positions across group boundaries (G = 8 makes many groups in a tiny input)
    rng = np.random.default_rng(2)
    x = rng.integers(0, 65536, 203, dtype=np.uint16, endpoint=False)
    dec = oracle.build_table(1.0)
    for G in (1, 8, 64, 512):
        out, cb, _ = oracle.compress(x, BF16, dec, G=G)
        assert np.array_equal(oracle.decompress(out, x.size, BF16), x)
        assert np.array_equal(fw.decode_slot(out), x)
        hd = fw.read_header(out)
        off = fw.section_offsets(x.size, BF16, G)
        idx = out[off["IDX"]:off["IDX"] + 4 * (-(-x.size // G))].view("<u4")
        E = (x >> 7) & 0xFF
        esc_mask = (E < 122) | (E > 128)
        want = np.concatenate([[0], np.cumsum(esc_mask)])[np.arange(0, x.size, G)]
        assert np.array_equal(idx, want) and hd["n_esc"] == int(esc_mask.sum())
        assert np.array_equal(out[off["ESC"]:off["ESC"] + hd["n_esc"]], E[esc_mask].astype(np.uint8))


# ---------------------------------------------------------------- error paths
def test_decoder_rejects_corrupt_streams():
    x = W.make("c1", 1 / 256).data
    dec = oracle.build_table(0.02)
    out, cb, _ = oracle.compress(x, BF16, dec)
    good = out[:int(cb[0])].copy()
    assert np.array_equal(oracle.decompress(good, x.size, BF16), x)
    so = fw.section_offsets(x.size, BF16, 512)
    for pos in (0, 4, 8, 13, 16, 24, 32, so["IDX"] + 4):
        bad = good.copy()
        bad[pos] ^= 0x01
        with pytest.raises(oracle.OracleError) as ei:
            oracle.decompress(bad, x.size, BF16)
        assert ei.value.code == 4
    with pytest.raises(oracle.OracleError):
        oracle.decompress(good[:-128], x.size, BF16)        # truncated
    with pytest.raises(oracle.OracleError):
        oracle.decompress(good, x.size + 1, BF16)           # wrong element count
    with pytest.raises(oracle.OracleError):
        oracle.compress(x[:1001], BF16, dec, n_chunks=2)    # equal split must divide
    with pytest.raises(oracle.OracleError):
        oracle.compress(x, 7, dec)                          # unknown dtype code
