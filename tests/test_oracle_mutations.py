"""Does a plausible mistake anywhere in the oracle fail one of its pins?

Every case below plants ONE mistake (a dropped term, a wrong sign or index, a shifted constant, a swapped order)
in a private copy of ``oracle/`` -- on the CPU, never in the repository's files and never in anything the GPU
runs -- and runs the pin tests against that copy in a child process.  The pins must fail for every planted
mistake and pass for the untouched copy.  A mistake that survives names a hole in the pins.

The pins that compare the oracle with the HIP library are left out: they are parity checks, not pins.
"""
import concurrent.futures
import os
import shutil
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
C, SIGMA, SWITCH = "zipccl_oracle.c", "sigma.py", "switcher.py"
CODEC = ["tests/test_oracle_pins.py", "--deselect",
         "tests/test_oracle_pins.py::test_encoder_is_unique_shortest_by_brute_force"]     # 14 s on its own; not needed here
REDUCE = ["tests/test_oracle_reduce_pins.py"]
SIG = ["tests/test_oracle_sigma_pins.py"]
SW = ["tests/test_switcher.py", "-k", "oracle"]

# (name, file, text as it stands, text with the mistake, pin files to run)
MISTAKES = [
    ("sign and mantissa swapped in the SM byte", C, "(sign << 7) | mant", "(mant << 1) | sign", CODEC),
    ("plane bits filled from the top of the byte", C, "p1[i >> 3] |= (uint8_t)(((code >> 1) & 1u) << (i & 7));",
     "p1[i >> 3] |= (uint8_t)(((code >> 1) & 1u) << (7 - (i & 7)));", CODEC),
    ("Eq.5 with 7 ln 2 for 14 ln 2", C, "0.5 * log2(14.0 * log(2.0) / 16383.0)", "0.5 * log2(7.0 * log(2.0) / 16383.0)", CODEC),
    ("window of eight exponents in Eq.2", C, "erf(ldexp(1.0, x + 7) / s)", "erf(ldexp(1.0, x + 8) / s)", CODEC),
    ("table one exponent too high", C, "dec[k] = (uint8_t)(e0 + k - 1)", "dec[k] = (uint8_t)(e0 + k)", CODEC),
    ("the window's first exponent coded as a zero-point too", C, "if (code == 0) esc[n_esc++] = (uint8_t)E;",
     "if (code == 0 || code == 1) esc[n_esc++] = (uint8_t)E;", CODEC),
    ("index holds the inclusive count", C, "put32(idx + 4 * (i / G), (uint32_t)n_esc);",
     "put32(idx + 4 * (i / G), (uint32_t)n_esc + (i > 0));", CODEC),
    ("argmax of Eq.2 taken the wrong way round", C, "(zo_pwin(sigma, xh) > zo_pwin(sigma, xl)) ? xh : xl",
     "(zo_pwin(sigma, xh) < zo_pwin(sigma, xl)) ? xh : xl", CODEC),
    ("slot capacity 128 bytes too large", C, "    c += zo_pad(4 * zo_ceil_div(n, G));", "    c += zo_pad(4 * zo_ceil_div(n, G)) + 128;", CODEC),
    ("fp32 low bytes lose a bit", C, "lo[2 * i + 1] = in[4 * i + 1];", "lo[2 * i + 1] = in[4 * i + 1] & 0x7Fu;", CODEC),
    ("decoder reads the wrong table entry for code 7", C, "            E = dec[code];", "            E = dec[code] + (code == 7u);", CODEC),
    ("decoder takes the zero-points of a group in reverse", C, "            E = esc[base + rank];",
     "            E = esc[base + (rank ^ 1u)];", CODEC),
    ("decoder puts the sign into the exponent's top bit", C, "((uint32_t)(sm[i] & 0x80u) << 8) | (E << 7)",
     "((uint32_t)(sm[i] & 0x80u) << 7) | (E << 7)", CODEC),
    ("reduce starts from +0", C, "if (p == 0) acc[i] = -0.0f;", "if (p == 0) acc[i] = 0.0f;", REDUCE),
    ("reduce adds the slots last to first", C, "const uint64_t off = (uint64_t)p * cap;",
     "const uint64_t off = (uint64_t)(n_peers - 1u - p) * cap;", REDUCE),
    ("reduce accumulates in FP64", C, "            acc[i] = acc[i] + x;", "            { static double wide[1 << 20]; wide[i] = (p == 0 ? -0.0 : wide[i]) + (double)x; acc[i] = (float)wide[i]; }", REDUCE),
    ("bf16 output rounds halves up", C, "u += 0x7FFFu + ((u >> 16) & 1u);", "u += 0x8000u;", REDUCE),
    ("NaN sums keep whatever bits the machine gave them", C, "if (isnan(acc[i])) bits = 0x7FC00000u;", "", REDUCE),
    ("sample standard deviation divides by N", SIGMA, "((x - m) ** 2).sum() / (x.size - 1)", "((x - m) ** 2).sum() / x.size", SIG),
    ("upper median for lower median", SIGMA, "np.sort(mag)[(mag.size - 1) // 2]", "np.sort(mag)[mag.size // 2]", SIG),
    ("zeros count as magnitudes", SIGMA, "mag = mag[(mag != 0) & (mag < 0x7F80)]", "mag = mag[mag < 0x7F80]", SIG),
    ("Inf and NaN count as magnitudes", SIGMA, "mag = mag[(mag != 0) & (mag < 0x7F80)]", "mag = mag[mag != 0]", SIG),
    ("the normal quartile to three digits", SIGMA, "PHI_INV_3_4 = 0.6744897501960817", "PHI_INV_3_4 = 0.674", SIG),
    ("sample position from the hash's low half", SIGMA, "(((k * SAMPLE_MULT) % (1 << 32)) >> 16) % stride",
     "((k * SAMPLE_MULT) % (1 << 32)) % stride", SIG),
    ("sample position fixed inside the block", SIGMA, "g = k * stride + (((k * SAMPLE_MULT) % (1 << 32)) >> 16) % stride",
     "g = k * stride", SIG),
    ("sampled groups of 256 values", SIGMA, "SAMPLE_GROUP = 512", "SAMPLE_GROUP = 256", SIG),
    ("switcher divides by the precision factor", SWITCH, "beta_a2a * e * s * d", "beta_a2a * e / s * d", SW),
]


def _run(name, file, old, new, pins):
    tmp = tempfile.mkdtemp(prefix="zipccl_mut_")
    try:
        dst = os.path.join(tmp, "oracle")
        shutil.copytree(os.path.join(ROOT, "oracle"), dst, ignore=shutil.ignore_patterns("*.so", "__pycache__", "*.tmp"))
        if file is not None:
            path = os.path.join(dst, file)
            text = open(path).read()
            assert text.count(old) == 1, f"{name}: the text to change occurs {text.count(old)} times in oracle/{file}"
            open(path, "w").write(text.replace(old, new))
        env = dict(os.environ, PYTHONPATH=os.pathsep.join([tmp, ROOT]), PYTHONDONTWRITEBYTECODE="1")
        code = ("import sys, oracle, pytest\n"                                      # exit 3: the copy is not what runs, or
                "assert oracle.__file__.startswith(sys.argv[1]), oracle.__file__\n"   # does not compile (no pin's merit)
                "try:\n    oracle.build(force=True)\nexcept Exception as e:\n    print(e)\n    sys.exit(3)\n"
                "sys.exit(pytest.main(sys.argv[2:]))")
        args = [os.path.join(ROOT, a) if a.endswith(".py") else a for a in pins]      # the copy's directory is the child's cwd
        cmd = [sys.executable, "-c", code, tmp, "--rootdir", ROOT, "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + args
        r = subprocess.run(cmd, cwd=tmp, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
        return name, r.returncode, r.stdout[-1500:]
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def test_untouched_copy_passes_every_pin_used_here():
    for pins in (CODEC, REDUCE, SIG, SW):
        name, rc, out = _run("untouched", None, None, None, pins)
        assert rc == 0, out


def test_every_planted_mistake_fails_a_pin():
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda m: _run(*m), MISTAKES))
    crashed = [(n, out) for n, rc, out in results if rc not in (0, 1)]          # 1 = a pin failed; anything else = harness trouble
    assert not crashed, crashed[0]
    survived = [n for n, rc, _ in results if rc == 0]
    assert not survived, f"no pin notices: {survived}"
