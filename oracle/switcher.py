"""Oracle for the adaptive Reduce-Scatter switcher (paper section 5.2, Eq.6 and Eq.7).
TEST INFRASTRUCTURE ONLY.  Plain Python floats (fp64).

  T_RS(d)  = alpha_RS  + beta_RS  * d                      (Eq.6)
  T_A2A(d) = alpha_A2A + beta_A2A * e * s * d              (Eq.7)

d = data size, alpha = start-up latency, beta = time per byte, e = compression factor of the zipped
All-to-All (compressed bytes / original bytes, so e < 1 when compression helps), s = precision scale
factor (e.g. 0.5 when the native Reduce-Scatter runs in a format twice as wide as the zipped path's).
The zipped Reduce-Scatter is chosen when T_A2A(d) < T_RS(d).
"""


def t_rs(alpha_rs, beta_rs, d):
    return alpha_rs + beta_rs * d


def t_a2a(alpha_a2a, beta_a2a, e, s, d):
    return alpha_a2a + beta_a2a * e * s * d


def prefers_zipped(alpha_rs, beta_rs, alpha_a2a, beta_a2a, e, s, d):
    return t_a2a(alpha_a2a, beta_a2a, e, s, d) < t_rs(alpha_rs, beta_rs, d)


def fit_linear(ds, ts):
    """Ordinary least squares for t = alpha + beta * d (the profiling step at initialisation)."""
    k = len(ds)
    md, mt = sum(ds) / k, sum(ts) / k
    sxx = sum((d - md) ** 2 for d in ds)
    sxy = sum((d - md) * (t - mt) for d, t in zip(ds, ts))
    beta = sxy / sxx
    return mt - beta * md, beta
