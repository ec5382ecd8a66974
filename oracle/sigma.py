"""Oracle for the device-side sigma estimate and table choice (paper section 4.1, last sentence:
sigma of a tensor is taken with torch.std, i.e. the unbiased sample standard deviation).
TEST INFRASTRUCTURE ONLY.  numpy in fp64."""
import numpy as np

from . import zipccl_oracle as zo


def words_to_f64(words, dtype):
    w = np.ascontiguousarray(words)
    if dtype == zo.BF16:
        return (w.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return w.view(np.float32).astype(np.float64)


def estimate_sigma(words, dtype):
    """sqrt(sum((x - mean)^2) / (N - 1)) in fp64; NaN when N < 2 or any value is not finite."""
    x = words_to_f64(words, dtype)
    if x.size < 2:
        return float("nan")
    with np.errstate(all="ignore"):
        m = x.sum() / x.size
        return float(np.sqrt(((x - m) ** 2).sum() / (x.size - 1)))


def estimate_table(words, dtype):
    """Table for the estimated sigma (Eq.5 / Eq.2); a sigma that is not a positive finite number
    (constant tensor, NaN/Inf inside, fewer than two values) falls back to the lowest window."""
    s = estimate_sigma(words, dtype)
    if not (s > 0.0) or not np.isfinite(s):
        return np.array([0, 1, 2, 3, 4, 5, 6, 7], dtype=np.uint8), s
    return zo.build_table(s), s
