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


# Phi^-1(3/4): the median of |w| for w ~ N(0, sigma^2) is sigma times this
PHI_INV_3_4 = 0.6744897501960817


def robust_sigma(words, dtype):
    """A sigma for Eq.5 that a few large entries cannot move (the tensors the paper feeds to section 4.1 are
    zero-mean Gaussians; activations with outlier channels or a parameter shard that also holds LayerNorm
    gains are not, and one part in twenty of such entries multiplies the sample standard deviation by ten).

    For w ~ N(0, sigma^2) half of the |w| lie below sigma * Phi^-1(3/4), so
        sigma = median(|w|) / Phi^-1(3/4).
    The median is taken over the magnitudes of the high 16-bit words (the bf16 value itself; an fp32 value
    truncated to its bf16 prefix, which is the part the exponent code works on), as integers: rank
    floor((K - 1) / 2) of the K magnitudes that are neither zero nor Inf/NaN (a zero is not a sample of the
    Gaussian and is a zero-point under every window).  That makes the estimate a count, exact and the same in
    any order of summation.  K = 0 gives NaN."""
    w = np.ascontiguousarray(words).reshape(-1)
    hi = w if dtype == zo.BF16 else (w >> np.uint32(16))
    mag = (hi & 0x7FFF).astype(np.uint16)
    mag = mag[(mag != 0) & (mag < 0x7F80)]
    if mag.size == 0:
        return float("nan")
    med = np.sort(mag)[(mag.size - 1) // 2]
    value = (np.array([med], dtype=np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)[0]
    return float(value / PHI_INV_3_4)


def robust_table(words, dtype):
    """Table for robust_sigma (Eq.5 / Eq.2); no usable magnitude at all falls back to the lowest window."""
    s = robust_sigma(words, dtype)
    if not (s > 0.0) or not np.isfinite(s):
        return np.array([0, 1, 2, 3, 4, 5, 6, 7], dtype=np.uint8), s
    return zo.build_table(s), s


def robust_chunk_tables(words, dtype, n_chunks, chunk_elems=None):
    """One table per peer chunk: robust_table of every chunk of the split on its own (section 4.1 takes sigma per
    layer; the chunks of a collective call may hold different layers or experts).  Returns (uint8[n_chunks, 8],
    float64[n_chunks])."""
    w = np.ascontiguousarray(words).reshape(-1)
    if chunk_elems is None:
        assert w.size % n_chunks == 0
        chunk_elems = [w.size // n_chunks] * n_chunks
    decs, sigmas, start = [], [], 0
    for n in chunk_elems:
        d, s = robust_table(w[start:start + int(n)], dtype)
        decs.append(d)
        sigmas.append(s)
        start += int(n)
    assert start == w.size
    return np.array(decs, dtype=np.uint8).reshape(n_chunks, 8), np.array(sigmas, dtype=np.float64)


# --- the same estimate from a sample of the tensor -----------------------------------------------------------
#
# The robust estimate reads the whole tensor to fix one integer (the window base).  A sample of one part in S
# fixes the same integer unless sigma sits within a few parts in ten thousand of a window boundary, at 1/S of
# the traffic.  The sample is taken in whole groups of 512 consecutive values (the codec's group: contiguous
# kilobytes, so it reads at full memory efficiency), stratified: the groups of a chunk are cut into blocks of S
# consecutive groups and one group is taken from every block, at a position inside the block that varies from
# block to block in a fixed pseudo-random way.  A fixed position would alias with the tensor's own periods (a
# row of 4096 values is 8 groups: a stride of 16 groups would only ever see columns 0..511); the varying one
# visits all positions equally often.  Position in block k:
#     ((k * 2654435761) mod 2^32) >> 16) mod S           (Knuth's multiplicative hash, upper half)
# A block's group that lies past the end of the chunk (last block only) contributes nothing; a last group that
# is cut short contributes the values it has.  S = 1 takes everything.

SAMPLE_GROUP = 512
SAMPLE_MULT = 2654435761


def sampled_groups(n, stride):
    """Indices of the groups of 512 values that the sample of a chunk of n values takes, in increasing order."""
    stride = int(stride)
    assert stride >= 1
    ng = -(-int(n) // SAMPLE_GROUP)
    out = []
    for k in range(-(-ng // stride)):
        g = k * stride + (((k * SAMPLE_MULT) % (1 << 32)) >> 16) % stride
        if g < ng:
            out.append(g)
    return np.array(out, dtype=np.int64)


def sample_of(words, stride):
    """The sampled values themselves, in order."""
    w = np.ascontiguousarray(words).reshape(-1)
    g = sampled_groups(w.size, stride)
    if g.size == 0:
        return w[:0]
    idx = (g[:, None] * SAMPLE_GROUP + np.arange(SAMPLE_GROUP, dtype=np.int64)[None, :]).reshape(-1)
    return w[idx[idx < w.size]]


def robust_sigma_sampled(words, dtype, stride):
    return robust_sigma(sample_of(words, stride), dtype)


def robust_chunk_tables_sampled(words, dtype, n_chunks, chunk_elems=None, stride=1):
    """robust_table of every chunk's own sample (group numbers count from the chunk's first value)."""
    w = np.ascontiguousarray(words).reshape(-1)
    if chunk_elems is None:
        assert w.size % n_chunks == 0
        chunk_elems = [w.size // n_chunks] * n_chunks
    decs, sigmas, start = [], [], 0
    for n in chunk_elems:
        d, s = robust_table(sample_of(w[start:start + int(n)], stride), dtype)
        decs.append(d)
        sigmas.append(s)
        start += int(n)
    assert start == w.size
    return np.array(decs, dtype=np.uint8).reshape(n_chunks, 8), np.array(sigmas, dtype=np.float64)
