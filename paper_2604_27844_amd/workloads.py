"""Seeded synthetic inputs standing in for the paper's communication tensors.

This module holds no part of the method: it only draws numbers and rounds them to the
wire dtype.  Both the HIP path and the CPU oracle are fed from here, so they see the
same bytes.  bf16 tensors are carried as numpy uint16 words, fp32 as uint32 words.

Workloads (sizes follow the five benchmark configurations; ``scale`` shrinks them for
parity tests while keeping their structure):
  c1  2^20 bf16 i.i.d. N(0, 0.02^2), 1 chunk
  c2  [4096 x 4096] bf16 N(0,1) activations, 8 outlier channels x50, 8 peer row-blocks
  c3  MoE dispatch buffer: 64 experts x Poisson(512) tokens x 7168 hidden, N(0, 0.5^2),
      one ragged chunk per expert
  c4  gradient bucket: 2^28 bf16 Student-t(nu=5) scaled to std 1e-4, 1% exact zeros, 64 chunks
  c5  FSDP parameter shard: 2^29 values, rows of 4096; every 20th row is a LayerNorm gain
      row N(1, 0.05^2), the rest N(0, 0.02^2); bf16 = rounded fp32 master; 64 chunks
  c5_fp32  the first 2^27 fp32 master values of c5, 64 chunks
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np

BF16, FP32 = 0, 1


@dataclass
class Workload:
    name: str
    data: np.ndarray            # uint16 (bf16 words) or uint32 (fp32 words), flat
    dtype: int                  # BF16 / FP32
    n_chunks: int
    chunk_elems: Optional[np.ndarray]   # uint64[n_chunks] for ragged chunks, None = equal split
    sigma: float                # nominal scale handed to the code-table builder
    note: str = ""

    @property
    def n_elems(self):
        return int(self.data.size)

    @property
    def nbytes(self):
        return int(self.data.nbytes)


def f32_to_bf16_words(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 words (no NaN in our inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def _normal_f32(rng, n, scale, block=1 << 24):
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, block):
        e = min(n, s + block)
        out[s:e] = rng.standard_normal(e - s, dtype=np.float32) * np.float32(scale)
    return out


def c1(scale=1.0, seed=0):
    n = max(1, int((1 << 20) * scale))
    rng = np.random.default_rng(seed)
    x = _normal_f32(rng, n, 0.02)
    return Workload("c1_gauss_1M", f32_to_bf16_words(x), BF16, 1, None, 0.02)


def c2(scale=1.0, seed=1):
    tokens = max(8, int(4096 * scale) // 8 * 8)
    hidden = 4096
    rng = np.random.default_rng(seed)
    x = _normal_f32(rng, tokens * hidden, 1.0).reshape(tokens, hidden)
    cols = rng.choice(hidden, size=8, replace=False)
    x[:, cols] *= np.float32(50.0)
    return Workload("c2_tp_allgather_act", f32_to_bf16_words(x.reshape(-1)), BF16, 8, None, 1.0,
                    note=f"outlier channels {sorted(int(c) for c in cols)}")


def c3(scale=1.0, seed=2):
    hidden = 7168
    rng = np.random.default_rng(seed)
    mean_tokens = max(1.0, 512 * scale)
    tokens = rng.poisson(mean_tokens, size=64).astype(np.uint64)
    chunk_elems = tokens * np.uint64(hidden)
    n = int(chunk_elems.sum())
    x = _normal_f32(rng, n, 0.5)
    return Workload("c3_moe_a2a_dispatch", f32_to_bf16_words(x), BF16, 64, chunk_elems, 0.5,
                    note=f"tokens/expert min {int(tokens.min())} max {int(tokens.max())}")


def c4(scale=1.0, seed=3):
    n = max(64, int((1 << 28) * scale) // 64 * 64)
    rng = np.random.default_rng(seed)
    nu = 5.0
    out = np.empty(n, dtype=np.float32)
    block = 1 << 24
    s_t = np.sqrt(nu / (nu - 2.0))  # std of Student-t(nu)
    for s in range(0, n, block):
        e = min(n, s + block)
        t = rng.standard_t(nu, size=e - s).astype(np.float32)
        t *= np.float32(1e-4 / s_t)
        t[rng.random(e - s, dtype=np.float32) < np.float32(0.01)] = 0.0
        out[s:e] = t
    return Workload("c4_grad_bucket", f32_to_bf16_words(out), BF16, 64, None, 1e-4)


def _c5_master(n, seed):
    row = 4096
    rng = np.random.default_rng(seed)
    x = _normal_f32(rng, n, 0.02)
    rows = (n + row - 1) // row
    for r in range(0, rows, 20):            # every 20th row holds LayerNorm gains (5 %)
        s, e = r * row, min(n, (r + 1) * row)
        x[s:e] = np.float32(1.0) + rng.standard_normal(e - s, dtype=np.float32) * np.float32(0.05)
    return x


def c5(scale=1.0, seed=4):
    n = max(64, int((1 << 29) * scale) // 64 * 64)
    x = _c5_master(n, seed)
    return Workload("c5_fsdp_param_shard_bf16", f32_to_bf16_words(x), BF16, 64, None, 0.02)


def c5_fp32(scale=1.0, seed=4):
    n = max(64, int((1 << 27) * scale) // 64 * 64)
    x = _c5_master(n, seed)     # same generator stream => the first values of the bf16 shard's master
    return Workload("c5_fsdp_master_fp32", np.ascontiguousarray(x).view(np.uint32).copy(), FP32, 64, None, 0.02)


ALL = {"c1": c1, "c2": c2, "c3": c3, "c4": c4, "c5": c5, "c5_fp32": c5_fp32}


def make(name, scale=1.0):
    return ALL[name](scale=scale)
