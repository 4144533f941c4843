"""Seeded synthetic inputs for the BigBird block-sparse attention path.

This module is shared by the tests, the benchmark and the smoke check.  It
holds no arithmetic of the method itself: only random draws, rounding to the
storage type, and the table of workload shapes.  Both the CPU oracle and the
HIP library are fed the *same* rounded values produced here.

Workload shapes follow the BigBird-ITC base model (App. E.1, hyper-parameter
table for MLM pre-training): block length 64, 2 global / 3 window / 3 random
blocks, sequence length 4096, 12 heads of width 64.  The paper's corpora are not
available, so tensors are standard-normal stand-ins of those shapes.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: tensor shape, pattern parameters and seeds."""

    name: str
    B: int
    H: int
    n: int
    d: int = 64
    b: int = 64
    g: int = 2
    w: int = 3
    r: int = 3
    dtype: str = "bf16"          # storage type of Q, K, V, O, dO: "bf16" or "f32"
    pattern_seed: int = 0
    data_seed: int = 0
    length_seed: int | None = None   # None: no key-padding mask
    backward: bool = False
    scale: float = field(default=0.125)

    @property
    def nb(self) -> int:
        return self.n // self.b


# The five benchmark configurations (forward fp32 small, forward bf16
# BERT-base-shaped, forward with key padding, forward+backward, long sequence).
WORKLOADS = {
    "cfg1_fp32_small": Workload("cfg1_fp32_small", B=1, H=2, n=1024, dtype="f32",
                                pattern_seed=0, data_seed=100),
    "cfg2_bert_base": Workload("cfg2_bert_base", B=4, H=12, n=4096,
                               pattern_seed=1, data_seed=101),
    "cfg3_key_padding": Workload("cfg3_key_padding", B=8, H=12, n=4096,
                                 pattern_seed=2, data_seed=102, length_seed=202),
    "cfg4_fwd_bwd": Workload("cfg4_fwd_bwd", B=2, H=12, n=4096,
                             pattern_seed=3, data_seed=103, backward=True),
    "cfg5_long_seq": Workload("cfg5_long_seq", B=1, H=16, n=16384,
                              pattern_seed=4, data_seed=104),
}


def round_to_bf16(x: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Round float32 values to bfloat16, nearest-even.

    Returns (values as float32 that are exactly bf16-representable, uint16 bit
    patterns).  Inputs are finite normals here, so no NaN handling is needed.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    bits = rounded.astype(np.uint16)
    vals = (rounded.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return vals.reshape(x.shape), bits.reshape(x.shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(bits.shape)


def make_tensors(B: int, H: int, n: int, d: int, seed: int, dtype: str,
                 with_dO: bool = False) -> dict[str, np.ndarray]:
    """Draw Q, K, V (and dO) ~ N(0,1) in that order from one seeded stream.

    The values are rounded once to the storage type.  The dict holds float32
    arrays `Q, K, V[, dO]` with the rounded values and, for bf16, the uint16 bit
    patterns under `Q_bits` etc.
    """
    rng = np.random.default_rng(seed)
    out: dict[str, np.ndarray] = {}
    names = ["Q", "K", "V"] + (["dO"] if with_dO else [])
    for name in names:
        x = rng.standard_normal((B, H, n, d), dtype=np.float32)
        if dtype == "bf16":
            vals, bits = round_to_bf16(x)
            out[name] = vals
            out[name + "_bits"] = bits
        elif dtype == "f32":
            out[name] = x
        else:
            raise ValueError(f"unknown dtype {dtype!r}")
    return out


def make_valid_lengths(B: int, n: int, b: int, seed: int, lo: int = 1024) -> np.ndarray:
    """Per-sequence valid lengths, uniform over the multiples of b in [lo, n]."""
    rng = np.random.default_rng(seed)
    lo_blk = max(1, (min(lo, n) + b - 1) // b)
    return (rng.integers(lo_blk, n // b + 1, size=B) * b).astype(np.int64)


def lengths_to_key_mask(lengths: np.ndarray, n: int) -> np.ndarray:
    """uint8 [B, n] with 1 for valid keys (position < length) and 0 for padding."""
    pos = np.arange(n)[None, :]
    return (pos < np.asarray(lengths)[:, None]).astype(np.uint8)


def workload_tensors(wl: Workload) -> dict[str, np.ndarray]:
    """All data inputs of a workload (tensors, optional key-padding mask)."""
    t = make_tensors(wl.B, wl.H, wl.n, wl.d, wl.data_seed, wl.dtype, with_dO=wl.backward)
    if wl.length_seed is not None:
        lengths = make_valid_lengths(wl.B, wl.n, wl.b, wl.length_seed)
        t["lengths"] = lengths
        t["key_mask"] = lengths_to_key_mask(lengths, wl.n)
    return t
