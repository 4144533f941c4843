"""Helpers for the GPU parity tests: move seeded inputs to the device, sample rows."""
import numpy as np


def device_tensor(t, name, dtype, dev="cuda:0"):
    """Device tensor of the rounded values in the input dict (bf16 from its bit patterns)."""
    import torch
    if dtype == "bf16":
        return torch.from_numpy(t[name + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(t[name], dtype=np.float32)).to(dev)


def device_qkv(t, dtype, dev="cuda:0", names=("Q", "K", "V")):
    return tuple(device_tensor(t, x, dtype, dev) for x in names)


def to_host(x):
    return x.float().cpu().numpy().astype(np.float64)


def sample_rows(nb, b, rng, extra_blocks=8):
    """Query rows covering both global blocks, blocks 1 and nb-2, and random interior blocks."""
    blocks = {0, nb - 1, 1, nb - 2} | {int(x) for x in rng.integers(2, max(3, nb - 2), size=extra_blocks)}
    rows = []
    for j in sorted(k for k in blocks if 0 <= k < nb):
        rows += [j * b, j * b + 31, j * b + 32, j * b + b - 1, j * b + int(rng.integers(0, b))]
    return sorted(set(rows))
