"""Seeded random tensors for the synthetic workloads (no method arithmetic).

Tensors are drawn with torch's seeded generators, on the CPU for small cases
and on the device for the full-size ones; the stored values are the ground
truth both sides read.
"""
import numpy as np

# torch is imported where it is used: the geometry-only users of this package do not pay for it


def torch_dtype(name):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def randn_tensor(shape, dtype, seed, device="cpu"):
    """i.i.d. N(0, 1) values of the given dtype ("f32" | "bf16"), seeded."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    return torch.randn(tuple(shape), dtype=torch_dtype(dtype), device=device, generator=gen)


def eps_table(seed, steps, n_tiles, choices=(0.01, 0.1)):
    """eps[k, tile], k = 0..steps-1, drawn uniformly from `choices` on the host.
    Row 0 is unused (step 0 takes the unperturbed inputs)."""
    rng = np.random.default_rng(int(seed))
    idx = rng.integers(0, len(choices), size=(steps, n_tiles))
    return np.asarray(choices, dtype=np.float64)[idx]


def perturb_(x, eps, seed, chunk=1 << 26):
    """In place x <- round_to_dtype(float32(x) + eps * n), n ~ N(0, 1) in fp32.
    The next denoising step's tile input of the gated workload."""
    import torch
    gen = torch.Generator(device=x.device)
    gen.manual_seed(int(seed))
    flat = x.view(-1)
    for s in range(0, flat.numel(), chunk):
        part = flat[s:s + chunk]
        n = torch.randn(part.shape, dtype=torch.float32, device=x.device, generator=gen)
        part.copy_((part.float() + float(eps) * n).to(x.dtype))
    return x


def sample_rows(seed, n_tokens, count, block=256):
    """Seeded query-row sample that always holds row 0, the last row and rows of
    the last (ragged) block of `block` rows."""
    rng = np.random.default_rng(int(seed))
    tail0 = ((n_tokens - 1) // block) * block
    forced = {0, n_tokens - 1, tail0, min(n_tokens - 1, tail0 + 1)}
    rows = set(int(r) for r in rng.integers(0, n_tokens, size=max(0, count - len(forced))))
    return np.array(sorted(rows | forced), dtype=np.int64)
