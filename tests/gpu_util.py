"""Helpers shared by the GPU parity tests (not a test module)."""
import numpy as np
import torch

import oracle
import paper_2508_17756_amd as sg
from synthetic import randn_tensor, torch_dtype

BF16_MAX_ABS, BF16_REL_L2 = 2e-2, 5e-3     # bf16 problems
F32_TOL = 1e-5                             # fp32 problems


def to_f64(t):
    """Exact widening of a stored bf16 / fp32 tensor to a numpy fp64 array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    max_abs = float(np.abs(got - ref).max()) if ref.size else 0.0
    rel_l2 = float(np.linalg.norm((got - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-300))
    return max_abs, rel_l2


def assert_close(got, ref, dtype, what=""):
    max_abs, rel_l2 = errors(got, ref)
    if dtype == "bf16":
        assert max_abs <= BF16_MAX_ABS and rel_l2 <= BF16_REL_L2, f"{what}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}"
    else:
        assert max_abs <= F32_TOL and rel_l2 <= F32_TOL, f"{what}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}"
    return max_abs, rel_l2


def canvas_qkv(g, device="cuda", seed_offset=0):
    return [randn_tensor(g.grid_shape, g.dtype, g.seed + 7 * s + seed_offset).to(device) for s in range(3)]


def gpu_tile_attention(g, q, k, v, tr, tc):
    out = torch.empty(g.tile_shape, dtype=torch_dtype(g.dtype), device=q.device)
    sg.sg_tile_attention(sg.make_problem(g), q, k, v, tr, tc, out)
    return out


def oracle_tile_attention_full(g, q, k, v, tr, tc):
    o = oracle.tile_attention(to_f64(q), to_f64(k), to_f64(v), g, tr, tc, g.scale)
    return np.stack([o[a] for a in range(g.heads)]).reshape(g.tile_shape)
