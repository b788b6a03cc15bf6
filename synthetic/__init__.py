"""Seeded synthetic workloads: shapes of the five benchmark configs and the
random tensors that fill them.  Holds no arithmetic of the method itself, so
both the HIP path's tests and the CPU oracle's tests may draw inputs from here.
"""
from .configs import TileGeometry, CONFIGS, config, scaled_down  # noqa: F401
from .inputs import randn_tensor, eps_table, perturb_, sample_rows, torch_dtype  # noqa: F401
