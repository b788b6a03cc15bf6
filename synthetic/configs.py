"""Geometry of the synthetic workloads (data only).

The canvas shapes stand in for the paper's workloads: a 720p tile is a
160 x 90 latent (80 x 45 tokens after 2 x 2 patchify), 2K is 160 x 90 tokens and
4K is 240 x 135 tokens, each with 21 latent frames (Section 8 of the paper, "Workloads"
gives the tile and canvas sizes); values are i.i.d. N(0, 1).
"""
from dataclasses import dataclass, replace
import math


@dataclass(frozen=True)
class TileGeometry:
    name: str
    T: int
    H: int
    W: int
    tile_h: int
    tile_w: int
    stride_h: int
    stride_w: int
    n_tile_rows: int
    n_tile_cols: int
    heads: int
    head_dim: int
    dtype: str            # "f32" | "bf16"
    seed: int
    steps: int = 1        # > 1: the cache gate runs over this many denoising steps
    threshold: float = -1.0

    @property
    def scale(self):
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def n_tiles(self):
        return self.n_tile_rows * self.n_tile_cols

    @property
    def tile_tokens(self):
        return self.T * self.tile_h * self.tile_w

    @property
    def grid_tokens(self):
        return self.T * self.H * self.W

    @property
    def grid_shape(self):
        return (self.heads, self.T, self.H, self.W, self.head_dim)

    @property
    def tile_shape(self):
        return (self.heads, self.T, self.tile_h, self.tile_w, self.head_dim)

    @property
    def attention_flops_per_tile(self):
        n = self.tile_tokens
        return 4.0 * n * n * self.head_dim * self.heads

    def single_tile(self):
        """The geometry whose canvas is exactly one tile of this one (packed tile)."""
        return replace(self, name=self.name + "/tile", H=self.tile_h, W=self.tile_w,
                       stride_h=self.tile_h, stride_w=self.tile_w,
                       n_tile_rows=1, n_tile_cols=1)


CONFIGS = {
    # 1: tiny fp32, 2x2 tiles of 3x10x10, stride 6 (overlap 4)
    "tiny_f32": TileGeometry("tiny_f32", 3, 16, 16, 10, 10, 6, 6, 2, 2, 2, 64, "f32", 1001),
    # 2: one 720p-sized tile, 75,600 tokens
    "tile720p_bf16": TileGeometry("tile720p_bf16", 21, 45, 80, 45, 80, 45, 80, 1, 1, 40, 128, "bf16", 1002),
    # 3: 2K canvas, 3x3 tiles of 21x48x80
    "canvas2k_bf16": TileGeometry("canvas2k_bf16", 21, 90, 160, 48, 80, 21, 40, 3, 3, 40, 128, "bf16", 1003),
    # 4: 4K canvas, 4x5 tiles of 21x45x80
    "canvas4k_bf16": TileGeometry("canvas4k_bf16", 21, 135, 240, 45, 80, 30, 40, 4, 5, 40, 128, "bf16", 1004),
    # 5: config 4 with the cache gate over 10 steps, threshold 0.05
    "canvas4k_gate_bf16": TileGeometry("canvas4k_gate_bf16", 21, 135, 240, 45, 80, 30, 40, 4, 5, 40, 128,
                                       "bf16", 1005, steps=10, threshold=0.05),
}


def config(name):
    return CONFIGS[name]


def scaled_down(name, T, tile_h, tile_w, heads, stride_h=None, stride_w=None, head_dim=None):
    """Same tile layout (tile counts, dtype, overlap structure) at a size the CPU
    oracle finishes in seconds.  Strides default to keeping the overlap fraction."""
    c = CONFIGS[name]
    sh = stride_h if stride_h is not None else max(1, round(tile_h * c.stride_h / c.tile_h))
    sw = stride_w if stride_w is not None else max(1, round(tile_w * c.stride_w / c.tile_w))
    return replace(c, name=c.name + "/small", T=T, tile_h=tile_h, tile_w=tile_w,
                   stride_h=sh, stride_w=sw,
                   H=sh * (c.n_tile_rows - 1) + tile_h, W=sw * (c.n_tile_cols - 1) + tile_w,
                   heads=heads, head_dim=head_dim or c.head_dim)
