"""A tiled step is a fixed sequence of launches with no host readback, so it can be captured in a HIP
graph and replayed: every replay must give what the same eager call gives on the same buffers."""
import numpy as np
import pytest
import torch

import paper_2508_17756_amd as sg
from synthetic import TileGeometry, randn_tensor, perturb_

pytestmark = pytest.mark.gpu


def _geom(name, T, H, W, th, tw, sh, sw, heads, d, dtype, seed):
    nr = (H - th) // sh + 1 if th < H else 1
    nc = (W - tw) // sw + 1 if tw < W else 1
    return TileGeometry(name, T, H, W, th, tw, sh, sw, nr, nc, heads, d, dtype, seed)


def test_cached_step_replays_from_a_graph():
    g = _geom("graph", 2, 14, 20, 8, 12, 6, 8, 2, 128, "bf16", 71)        # 2 x 2 tiles, N = 192
    n = g.n_tiles
    p = sg.make_problem(g)

    def state():
        return dict(cache_x=[torch.zeros((3,) + g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)],
                    cache_out=[torch.zeros(g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)],
                    has_cache=torch.zeros(n, dtype=torch.uint8, device="cuda"),
                    scores=torch.zeros(n, dtype=torch.float32, device="cuda"),
                    rec=torch.zeros(n, dtype=torch.uint8, device="cuda"),
                    ws=torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda"),
                    canvas=torch.zeros(g.grid_shape, dtype=torch.bfloat16, device="cuda"))

    tile_x = [randn_tensor((3,) + g.tile_shape, "bf16", 900 + i).cuda() for i in range(n)]

    def step(st):
        sg.sg_denoise_step_tiled(p, st["canvas"], st["cache_out"], tile_x=tile_x, cache_x=st["cache_x"],
                                 has_cache=st["has_cache"], threshold=0.05, scores=st["scores"], recompute=st["rec"],
                                 workspace=st["ws"])

    eager, graphed = state(), state()
    step(eager)                                          # first eager call also does the one-time kernel set-up
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step(graphed)
    torch.cuda.synchronize()
    eps = [None, [0.01, 0.2, 0.01, 0.2], [0.2, 0.01, 0.01, 0.01], [0.01, 0.01, 0.01, 0.01]]
    for k in range(4):
        if k:                                            # eager work between the replays: the inputs drift
            for i in range(n):
                perturb_(tile_x[i], eps[k][i], 9000 + 10 * k + i)
            step(eager)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(graphed["rec"], eager["rec"]), k
        assert torch.equal(graphed["scores"], eager["scores"]), k
        assert torch.equal(graphed["canvas"], eager["canvas"]), k
        assert torch.equal(graphed["has_cache"], eager["has_cache"])
        for a, b in zip(graphed["cache_out"] + graphed["cache_x"], eager["cache_out"] + eager["cache_x"]):
            assert torch.equal(a, b)
        if k:
            assert graphed["rec"].cpu().tolist() == [int(e == 0.2) for e in eps[k]]


@pytest.mark.parametrize("shift", [(0, 0), (3, 5)])
def test_canvas_step_through_the_register_staged_kernel_replays_from_a_graph(shift):
    """head_dim 64 read in place from a canvas takes the register-staged attention kernel (and, with a shift, its
    wrapping loader): the canvas step captured once, replayed three times with eager work on the inputs in between,
    must equal the eager step every time.  The first eager call does the kernel's one-time set-up outside of capture."""
    g = _geom("graph64", 2, 14, 20, 8, 12, 6, 8, 2, 64, "bf16", 73)       # 2 x 2 overlapping tiles, N = 192
    p = sg.make_problem(g, shift=shift)
    qkv = [randn_tensor(g.grid_shape, "bf16", 950 + s).cuda() for s in range(3)]

    def buffers():
        return ([torch.zeros(g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(g.n_tiles)],
                torch.zeros(g.grid_shape, dtype=torch.bfloat16, device="cuda"))

    (t_eager, c_eager), (t_graph, c_graph) = buffers(), buffers()
    sg.sg_denoise_step_tiled(p, c_eager, t_eager, q=qkv[0], k=qkv[1], v=qkv[2])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        sg.sg_denoise_step_tiled(p, c_graph, t_graph, q=qkv[0], k=qkv[1], v=qkv[2])
    torch.cuda.synchronize()
    for k in range(3):
        if k:
            for s in range(3):
                perturb_(qkv[s], 0.3, 9500 + 10 * k + s)
            sg.sg_denoise_step_tiled(p, c_eager, t_eager, q=qkv[0], k=qkv[1], v=qkv[2])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(c_graph, c_eager), k
        for a, b in zip(t_graph, t_eager):
            assert torch.equal(a, b), k
        assert float(c_graph.float().abs().max()) > 0
