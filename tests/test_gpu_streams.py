"""The library keeps no state between calls (each caller brings its own workspace), so calls on different
streams, and from different host threads, may overlap freely: whatever runs concurrently must give, bit for
bit, what the same calls give one after the other.  Every reduction adds in a fixed order, so the comparison
is exact."""
import threading

import pytest
import torch

import paper_2508_17756_amd as sg
from synthetic import TileGeometry, randn_tensor, perturb_

pytestmark = pytest.mark.gpu


def _geom(name, T, H, W, th, tw, sh, sw, heads, d, dtype, seed):
    nr = (H - th) // sh + 1 if th < H else 1
    nc = (W - tw) // sw + 1 if tw < W else 1
    return TileGeometry(name, T, H, W, th, tw, sh, sw, nr, nc, heads, d, dtype, seed)


class _CachedRun:
    """Buffers of one caller of the cached step on a 2 x 2 tiling, and the steps it takes."""

    def __init__(self, seed):
        self.g = g = _geom("streams", 2, 22, 28, 14, 16, 8, 12, 4, 128, "bf16", seed)     # N = 448 per tile
        n = g.n_tiles
        self.p = sg.make_problem(g)
        self.tile_x = [randn_tensor((3,) + g.tile_shape, "bf16", seed + 10 + i).cuda() for i in range(n)]
        self.cache_x = [torch.zeros((3,) + g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
        self.cache_out = [torch.zeros(g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
        self.has_cache = torch.zeros(n, dtype=torch.uint8, device="cuda")
        self.scores = torch.zeros(n, dtype=torch.float32, device="cuda")
        self.rec = torch.zeros(n, dtype=torch.uint8, device="cuda")
        self.ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        self.canvas = torch.zeros(g.grid_shape, dtype=torch.bfloat16, device="cuda")
        self.std = torch.zeros(n, dtype=torch.float32, device="cuda")
        self.seed = seed
        self.history = []

    def step(self, k):
        eps = [0.2, 0.01, 0.2, 0.01]
        if k:
            for i, x in enumerate(self.tile_x):
                perturb_(x, eps[(i + k) % 4], self.seed + 100 * k + i)
        sg.sg_denoise_step_tiled(self.p, self.canvas, self.cache_out, tile_x=self.tile_x, cache_x=self.cache_x,
                                 has_cache=self.has_cache, threshold=0.05, scores=self.scores, recompute=self.rec,
                                 workspace=self.ws)
        sg.sg_tile_std(self.cache_out, self.std, self.ws)
        self.history.append((self.rec.clone(), self.scores.clone(), self.canvas.clone(), self.std.clone()))

    def steps(self, count):
        for k in range(count):
            self.step(k)

    def same_as(self, other):
        assert len(self.history) == len(other.history)
        for k, (a, b) in enumerate(zip(self.history, other.history)):
            for x, y in zip(a, b):
                assert torch.equal(x, y), k
        for x, y in zip(self.cache_out + self.cache_x, other.cache_out + other.cache_x):
            assert torch.equal(x, y)


def test_calls_on_two_streams_overlap_without_touching_each_other():
    serial = [_CachedRun(501), _CachedRun(777)]
    for r in serial:
        r.steps(4)
    torch.cuda.synchronize()
    overlapped = [_CachedRun(501), _CachedRun(777)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    # the two callers' steps are enqueued alternately, each on its own stream, with no synchronisation between them
    for k in range(4):
        for r, s in zip(overlapped, streams):
            with torch.cuda.stream(s):
                r.step(k)
    torch.cuda.synchronize()
    for a, b in zip(overlapped, serial):
        a.same_as(b)
    assert any(int(h[0].sum()) not in (0, 4) for h in serial[0].history[1:])     # the gate did split the tiles


def test_host_threads_call_the_library_at_the_same_time():
    serial = [_CachedRun(1501), _CachedRun(1777), _CachedRun(1999)]
    for r in serial:
        r.steps(3)
    torch.cuda.synchronize()
    threaded = [_CachedRun(1501), _CachedRun(1777), _CachedRun(1999)]
    torch.cuda.synchronize()
    failures = []

    def work(run):
        try:
            torch.cuda.set_device(0)
            with torch.cuda.stream(torch.cuda.Stream()):
                run.steps(3)
                torch.cuda.current_stream().synchronize()
        except Exception as exc:       # reported by the main thread
            failures.append(exc)

    threads = [threading.Thread(target=work, args=(r,)) for r in threaded]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not any(t.is_alive() for t in threads)
    assert not failures, failures
    torch.cuda.synchronize()
    for a, b in zip(threaded, serial):
        a.same_as(b)
