"""GPU parity of tile shifting (sg_tile_slice, shifted sg_tile_blend) and of the fused scheduler update
(sg_tile_blend_update) against the oracle."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2508_17756_amd as sg
from synthetic import CONFIGS, TileGeometry, randn_tensor, torch_dtype
from gpu_util import to_f64, assert_close

pytestmark = pytest.mark.gpu


def _geom(name, T, H, W, th, tw, sh, sw, heads, d, dtype, seed):
    nr = (H - th) // sh + 1 if th < H else 1
    nc = (W - tw) // sw + 1 if tw < W else 1
    return TileGeometry(name, T, H, W, th, tw, sh, sw, nr, nc, heads, d, dtype, seed)


GEOMS = {
    "paper_2x3": lambda dt, d: _geom("p", 2, 6, 12, 3, 4, 3, 4, 2, d, dt, 11),        # non-overlapping, as in the paper
    "overlap_2x2": lambda dt, d: replace(CONFIGS["tiny_f32"], dtype=dt, head_dim=d),
    "triple_3x2": lambda dt, d: _geom("t", 2, 9, 7, 5, 4, 2, 3, 3, d, dt, 12),
    "cover_5x4": lambda dt, d: _geom("c", 1, 15, 13, 9, 7, 2, 2, 3, d, dt, 13),
}


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shift", [(0, 0), (1, 0), (0, 3), (2, 5), (5, 11)])
@pytest.mark.parametrize("token_major", [False, True])
def test_slice_is_the_wrapped_window(dtype, shift, token_major):
    d = 64 if dtype == "f32" else 128
    g = GEOMS["paper_2x3"](dtype, d)
    canv = [randn_tensor(g.grid_shape, dtype, 20 + s).cuda() for s in range(3)]
    p = sg.make_problem(g, token_major=token_major, shift=shift)
    dev = [t.permute(1, 2, 3, 0, 4).contiguous() for t in canv] if token_major else canv
    for n_src in (1, 3):
        for tr, tc in ((0, 0), (1, 2), (1, 0)):
            dst = torch.full((n_src,) + g.tile_shape, float("nan"), dtype=torch_dtype(dtype), device="cuda")
            sg.sg_tile_slice(p, dev[:n_src], tr, tc, dst)
            for s in range(n_src):
                ref = oracle.slice_tile_shifted(to_f64(canv[s]), g, tr, tc, *shift)
                assert np.array_equal(to_f64(dst[s]), ref), (n_src, tr, tc, s)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", list(GEOMS))
@pytest.mark.parametrize("shift", [(0, 0), (1, 2), (4, 6)])
def test_shifted_blend_and_fused_update(dtype, shape, shift):
    d = 64 if dtype == "f32" else 128
    g = GEOMS[shape](dtype, d)
    tiles = [randn_tensor(g.tile_shape, dtype, 600 + i).cuda() for i in range(g.n_tiles)]
    p = sg.make_problem(g, shift=shift)
    out = torch.full(g.grid_shape, float("nan"), dtype=torch_dtype(dtype), device="cuda")
    sg.sg_tile_blend(p, tiles, out)
    ref = oracle.blend_shifted([to_f64(t) for t in tiles], g, *shift)
    assert_close(to_f64(out), ref, dtype, f"{shape} {shift}")
    # scheduler update fused behind the blend: out of place, then in place
    lat = randn_tensor(g.grid_shape, dtype, 77).cuda()
    ref_u = oracle.fuse_and_denoise([to_f64(t) for t in tiles], g, to_f64(lat), 0.875, -0.05, *shift)
    new = torch.full(g.grid_shape, float("nan"), dtype=torch_dtype(dtype), device="cuda")
    sg.sg_tile_blend_update(p, tiles, lat, 0.875, -0.05, new)
    assert_close(to_f64(new), ref_u, dtype, f"update {shape} {shift}")
    inplace = lat.clone()
    sg.sg_tile_blend_update(p, tiles, inplace, 0.875, -0.05, inplace)
    assert torch.equal(inplace, new)
    # c_latent = 1, c_noise = 0 leaves the latent bit for bit; c_latent = 0, c_noise = 1 is the plain blend
    keep = lat.clone()
    sg.sg_tile_blend_update(p, tiles, keep, 1.0, 0.0, keep)
    assert torch.equal(keep, lat)
    sg.sg_tile_blend_update(p, tiles, lat, 0.0, 1.0, new)
    assert torch.equal(new, out)


@pytest.mark.parametrize("shift", [(0, 0), (2, 7), (5, 11)])
def test_slice_then_blend_is_the_identity_for_non_overlapping_tiles(shift):
    g = GEOMS["paper_2x3"]("bf16", 128)
    c = randn_tensor(g.grid_shape, "bf16", 5).cuda()
    p = sg.make_problem(g, shift=shift)
    tiles = []
    for tr in range(g.n_tile_rows):
        for tc in range(g.n_tile_cols):
            t = torch.empty((1,) + g.tile_shape, dtype=torch.bfloat16, device="cuda")
            sg.sg_tile_slice(p, [c], tr, tc, t)
            tiles.append(t[0])
    out = torch.empty_like(c)
    sg.sg_tile_blend(p, tiles, out)
    assert torch.equal(out, c)


def test_shifted_step_bf16():
    """One stage-2 step under a shifted partition: gather every tile's Q, K, V, attend the packed tiles,
    fuse at the shifted positions and apply the scheduler update — against the oracle end to end."""
    g = _geom("sh", 2, 16, 24, 8, 12, 8, 12, 2, 128, "bf16", 31)         # 2 x 2 non-overlapping tiles, N = 192
    shift = (3, 7)
    p = sg.make_problem(g, shift=shift)
    qkv = [randn_tensor(g.grid_shape, "bf16", g.seed + 7 * s).cuda() for s in range(3)]
    n = g.n_tiles
    tile_x = []
    for tr in range(g.n_tile_rows):
        for tc in range(g.n_tile_cols):
            t = torch.empty((3,) + g.tile_shape, dtype=torch.bfloat16, device="cuda")
            sg.sg_tile_slice(p, qkv, tr, tc, t)
            tile_x.append(t)
    cache_x = [torch.zeros_like(t) for t in tile_x]
    cache_out = [torch.zeros(g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    has_cache = torch.zeros(n, dtype=torch.uint8, device="cuda")
    scores = torch.empty(n, dtype=torch.float32, device="cuda")
    rec = torch.empty(n, dtype=torch.uint8, device="cuda")
    ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    noise = torch.empty(g.grid_shape, dtype=torch.bfloat16, device="cuda")
    sg.sg_denoise_step_tiled(p, noise, cache_out, tile_x=tile_x, cache_x=cache_x, has_cache=has_cache, threshold=0.05,
                             scores=scores, recompute=rec, workspace=ws)
    latent = randn_tensor(g.grid_shape, "bf16", 99).cuda()
    new_latent = torch.empty_like(latent)
    sg.sg_tile_blend_update(p, cache_out, latent, 1.0, -0.25, new_latent)
    torch.cuda.synchronize()
    outs = []
    for tr in range(g.n_tile_rows):
        for tc in range(g.n_tile_cols):
            Q, K, V = (oracle.slice_tile_shifted(to_f64(t), g, tr, tc, *shift) for t in qkv)
            o = np.stack([oracle.attention(Q[a].reshape(-1, 128), K[a].reshape(-1, 128), V[a].reshape(-1, 128), g.scale)
                          for a in range(g.heads)]).reshape(g.tile_shape)
            outs.append(o)
    assert_close(to_f64(noise), oracle.blend_shifted(outs, g, *shift), "bf16", "fused noise")
    assert_close(to_f64(new_latent), oracle.fuse_and_denoise(outs, g, to_f64(latent), 1.0, -0.25, *shift), "bf16", "latent")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shift", [(0, 0), (3, 5)])
@pytest.mark.parametrize("room", [1, 3, 4])
def test_canvas_step_gathers_tiles_when_given_a_workspace(dtype, shift, room):
    """Canvas mode with room for `room` packed tiles in the workspace (the 4 tiles go through in groups of 1, of 3 + 1,
    or all at once): same numbers as reading in place (bit for bit, the arithmetic is the same) and, under a shifted
    partition, the oracle's shifted step."""
    d = 64 if dtype == "f32" else 128
    g = _geom("cw", 2, 14, 20, 8, 12, 6, 8, 2, d, dtype, 41)              # 2 x 2 overlapping tiles
    td = torch_dtype(dtype)
    qkv = [randn_tensor(g.grid_shape, dtype, g.seed + 7 * s).cuda() for s in range(3)]
    E = int(np.prod(g.tile_shape))
    ws = torch.empty(room * (3 * E * (2 if dtype == "bf16" else 4) + 256), dtype=torch.uint8, device="cuda")
    p = sg.make_problem(g, shift=shift)
    tiles = [torch.empty(g.tile_shape, dtype=td, device="cuda") for _ in range(g.n_tiles)]
    canvas = torch.empty(g.grid_shape, dtype=td, device="cuda")
    sg.sg_denoise_step_tiled(p, canvas, tiles, q=qkv[0], k=qkv[1], v=qkv[2], workspace=ws)
    torch.cuda.synchronize()
    outs = []
    for tr in range(g.n_tile_rows):
        for tc in range(g.n_tile_cols):
            Q, K, V = (oracle.slice_tile_shifted(to_f64(t), g, tr, tc, *shift) for t in qkv)
            outs.append(np.stack([oracle.attention(Q[a].reshape(-1, d), K[a].reshape(-1, d), V[a].reshape(-1, d), g.scale)
                                  for a in range(g.heads)]).reshape(g.tile_shape))
    assert_close(to_f64(canvas), oracle.blend_shifted(outs, g, *shift), dtype, "canvas")
    if shift == (0, 0):
        tiles2 = [torch.empty(g.tile_shape, dtype=td, device="cuda") for _ in range(g.n_tiles)]
        canvas2 = torch.empty(g.grid_shape, dtype=td, device="cuda")
        sg.sg_denoise_step_tiled(p, canvas2, tiles2, q=qkv[0], k=qkv[1], v=qkv[2])
        assert torch.equal(canvas2, canvas) and all(torch.equal(a, b) for a, b in zip(tiles, tiles2))
    else:                                                                  # wrapped windows read in place: same numbers
        tiles2 = [torch.full(g.tile_shape, float("nan"), dtype=td, device="cuda") for _ in range(g.n_tiles)]
        canvas2 = torch.full(g.grid_shape, float("nan"), dtype=td, device="cuda")
        sg.sg_denoise_step_tiled(p, canvas2, tiles2, q=qkv[0], k=qkv[1], v=qkv[2])
        assert torch.equal(canvas2, canvas) and all(torch.equal(a, b) for a, b in zip(tiles, tiles2))


WRAP_CASES = [
    # name, T, H, W, th, tw, sh, sw, heads, d, dtype, token_major, shift
    ("bf16_w16_rows_and_cols", 3, 20, 40, 12, 16, 8, 8, 2, 128, "bf16", False, (5, 9)),      # N = 576; tile width 16
    ("bf16_w13_odd", 2, 17, 21, 9, 13, 8, 8, 2, 128, "bf16", False, (16, 20)),               # odd width: per-lane walk either way
    ("bf16_paper_nonoverlap", 2, 12, 24, 6, 8, 6, 8, 2, 128, "bf16", False, (1, 1)),         # the paper's partition, shift tile/…
    ("bf16_token_major", 2, 12, 24, 6, 8, 6, 8, 3, 128, "bf16", True, (7, 3)),
    ("bf16_d64", 2, 12, 24, 6, 8, 6, 8, 2, 64, "bf16", False, (2, 21)),                      # head_dim 64 in place: register-staged kernel
    ("f32_d64", 3, 16, 16, 10, 10, 6, 6, 2, 64, "f32", False, (3, 11)),
    ("f32_d128_token_major", 2, 9, 11, 5, 6, 4, 5, 2, 128, "f32", True, (8, 10)),
]


@pytest.mark.parametrize("case", WRAP_CASES, ids=[c[0] for c in WRAP_CASES])
def test_attention_reads_a_wrapped_window_in_place(case):
    """sg_tile_attention under a shifted partition (Algorithm 1 "Shift" + "SliceTile"): every tile, whether its
    window wraps around a canvas edge or not, against the oracle's attention of the oracle's shifted slice."""
    name, T, H, W, th, tw, sh, sw, heads, d, dtype, token_major, shift = case
    g = _geom(name, T, H, W, th, tw, sh, sw, heads, d, dtype, 71)
    td = torch_dtype(dtype)
    qkv = [randn_tensor(g.grid_shape, dtype, g.seed + 7 * s).cuda() for s in range(3)]
    dev = [t.permute(1, 2, 3, 0, 4).contiguous() for t in qkv] if token_major else qkv
    p = sg.make_problem(g, token_major=token_major, shift=shift)
    wrapped = 0
    for tr in range(g.n_tile_rows):
        for tc in range(g.n_tile_cols):
            out = torch.full(g.tile_shape, float("nan"), dtype=td, device="cuda")
            sg.sg_tile_attention(p, dev[0], dev[1], dev[2], tr, tc, out)
            Q, K, V = (oracle.slice_tile_shifted(to_f64(t), g, tr, tc, *shift) for t in qkv)
            ref = np.stack([oracle.attention(Q[a].reshape(-1, d), K[a].reshape(-1, d), V[a].reshape(-1, d), g.scale)
                            for a in range(g.heads)]).reshape(g.tile_shape)
            assert_close(to_f64(out), ref, dtype, f"{name} tile {tr},{tc}")
            y, x = (tr * sh + shift[0]) % H, (tc * sw + shift[1]) % W
            wrapped += int(y + th > H or x + tw > W)
    assert 0 < wrapped < g.n_tiles or g.n_tiles == 1      # the case exercises both kinds of window


def _random_tilings(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        T = int(rng.integers(1, 4))
        th, tw = int(rng.integers(1, 10)), int(rng.integers(1, 10))
        sh, sw = int(rng.integers(1, th + 1)), int(rng.integers(1, tw + 1))
        nr, nc = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        H, W = (nr - 1) * sh + th, (nc - 1) * sw + tw
        heads = int(rng.integers(1, 4))
        out.append((T, H, W, th, tw, sh, sw, nr, nc, heads, int(rng.integers(0, H)), int(rng.integers(0, W)),
                    str(rng.choice(["f32", "bf16"]))))
    return out


@pytest.mark.parametrize("case", _random_tilings(30, 77), ids=lambda c: "T%d_%dx%d_tile%dx%d_s%dx%d_%dx%d_h%d_shift%d_%d_%s" % c)
def test_blend_slice_update_random_tilings(case):
    """Seeded random tilings (coverage from 1 x 1 up to 9 x 9, odd plane counts, any shift): slice, blend and
    fused update against the oracle."""
    T, H, W, th, tw, sh, sw, nr, nc, heads, dy, dx, dtype = case
    d = 64 if dtype == "f32" else 128
    g = TileGeometry("rt", T, H, W, th, tw, sh, sw, nr, nc, heads, d, dtype, 500 + H * 31 + W)
    p = sg.make_problem(g, shift=(dy, dx))
    tiles = [randn_tensor(g.tile_shape, dtype, g.seed + i).cuda() for i in range(g.n_tiles)]
    out = torch.full(g.grid_shape, float("nan"), dtype=torch_dtype(dtype), device="cuda")
    sg.sg_tile_blend(p, tiles, out)
    assert_close(to_f64(out), oracle.blend_shifted([to_f64(t) for t in tiles], g, dy, dx), dtype, "blend")
    lat = randn_tensor(g.grid_shape, dtype, g.seed + 999).cuda()
    ref = oracle.fuse_and_denoise([to_f64(t) for t in tiles], g, to_f64(lat), 1.0, 0.125, dy, dx)
    sg.sg_tile_blend_update(p, tiles, lat, 1.0, 0.125, lat)
    assert_close(to_f64(lat), ref, dtype, "update")
    c = randn_tensor(g.grid_shape, dtype, g.seed + 5).cuda()
    tr, tc = (g.seed * 3) % nr, (g.seed * 7) % nc
    dst = torch.full((1,) + g.tile_shape, float("nan"), dtype=torch_dtype(dtype), device="cuda")
    sg.sg_tile_slice(p, [c], tr, tc, dst)
    assert np.array_equal(to_f64(dst[0]), oracle.slice_tile_shifted(to_f64(c), g, tr, tc, dy, dx))


def test_refine_step_from_canvas_tensors_under_moving_partitions():
    """sg_refine_step_canvas = Shift + SliceTile of every tile + sg_refine_step: bit for bit the same as
    sg_tile_slice per tile followed by sg_refine_step, over four steps whose partition moves every step; the
    first step (every tile recomputed) is also checked against the oracle end to end."""
    g = _geom("rc", 2, 16, 24, 8, 12, 8, 12, 2, 128, "bf16", 41)         # 2 x 2 non-overlapping tiles, as in the paper
    n, E = g.n_tiles, int(np.prod(g.tile_shape))
    shifts = [(0, 0), (3, 7), (6, 14), (9, 21)]
    qkv = [randn_tensor(g.grid_shape, "bf16", g.seed + 5 * s).cuda() for s in range(3)]
    qkv0 = [to_f64(t) for t in qkv]

    def fresh():
        return dict(x=[[torch.zeros((3,) + g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)] for _ in range(2)],
                    outs=[[torch.zeros(g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)] for _ in range(2)],
                    delta=[torch.zeros(E, dtype=torch.float32, device="cuda") for _ in range(n)],
                    state=sg.GainState(n),
                    step_change=torch.zeros(n, dtype=torch.float32, device="cuda"),
                    scores=torch.zeros(n, dtype=torch.float32, device="cuda"),
                    rec=torch.zeros(n, dtype=torch.uint8, device="cuda"),
                    ws=torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda"),
                    latent=randn_tensor(g.grid_shape, "bf16", 778).cuda())

    a, b = fresh(), fresh()
    latent0 = to_f64(a["latent"])
    gen = torch.Generator(device="cuda")
    for k, shift in enumerate(shifts):
        p = sg.make_problem(g, shift=shift)
        if k:   # the canvas drifts a little between the steps
            gen.manual_seed(4100 + k)
            for t in qkv:
                t.add_((0.01 * torch.randn(t.shape, generator=gen, device="cuda", dtype=torch.float32)).to(t.dtype))
        coef = (1.0, -0.1 * (k + 1))
        upd = lambda d: dict(latent_in=d["latent"], latent_out=d["latent"], c_latent=coef[0], c_noise=coef[1])
        cur, prev = k % 2, (k + 1) % 2
        # (a) one call from the canvas tensors
        sg.sg_denoise_step_gain(p, None, a["x"][cur], a["x"][prev], a["outs"][cur], a["outs"][prev], a["delta"], a["state"],
                                0.05, a["step_change"], a["scores"], a["rec"], a["ws"], update=upd(a), canvas=qkv)
        # (b) the parts
        for tr in range(g.n_tile_rows):
            for tc in range(g.n_tile_cols):
                sg.sg_tile_slice(p, qkv, tr, tc, b["x"][cur][tr * g.n_tile_cols + tc])
        sg.sg_denoise_step_gain(p, None, b["x"][cur], b["x"][prev], b["outs"][cur], b["outs"][prev], b["delta"], b["state"],
                                0.05, b["step_change"], b["scores"], b["rec"], b["ws"], update=upd(b))
        torch.cuda.synchronize()
        for key in ("step_change", "scores", "rec", "latent"):
            assert torch.equal(a[key], b[key]), (k, key)
        for ta, tb in zip(a["x"][cur] + a["outs"][cur] + a["delta"], b["x"][cur] + b["outs"][cur] + b["delta"]):
            assert torch.equal(ta, tb), k
        if k == 0:
            assert a["rec"].cpu().tolist() == [1] * n
            outs = []
            for tr in range(g.n_tile_rows):
                for tc in range(g.n_tile_cols):
                    Q, K, V = (oracle.slice_tile_shifted(t, g, tr, tc, *shift) for t in qkv0)
                    outs.append(np.stack([oracle.attention(Q[h].reshape(-1, 128), K[h].reshape(-1, 128),
                                                           V[h].reshape(-1, 128), g.scale)
                                          for h in range(g.heads)]).reshape(g.tile_shape))
            assert_close(to_f64(a["latent"]), oracle.fuse_and_denoise(outs, g, latent0, coef[0], coef[1], *shift), "bf16", "latent")


def test_refine_step_canvas_rejected_call_gathers_nothing():
    g = _geom("rc", 2, 16, 24, 8, 12, 8, 12, 2, 128, "bf16", 41)
    n, E = g.n_tiles, int(np.prod(g.tile_shape))
    p = sg.make_problem(g)
    qkv = [torch.zeros(g.grid_shape, dtype=torch.bfloat16, device="cuda") for _ in range(3)]
    x = [[torch.zeros((3,) + g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)] for _ in range(2)]
    outs = [[torch.zeros(g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n)] for _ in range(2)]
    delta = [torch.zeros(E, dtype=torch.float32, device="cuda") for _ in range(n)]
    f = lambda: torch.zeros(n, dtype=torch.float32, device="cuda")
    ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    grid = torch.zeros(g.grid_shape, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sg.SgError):      # no workspace: rejected before any tile is gathered
        sg.sg_denoise_step_gain(p, grid, x[0], x[1], outs[0], outs[1], delta, sg.GainState(n), 0.05, f(), f(),
                                torch.zeros(n, dtype=torch.uint8, device="cuda"), None, canvas=qkv)
    torch.cuda.synchronize()
    assert all(int(t.abs().sum()) == 0 for t in x[0])


def test_canvas_steps_follow_the_shift_schedule():
    """Algorithm 1 over six steps on a non-overlapping 2 x 2 partition with loop step 4, shifting every second step:
    each step asks the library where the partition sits, runs the tiled step there (windows that wrap are read in
    place) and must give the oracle's shifted attention and Fuse; after the loop the partition is back at the start."""
    g = _geom("sched", 2, 16, 24, 8, 12, 8, 12, 2, 128, "bf16", 41)         # 2 x 2 non-overlapping tiles, N = 192
    qkv = [randn_tensor(g.grid_shape, "bf16", g.seed + 7 * s).cuda() for s in range(3)]
    host = [to_f64(t) for t in qkv]
    tiles = [torch.empty(g.tile_shape, dtype=torch.bfloat16, device="cuda") for _ in range(g.n_tiles)]
    canvas = torch.empty(g.grid_shape, dtype=torch.bfloat16, device="cuda")
    seen = []
    for step in range(9):
        shift = sg.sg_shift_schedule(sg.make_problem(g), step, loop_step=4, frequency=2)
        assert shift == oracle.shift_schedule(step, g.tile_h, g.tile_w, 4, 2)
        seen.append(shift)
        if step in (1, 3, 5, 7):       # one step of every position is enough
            continue
        p = sg.make_problem(g, shift=shift)
        sg.sg_denoise_step_tiled(p, canvas, tiles, q=qkv[0], k=qkv[1], v=qkv[2])
        torch.cuda.synchronize()
        outs = []
        for tr in range(g.n_tile_rows):
            for tc in range(g.n_tile_cols):
                Q, K, V = (oracle.slice_tile_shifted(t, g, tr, tc, *shift) for t in host)
                outs.append(np.stack([oracle.attention(Q[a].reshape(-1, 128), K[a].reshape(-1, 128), V[a].reshape(-1, 128), g.scale)
                                      for a in range(g.heads)]).reshape(g.tile_shape))
        for t, o in zip(tiles, outs):
            assert_close(to_f64(t), o, "bf16", f"step {step}")
        assert_close(to_f64(canvas), oracle.blend_shifted(outs, g, *shift), "bf16", f"canvas at step {step}")
    assert seen == [(0, 0), (0, 0), (2, 3), (2, 3), (4, 6), (4, 6), (6, 9), (6, 9), (0, 0)]
