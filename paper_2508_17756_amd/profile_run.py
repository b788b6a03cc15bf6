#!/usr/bin/env python3
"""Launches each kernel of the library a few times, for use under rocprofv3.

    rocprofv3 --kernel-trace --stats -d OUT -o NAME -- python3 paper_2508_17756_amd/profile_run.py
    rocprofv3 --pmc FETCH_SIZE   -d OUT -o NAME -- python3 paper_2508_17756_amd/profile_run.py
    rocprofv3 --pmc WRITE_SIZE   -d OUT -o NAME -- python3 paper_2508_17756_amd/profile_run.py

Sections (choose with --kernels, comma separated):
  copy       an elementwise copy of a 2 GiB buffer (reads 2 GiB, writes 2 GiB): the known
             traffic the FETCH_SIZE / WRITE_SIZE counters are scaled by
  attention  sg_tile_attention on the 75,600-token tile, 40 heads x 128, bf16
  attention64  the same tile at 48 heads x 64 (not in the default list)
  blend      sg_tile_blend of the 4K canvas (20 tiles of 75,600 tokens -> 21 x 135 x 240)
  gate       sg_cache_gate over 4 tiles of packed Q,K,V (2.32 GB per tile and side)
  update     sg_tile_blend_update of the 4K canvas (blend + scheduler update in place)
  refresh    sg_gain_refresh over 8 tiles, every second one recomputed
  std        sg_tile_std over 8 tile outputs
  similarity sg_tile_similarity over 8 pairs of tile outputs
Every section prints the bytes (or FLOP) the algorithm needs per launch, so a counter
summary can be set beside it.  Inputs are seeded synthetic N(0,1) values generated on the device.
"""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--kernels", default="copy,attention,blend,gate,update,refresh,std,similarity")
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()
    todo = args.kernels.split(",")

    import numpy as np
    import torch
    import paper_2508_17756_amd as sg
    from synthetic import CONFIGS, randn_tensor

    seed = [7000]

    def rnd(shape, dtype="bf16"):
        """seeded N(0,1) device tensor; every call takes the next seed"""
        seed[0] += 1
        return randn_tensor(shape, dtype, seed[0], device="cuda")

    sg.load_library()
    torch.cuda.set_device(0)

    def say(msg):
        print(msg, flush=True)

    if "copy" in todo:
        n = 1 << 30
        a = rnd((n,))
        b = torch.empty_like(a)
        for _ in range(args.reps):
            torch.neg(a, out=b)          # one elementwise kernel: reads 2 GiB, writes 2 GiB
        torch.cuda.synchronize()
        say("copy: elementwise neg of %d bf16 values, %d launches, %d bytes read + %d bytes written per launch"
            % (n, args.reps, 2 * n, 2 * n))
        del a, b

    if "attention" in todo:
        g = CONFIGS["tile720p_bf16"]
        p = sg.make_problem(g)
        q, k, v = (rnd(g.grid_shape) for _ in range(3))
        out = torch.empty(g.tile_shape, dtype=torch.bfloat16, device="cuda")
        for _ in range(args.reps):
            sg.sg_tile_attention(p, q, k, v, 0, 0, out)
        torch.cuda.synchronize()
        E = int(np.prod(g.tile_shape))
        say("attention: %d launches, %.6e FLOP per launch, algorithmic HBM bytes per launch %d (Q,K,V read once, O written once)"
            % (args.reps, g.attention_flops_per_tile, 4 * E * 2))
        del q, k, v, out

    if "attention64" in todo:
        from dataclasses import replace
        g = replace(CONFIGS["tile720p_bf16"], heads=48, head_dim=64)
        p = sg.make_problem(g)
        q, k, v = (rnd(g.grid_shape) for _ in range(3))
        out = torch.empty(g.tile_shape, dtype=torch.bfloat16, device="cuda")
        for _ in range(args.reps):
            sg.sg_tile_attention(p, q, k, v, 0, 0, out)
        torch.cuda.synchronize()
        say("attention64: %d launches, %.6e FLOP per launch (48 heads x 64)" % (args.reps, 4.0 * g.tile_tokens ** 2 * 64 * 48))
        del q, k, v, out

    if "blend" in todo:
        g = CONFIGS["canvas4k_bf16"]
        p = sg.make_problem(g)
        tiles = [rnd(g.tile_shape) for _ in range(g.n_tiles)]
        canvas = torch.empty(g.grid_shape, dtype=torch.bfloat16, device="cuda")
        for _ in range(args.reps):
            sg.sg_tile_blend(p, tiles, canvas)
        torch.cuda.synchronize()
        say("blend: %d launches, per launch %d bytes read (tile outputs) + %d bytes written (canvas)"
            % (args.reps, 2 * g.n_tiles * int(np.prod(g.tile_shape)), 2 * int(np.prod(g.grid_shape))))
        del tiles, canvas

    if "update" in todo:
        g = CONFIGS["canvas4k_bf16"]
        p = sg.make_problem(g)
        tiles = [rnd(g.tile_shape) for _ in range(g.n_tiles)]
        latent = rnd(g.grid_shape)
        for _ in range(args.reps):
            sg.sg_tile_blend_update(p, tiles, latent, 1.0, -0.02, latent)
        torch.cuda.synchronize()
        say("update: %d launches, per launch %d bytes read (tile outputs + latent) + %d bytes written (latent)"
            % (args.reps, 2 * (g.n_tiles * int(np.prod(g.tile_shape)) + int(np.prod(g.grid_shape))),
               2 * int(np.prod(g.grid_shape))))
        del tiles, latent

    if "refresh" in todo or "std" in todo or "similarity" in todo:
        g = CONFIGS["canvas4k_bf16"]
        n, E = 8, int(np.prod(g.tile_shape))
        o_cur = [rnd(g.tile_shape) for _ in range(n)]
        ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        if "refresh" in todo:
            o_prev = [rnd(g.tile_shape) for _ in range(n)]
            latent = [rnd(g.tile_shape) for _ in range(n)]
            delta = [torch.zeros(E, dtype=torch.float32, device="cuda") for _ in range(n)]
            state = sg.GainState(n)
            state.has_prev.fill_(1)
            half = torch.tensor([i % 2 for i in range(n)], dtype=torch.uint8, device="cuda")
            step_change = torch.full((n,), 0.05, dtype=torch.float32, device="cuda")
            for _ in range(args.reps):
                sg.sg_gain_refresh(o_cur, o_prev, latent, delta, half, step_change, state, ws)
            torch.cuda.synchronize()
            say("refresh: %d launches over %d tiles (%d recomputed), per launch %d bytes read + %d bytes written"
                % (args.reps, n, n // 2, E * (6 * (n // 2) + 6 * (n - n // 2)), E * (4 * (n // 2) + 2 * (n - n // 2))))
            del o_prev, latent, delta
        if "std" in todo:
            out = torch.empty(n, dtype=torch.float32, device="cuda")
            for _ in range(args.reps):
                sg.sg_tile_std(o_cur, out, ws)
            torch.cuda.synchronize()
            say("std: %d launches over %d tiles, per launch %d bytes read" % (args.reps, n, 2 * E * n))
        if "similarity" in todo:
            o_old = [rnd(g.tile_shape) for _ in range(n)]
            l1 = torch.empty(n, dtype=torch.float32, device="cuda")
            cs = torch.empty(n, dtype=torch.float32, device="cuda")
            for _ in range(args.reps):
                sg.sg_tile_similarity(o_cur, o_old, l1, cs, ws)
            torch.cuda.synchronize()
            say("similarity: %d launches over %d tiles, per launch %d bytes read" % (args.reps, n, 2 * 2 * E * n))
            del o_old
        del o_cur

    if "gate" in todo:
        g = CONFIGS["canvas4k_bf16"]
        n, E = 4, int(np.prod(g.tile_shape))
        cur = [rnd((3 * E,)) for _ in range(n)]
        old = [rnd((3 * E,)) for _ in range(n)]
        has = torch.ones(n, dtype=torch.uint8, device="cuda")
        sc = torch.empty(n, dtype=torch.float32, device="cuda")
        rc = torch.empty(n, dtype=torch.uint8, device="cuda")
        ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        for _ in range(args.reps):
            sg.sg_cache_gate(cur, old, has, 0.05, sc, rc, ws)
        torch.cuda.synchronize()
        say("gate: %d launches over %d tiles, per launch %d bytes read" % (args.reps, n, 2 * 3 * E * 2 * n))


if __name__ == "__main__":
    main()
