"""GPU parity of the region-aware threshold control (sg_tile_std, sg_region_thresholds) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_17756_amd as sg
from synthetic import randn_tensor, torch_dtype, perturb_
from gpu_util import to_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("elems", [8, 4096 + 8, 2 * 3 * 10 * 10 * 64, 1 << 21])
def test_tile_std_small(dtype, elems):
    n = 5
    scale = [1.0, 0.01, 3.0, 1.0, 0.0]
    shift = [0.0, 0.0, -2.0, 50.0, 1.5]          # tile 3: mean far from zero; tile 4: constant
    x = [(randn_tensor((elems,), "f32", 40 + i) * scale[i] + shift[i]).to(torch_dtype(dtype)).cuda() for i in range(n)]
    out = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    sg.sg_tile_std(x, out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for i in range(n):
        ref = oracle.tile_std(to_f64(x[i]))
        assert abs(got[i] - ref) <= 2e-5 * max(ref, 1e-3), (i, got[i], ref)
    assert got[4] == 0.0


@pytest.mark.parametrize("mode", ["MaxMin", "TopSelect"])
def test_region_thresholds_follow_algorithm_2(mode):
    """Eight steps, thresholds adjusted every third step: the device tracker and policy against the
    oracle's, both fed the same stored per-step standard deviations."""
    n, tau, alpha, every = 7, 0.05, 0.4, 3
    code = sg.SG_REGION_MAXMIN if mode == "MaxMin" else sg.SG_REGION_TOPSELECT
    rng = np.random.default_rng(7)
    track_mean = torch.full((n,), 123.0, dtype=torch.float64, device="cuda")     # garbage: the first update overwrites it
    track_count = torch.zeros(1, dtype=torch.int32, device="cuda")
    thr = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
    sigma = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
    tr = oracle.StdTracker(n)
    ref_thr = np.full(n, float(np.float32(tau)))
    for s in range(1, 9):
        stds = torch.tensor(rng.random(n) + 0.1, dtype=torch.float32)
        if s == 5:
            stds[2] = stds[4]                                                     # a tie on this step's values
        adjust = s % every == 0
        sg.sg_region_thresholds(stds.cuda(), track_mean, track_count, tau, alpha, code, adjust, thr, sigma=sigma)
        torch.cuda.synchronize()
        tr.update(stds.numpy().astype(np.float64))
        if adjust:
            ref_thr = oracle.region_thresholds(tr.normalized(), float(np.float32(tau)), float(np.float32(alpha)), mode)
            np.testing.assert_allclose(sigma.cpu().numpy(), tr.normalized(), rtol=0, atol=1e-6)
        np.testing.assert_array_equal(track_mean.cpu().numpy(), tr.mean)          # same fp64 recurrence
        np.testing.assert_allclose(thr.cpu().numpy(), ref_thr, rtol=1e-6)
        assert int(track_count.item()) == s


def test_region_thresholds_edge_cases():
    def run(stds, mode, adjust=True, tau=1.0, alpha=0.2):
        n = len(stds)
        tm = torch.zeros(n, dtype=torch.float64, device="cuda")
        tc = torch.zeros(1, dtype=torch.int32, device="cuda")
        thr = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
        sg.sg_region_thresholds(torch.tensor(stds, dtype=torch.float32, device="cuda"), tm, tc, tau, alpha, mode, adjust, thr)
        torch.cuda.synchronize()
        return thr.cpu().numpy()
    np.testing.assert_allclose(run([0.5, 0.9, 0.9, 0.1, 0.1], sg.SG_REGION_MAXMIN), [1, 1.2, 1, 0.9, 1], rtol=1e-6)
    np.testing.assert_allclose(run([0.5, 0.9, 0.9, 0.1, 0.1], sg.SG_REGION_TOPSELECT), [1, 1.2, 1.1, 1, 1], rtol=1e-6)
    np.testing.assert_allclose(run([0.3, 0.3], sg.SG_REGION_MAXMIN), [0.9, 1.0], rtol=1e-6)     # all equal
    np.testing.assert_allclose(run([0.3], sg.SG_REGION_TOPSELECT), [1.2], rtol=1e-6)            # one tile
    np.testing.assert_allclose(run([0.3, 0.7, 0.1], sg.SG_REGION_MAXMIN, adjust=False), [1, 1, 1], rtol=1e-6)
    big = list(np.linspace(0.1, 0.9, 300))                                                        # more tiles than threads
    got = run(big, sg.SG_REGION_TOPSELECT)
    assert got[299] == np.float32(1.2) and got[298] == np.float32(1.1) and (got[:298] == 1.0).all()


def test_std_tracker_drives_the_gain_gate_thresholds():
    """The thresholds produced here are what sg_gain_gate consumes: a tile whose threshold was raised
    reuses where its neighbour with the same score recomputes."""
    n, elems = 3, 4096
    prev = [randn_tensor((elems,), "bf16", 70 + i).cuda() for i in range(n)]
    cur = [(p.float() * 1.0625).to(torch.bfloat16) for p in prev]                 # every tile: d = 1/16 up to bf16 rounding
    state = sg.GainState(n)
    state.has_prev.fill_(1)
    state.has_gain.fill_(1)
    state.gain.fill_(1.0)
    tm = torch.zeros(n, dtype=torch.float64, device="cuda")
    tc = torch.zeros(1, dtype=torch.int32, device="cuda")
    thr = torch.empty(n, dtype=torch.float32, device="cuda")
    sg.sg_region_thresholds(torch.tensor([0.2, 0.8, 0.5], device="cuda"), tm, tc, 0.05, 0.4, sg.SG_REGION_MAXMIN, True, thr)
    step = torch.empty(n, dtype=torch.float32, device="cuda")
    scores = torch.empty(n, dtype=torch.float32, device="cuda")
    rec = torch.empty(n, dtype=torch.uint8, device="cuda")
    ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    sg.sg_gain_gate(cur, prev, state, 0.05, step, scores, rec, ws, tile_thresholds=thr)
    torch.cuda.synchronize()
    assert all(abs(v - 0.0625) < 1e-3 for v in scores.cpu().tolist())             # thresholds 0.04, 0.07, 0.05
    assert rec.cpu().tolist() == [1, 0, 1]


# ------------------------------------------------------------------ similarity pair of Equation 3
def _similarity(x_new, x_old):
    n = len(x_new)
    l1 = torch.full((max(n, 1),), -5.0, dtype=torch.float32, device="cuda")
    cs = torch.full((max(n, 1),), -5.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    sg.sg_tile_similarity(x_new, x_old, l1, cs, ws)
    torch.cuda.synchronize()
    return l1.cpu().numpy()[:n], cs.cpu().numpy()[:n]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("elems", [8, 1000, 4099, 3 * 2 * 3 * 10 * 10 * 64, (1 << 20) + 3])
def test_similarity_against_the_oracle(dtype, elems):
    """Relative L1 distance and cosine similarity (Equation 3) of five tile pairs: identical, barely moved, moved,
    opposite, unrelated; element counts that are ragged against the 16-byte vectors and against the workgroups."""
    n = 5
    old = [randn_tensor((elems,), dtype, 2100 + i).cuda() for i in range(n)]
    new = [old[0].clone(), perturb_(old[1].clone(), 0.01, 2201), perturb_(old[2].clone(), 0.5, 2202), -old[3],
           randn_tensor((elems,), dtype, 2204).cuda()]
    l1, cs = _similarity(new, old)
    for i in range(n):
        ref_l1, ref_cs = oracle.similarity(to_f64(new[i]), to_f64(old[i]))
        assert abs(l1[i] - ref_l1) <= 2e-6 * max(1.0, ref_l1), (i, l1[i], ref_l1)
        assert abs(cs[i] - ref_cs) <= 3e-6, (i, cs[i], ref_cs)
    assert l1[0] == 0.0 and abs(cs[0] - 1.0) <= 3e-6 and abs(cs[3] + 1.0) <= 3e-6 and abs(l1[3] - 2.0) <= 4e-6


def test_similarity_zero_tensors_many_tiles_and_arguments():
    x = randn_tensor((4096,), "bf16", 2300).cuda()
    z = torch.zeros_like(x)
    l1, cs = _similarity([x, z, z], [z, x, z])
    assert np.isinf(l1[0]) and cs[0] == 0.0 and l1[1] == 1.0 and cs[1] == 0.0 and np.isinf(l1[2]) and cs[2] == 0.0
    n = 70                                                           # more than one launch's table of pointers
    old = [randn_tensor((2048,), "bf16", 2400 + i).cuda() for i in range(n)]
    new = [perturb_(t.clone(), 0.05 * (1 + i % 4), 2500 + i) for i, t in enumerate(old)]
    l1, cs = _similarity(new, old)
    for i in (0, 1, 63, 64, 69):
        ref_l1, ref_cs = oracle.similarity(to_f64(new[i]), to_f64(old[i]))
        assert abs(l1[i] - ref_l1) <= 2e-6 * max(1.0, ref_l1) and abs(cs[i] - ref_cs) <= 3e-6, i
    _similarity([], [])
    with pytest.raises(sg.SgError) as e:
        sg.sg_tile_similarity([x], [x], torch.empty(1, device="cuda"), torch.empty(1, device="cuda"),
                              torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == sg.SG_ERR_WORKSPACE
