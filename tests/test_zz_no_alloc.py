"""sg_cache_gate_static (the gate without a workspace, for callers that cannot allocate) against
sg_cache_gate on the same inputs: same kernels, so scores and decisions must be identical bit for bit;
both are also held to the oracle.  Two calls in a row share the library's fixed scratch, the second on
fewer, smaller tiles."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2508_17756_amd as sg
from synthetic import randn_tensor
from gpu_util import to_f64

pytestmark = pytest.mark.gpu


def _case(n_tiles, elems, seed, dtype="bf16"):
    cached = [randn_tensor((elems,), dtype, seed + 2 * i).cuda() for i in range(n_tiles)]
    cur = []
    for i, c in enumerate(cached):
        eps = 0.1 if i % 3 == 0 else 0.01            # scores near 0.1 and 0.01 around the 0.05 threshold
        noise = randn_tensor((elems,), "f32", seed + 2 * i + 1).cuda()
        cur.append((c.float() + eps * noise).to(c.dtype))
    has = torch.ones(n_tiles, dtype=torch.uint8, device="cuda")
    if n_tiles > 2:
        has[1] = 0                                    # one tile without a cache
    return cur, cached, has


def _both(cur, cached, has, thr):
    n = len(cur)
    ws = torch.empty(sg.sg_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    s_ref = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
    r_ref = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    sg.sg_cache_gate(cur, cached, has, thr, s_ref, r_ref, ws)
    s_new = torch.full((n,), -2.0, dtype=torch.float32, device="cuda")
    r_new = torch.full((n,), 9, dtype=torch.uint8, device="cuda")
    sg.sg_cache_gate_static(cur, cached, has, thr, s_new, r_new)
    torch.cuda.synchronize()
    return s_ref.cpu().numpy(), r_ref.cpu().numpy(), s_new.cpu().numpy(), r_new.cpu().numpy()


def _check_against_oracle(cur, cached, has, thr, scores, rec):
    thr32 = float(np.float32(thr))
    for i in range(len(cur)):
        if not has[i]:
            assert np.isinf(scores[i]) and rec[i] == 1
            continue
        ref = oracle.gate_score(to_f64(cur[i]), to_f64(cached[i]))
        assert abs(scores[i] - ref) <= 2e-6 * max(1.0, ref), (i, scores[i], ref)
        if abs(ref - thr32) > 1e-4:
            assert bool(rec[i]) == (ref >= thr32), (i, ref)


def test_static_gate_matches_workspace_gate_twice_in_a_row():
    thr = 0.05
    # first call: 7 tiles of 3 * 4099 * 8 + 5 elements (ragged against the 16-byte vectors)
    cur, cached, has = _case(7, 3 * 4099 * 8 + 5, 9100)
    s_ref, r_ref, s_new, r_new = _both(cur, cached, has, thr)
    assert np.array_equal(s_ref.view(np.uint32), s_new.view(np.uint32))
    assert np.array_equal(r_ref, r_new)
    _check_against_oracle(cur, cached, has.cpu().numpy(), thr, s_new, r_new)
    # second call right behind it: fewer and smaller tiles, so most of the scratch keeps the first call's sums
    cur2, cached2, has2 = _case(3, 1000, 9300, "f32")
    s_ref2, r_ref2, s_new2, r_new2 = _both(cur2, cached2, has2, thr)
    assert np.array_equal(s_ref2.view(np.uint32), s_new2.view(np.uint32))
    assert np.array_equal(r_ref2, r_new2)
    _check_against_oracle(cur2, cached2, has2.cpu().numpy(), thr, s_new2, r_new2)


def test_static_gate_limits_and_argument_checks():
    lib = sg.load_library()
    n = sg.SG_STATIC_GATE_MAX_TILES + 1
    arr = (ctypes.c_void_p * n)(*([256] * n))
    assert lib.sg_cache_gate_static(arr, arr, 256, n, 64, sg.SG_BF16, 0.05, 256, 256, None) == sg.SG_ERR_WORKSPACE
    assert lib.sg_cache_gate_static(arr, arr, 256, -1, 64, sg.SG_BF16, 0.05, 256, 256, None) == sg.SG_ERR_INVALID_ARG
    assert lib.sg_cache_gate_static(arr, arr, 256, 2, 64, sg.SG_BF16, float("nan"), 256, 256, None) == sg.SG_ERR_INVALID_ARG
    assert lib.sg_cache_gate_static(arr, None, 256, 2, 64, sg.SG_BF16, 0.05, 256, 256, None) == sg.SG_ERR_INVALID_ARG
    assert lib.sg_cache_gate_static(None, None, None, 0, 64, sg.SG_BF16, 0.05, None, None, None) == sg.SG_OK
    # the largest admitted tile count runs
    cur, cached, has = _case(sg.SG_STATIC_GATE_MAX_TILES, 2048, 9500)
    s_ref, r_ref, s_new, r_new = _both(cur, cached, has, 0.05)
    assert np.array_equal(s_ref.view(np.uint32), s_new.view(np.uint32)) and np.array_equal(r_ref, r_new)
