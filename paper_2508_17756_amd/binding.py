"""ctypes binding with the same names as the C ABI in include/supergen_tile.h.

Argument marshalling only: tensors are torch tensors used as device buffers (their
data_ptr() and the current HIP stream are handed to the library); every step of the path
runs inside the library's kernels.  There is no fallback: if the shared library has not
been built, loading raises.
"""
import ctypes
import os

SG_F32, SG_BF16 = 0, 1
SG_OK, SG_ERR_INVALID_ARG, SG_ERR_UNSUPPORTED, SG_ERR_WORKSPACE, SG_ERR_HIP = 0, -1, -2, -3, -4
SG_REGION_MAXMIN, SG_REGION_TOPSELECT = 0, 1
SG_STATIC_GATE_MAX_TILES = 64

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class SgError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        text = load_library().sg_status_string(status).decode()
        super().__init__("%s failed: %s (%d)" % (where, text, status))


class sg_problem(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("tile_h", ctypes.c_int32), ("tile_w", ctypes.c_int32),
                ("stride_h", ctypes.c_int32), ("stride_w", ctypes.c_int32),
                ("n_tile_rows", ctypes.c_int32), ("n_tile_cols", ctypes.c_int32),
                ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("grid_stride_token", ctypes.c_int64), ("grid_stride_head", ctypes.c_int64),
                ("shift_h", ctypes.c_int32), ("shift_w", ctypes.c_int32)]


class sg_step_io(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("tile_x", ctypes.POINTER(ctypes.c_void_p)),
                ("cache_x", ctypes.POINTER(ctypes.c_void_p)),
                ("cache_out", ctypes.POINTER(ctypes.c_void_p)),
                ("has_cache", ctypes.c_void_p),
                ("threshold", ctypes.c_float),
                ("scores", ctypes.c_void_p), ("recompute", ctypes.c_void_p),
                ("grid_out", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


class sg_gain_state(ctypes.Structure):
    _fields_ = [("has_prev", ctypes.c_void_p), ("has_gain", ctypes.c_void_p),
                ("gain", ctypes.c_void_p), ("path_len", ctypes.c_void_p)]


class sg_gain_step_io(ctypes.Structure):
    _fields_ = [("tile_x", ctypes.POINTER(ctypes.c_void_p)), ("prev_x", ctypes.POINTER(ctypes.c_void_p)),
                ("latent", ctypes.POINTER(ctypes.c_void_p)),
                ("out_cur", ctypes.POINTER(ctypes.c_void_p)), ("out_prev", ctypes.POINTER(ctypes.c_void_p)),
                ("delta", ctypes.POINTER(ctypes.c_void_p)),
                ("state", sg_gain_state),
                ("threshold", ctypes.c_float),
                ("tile_thresholds", ctypes.c_void_p),
                ("step_change", ctypes.c_void_p), ("scores", ctypes.c_void_p), ("recompute", ctypes.c_void_p),
                ("grid_out", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


class sg_region_control(ctypes.Structure):
    _fields_ = [("track_mean", ctypes.c_void_p), ("track_count", ctypes.c_void_p), ("tile_std", ctypes.c_void_p),
                ("thresholds", ctypes.c_void_p), ("sigma", ctypes.c_void_p),
                ("tau_base", ctypes.c_float), ("alpha", ctypes.c_float),
                ("mode", ctypes.c_int32), ("adjust", ctypes.c_int32)]


class sg_scheduler_update(ctypes.Structure):
    _fields_ = [("latent_in", ctypes.c_void_p), ("latent_out", ctypes.c_void_p),
                ("c_latent", ctypes.c_float), ("c_noise", ctypes.c_float)]


def library_path():
    return os.path.join(_PKG, "libsupergen_tile.so")


def load_library():
    """Loads the in-tree shared library; raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError("%s is missing: build it with `python -m paper_2508_17756_amd.build` "
                          "(there is no CPU fallback)" % path)
    lib = ctypes.CDLL(path)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    pp = ctypes.POINTER(ctypes.c_void_p)
    lib.sg_version.restype = ctypes.c_char_p
    lib.sg_version.argtypes = []
    lib.sg_status_string.restype = ctypes.c_char_p
    lib.sg_status_string.argtypes = [ctypes.c_int]
    lib.sg_last_hip_error.restype = ctypes.c_int
    lib.sg_last_hip_error.argtypes = []
    lib.sg_problem_validate.restype = ctypes.c_int
    lib.sg_problem_validate.argtypes = [ctypes.POINTER(sg_problem)]
    lib.sg_workspace_bytes.restype = ctypes.c_int
    lib.sg_workspace_bytes.argtypes = [i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.sg_tile_attention.restype = ctypes.c_int
    lib.sg_tile_attention.argtypes = [ctypes.POINTER(sg_problem), vp, vp, vp, i32, i32, vp, vp]
    lib.sg_tile_blend.restype = ctypes.c_int
    lib.sg_tile_blend.argtypes = [ctypes.POINTER(sg_problem), pp, vp, vp]
    lib.sg_tile_blend_update.restype = ctypes.c_int
    lib.sg_tile_blend_update.argtypes = [ctypes.POINTER(sg_problem), pp, vp, f32, f32, vp, vp]
    lib.sg_partition_tiles.restype = ctypes.c_int
    lib.sg_partition_tiles.argtypes = [ctypes.POINTER(sg_problem), i32, i32, i32, i32]
    lib.sg_shift_schedule.restype = ctypes.c_int
    lib.sg_shift_schedule.argtypes = [ctypes.POINTER(sg_problem), i32, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.sg_tile_slice.restype = ctypes.c_int
    lib.sg_tile_slice.argtypes = [ctypes.POINTER(sg_problem), pp, i32, i32, i32, vp, vp]
    lib.sg_cache_gate.restype = ctypes.c_int
    lib.sg_cache_gate.argtypes = [pp, pp, vp, i32, i64, i32, f32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sg_cache_gate_static.restype = ctypes.c_int
    lib.sg_cache_gate_static.argtypes = [pp, pp, vp, i32, i64, i32, f32, vp, vp, vp]
    lib.sg_denoise_step_tiled.restype = ctypes.c_int
    lib.sg_denoise_step_tiled.argtypes = [ctypes.POINTER(sg_problem), ctypes.POINTER(sg_step_io), vp]
    lib.sg_gain_gate.restype = ctypes.c_int
    lib.sg_gain_gate.argtypes = [pp, pp, ctypes.POINTER(sg_gain_state), i32, i64, i32, f32, vp, vp, vp, vp, vp,
                                 ctypes.c_size_t, vp]
    lib.sg_gain_refresh.restype = ctypes.c_int
    lib.sg_gain_refresh.argtypes = [pp, pp, pp, pp, vp, vp, ctypes.POINTER(sg_gain_state), i32, i64, i32, vp,
                                    ctypes.c_size_t, vp]
    lib.sg_denoise_step_gain.restype = ctypes.c_int
    lib.sg_denoise_step_gain.argtypes = [ctypes.POINTER(sg_problem), ctypes.POINTER(sg_gain_step_io), vp]
    lib.sg_refine_step.restype = ctypes.c_int
    lib.sg_refine_step.argtypes = [ctypes.POINTER(sg_problem), ctypes.POINTER(sg_gain_step_io),
                                   ctypes.POINTER(sg_region_control), ctypes.POINTER(sg_scheduler_update), vp]
    lib.sg_refine_step_canvas.restype = ctypes.c_int
    lib.sg_refine_step_canvas.argtypes = [ctypes.POINTER(sg_problem), vp, vp, vp, pp, ctypes.POINTER(sg_gain_step_io),
                                          ctypes.POINTER(sg_region_control), ctypes.POINTER(sg_scheduler_update), vp]
    lib.sg_tile_std.restype = ctypes.c_int
    lib.sg_tile_std.argtypes = [pp, i32, i64, i32, vp, vp, ctypes.c_size_t, vp]
    lib.sg_tile_similarity.restype = ctypes.c_int
    lib.sg_tile_similarity.argtypes = [pp, pp, i32, i64, i32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sg_region_thresholds.restype = ctypes.c_int
    lib.sg_region_thresholds.argtypes = [vp, vp, vp, i32, f32, f32, i32, i32, vp, vp, vp]
    _LIB = lib
    return lib


# ------------------------------------------------------------------ marshalling helpers
def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return SG_F32
    if t.dtype == torch.bfloat16:
        return SG_BF16
    raise TypeError("tensors must be float32 or bfloat16")


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _ptr_array(tensors):
    arr = (ctypes.c_void_p * max(1, len(tensors)))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def _check(status, where):
    if status != SG_OK:
        raise SgError(status, where)


def make_problem(geom, dtype=None, token_major=False, shift=(0, 0)):
    """sg_problem for a geometry object with the fields of synthetic.TileGeometry (or any
    object with T, H, W, tile_h, tile_w, stride_h, stride_w, n_tile_rows, n_tile_cols, heads,
    head_dim, scale, dtype); canvas tensors are [heads][T][H][W][d] unless token_major."""
    p = sg_problem()
    for f in ("T", "H", "W", "tile_h", "tile_w", "stride_h", "stride_w", "n_tile_rows", "n_tile_cols",
              "heads", "head_dim"):
        setattr(p, f, int(getattr(geom, f)))
    d = dtype if dtype is not None else geom.dtype
    p.dtype = {"f32": SG_F32, "bf16": SG_BF16, SG_F32: SG_F32, SG_BF16: SG_BF16}[d]
    p.scale = float(geom.scale)
    if token_major:
        p.grid_stride_token = p.heads * p.head_dim
        p.grid_stride_head = p.head_dim
    else:
        p.grid_stride_token = p.head_dim
        p.grid_stride_head = p.T * p.H * p.W * p.head_dim
    p.shift_h, p.shift_w = int(shift[0]), int(shift[1])
    return p


# ------------------------------------------------------------------ the ABI, same names
def sg_version():
    return load_library().sg_version().decode()


def sg_status_string(status):
    return load_library().sg_status_string(int(status)).decode()


def sg_problem_validate(p):
    return load_library().sg_problem_validate(ctypes.byref(p))


def sg_workspace_bytes(n_tiles):
    out = ctypes.c_size_t(0)
    _check(load_library().sg_workspace_bytes(int(n_tiles), ctypes.byref(out)), "sg_workspace_bytes")
    return out.value


def sg_tile_attention(p, q, k, v, tile_row, tile_col, out_tile):
    """Enqueues the attention of tile (tile_row, tile_col) on the current stream."""
    st = load_library().sg_tile_attention(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), int(tile_row),
                                          int(tile_col), _ptr(out_tile), _stream())
    _check(st, "sg_tile_attention")
    return out_tile


def sg_tile_blend(p, tile_out, grid_out):
    arr = _ptr_array(tile_out)
    st = load_library().sg_tile_blend(ctypes.byref(p), arr, _ptr(grid_out), _stream())
    _check(st, "sg_tile_blend")
    return grid_out


def sg_tile_blend_update(p, tile_out, latent_in, c_latent, c_noise, latent_out):
    st = load_library().sg_tile_blend_update(ctypes.byref(p), _ptr_array(tile_out), _ptr(latent_in), float(c_latent),
                                             float(c_noise), _ptr(latent_out), _stream())
    _check(st, "sg_tile_blend_update")
    return latent_out


def sg_partition_tiles(p, tile_h, tile_w, overlap_h=0, overlap_w=0):
    """PartitionTiles: fills the tiling fields of p for its canvas p.H x p.W; returns p."""
    _check(load_library().sg_partition_tiles(ctypes.byref(p), int(tile_h), int(tile_w), int(overlap_h), int(overlap_w)),
           "sg_partition_tiles")
    return p


def sg_shift_schedule(p, step, loop_step=16, frequency=1):
    """(shift_h, shift_w) of the partition at denoising step `step` (Algorithm 1 "ShiftThisStep" / "Shift")."""
    dy, dx = ctypes.c_int32(0), ctypes.c_int32(0)
    st = load_library().sg_shift_schedule(ctypes.byref(p), int(step), int(loop_step), int(frequency), ctypes.byref(dy),
                                          ctypes.byref(dx))
    _check(st, "sg_shift_schedule")
    return dy.value, dx.value


def sg_tile_slice(p, src, tile_row, tile_col, dst):
    """src: list of 1..3 canvas tensors; dst: packed [len(src)][heads][T][tile_h][tile_w][d]."""
    st = load_library().sg_tile_slice(ctypes.byref(p), _ptr_array(src), len(src), int(tile_row), int(tile_col),
                                      _ptr(dst), _stream())
    _check(st, "sg_tile_slice")
    return dst


def sg_cache_gate(x_cur, x_cached, has_cache, threshold, scores, recompute, workspace, elems_per_tile=None):
    n = len(x_cur)
    elems = int(elems_per_tile if elems_per_tile is not None else (x_cur[0].numel() if n else 0))
    dt = _dtype_code(x_cur[0]) if n else SG_BF16
    st = load_library().sg_cache_gate(_ptr_array(x_cur), _ptr_array(x_cached), _ptr(has_cache), n, elems, dt,
                                      float(threshold), _ptr(scores), _ptr(recompute), _ptr(workspace),
                                      workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                      _stream())
    _check(st, "sg_cache_gate")
    return scores, recompute


def sg_cache_gate_static(x_cur, x_cached, has_cache, threshold, scores, recompute, elems_per_tile=None):
    """sg_cache_gate without a workspace (the library's fixed scratch; at most SG_STATIC_GATE_MAX_TILES tiles)."""
    n = len(x_cur)
    elems = int(elems_per_tile if elems_per_tile is not None else (x_cur[0].numel() if n else 0))
    dt = _dtype_code(x_cur[0]) if n else SG_BF16
    st = load_library().sg_cache_gate_static(_ptr_array(x_cur), _ptr_array(x_cached), _ptr(has_cache), n, elems, dt,
                                             float(threshold), _ptr(scores), _ptr(recompute), _stream())
    _check(st, "sg_cache_gate_static")
    return scores, recompute


def sg_denoise_step_tiled(p, grid_out, cache_out, q=None, k=None, v=None, tile_x=None, cache_x=None,
                          has_cache=None, threshold=-1.0, scores=None, recompute=None, workspace=None):
    io = sg_step_io()
    io.q, io.k, io.v = _ptr(q), _ptr(k), _ptr(v)
    keep = [_ptr_array(cache_out)]
    io.cache_out = keep[0]
    if tile_x is not None:
        keep += [_ptr_array(tile_x), _ptr_array(cache_x)]
        io.tile_x, io.cache_x = keep[1], keep[2]
    io.has_cache = _ptr(has_cache)
    io.threshold = float(threshold)
    io.scores, io.recompute = _ptr(scores), _ptr(recompute)
    io.grid_out = _ptr(grid_out)
    io.workspace = _ptr(workspace)
    io.workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = load_library().sg_denoise_step_tiled(ctypes.byref(p), ctypes.byref(io), _stream())
    _check(st, "sg_denoise_step_tiled")
    return grid_out


class GainState:
    """Device-resident per-tile state of the gain / path-length cache policy (zero-initialised)."""

    def __init__(self, n_tiles, device="cuda"):
        import torch
        n = max(1, int(n_tiles))
        self.has_prev = torch.zeros(n, dtype=torch.uint8, device=device)
        self.has_gain = torch.zeros(n, dtype=torch.uint8, device=device)
        self.gain = torch.zeros(n, dtype=torch.float32, device=device)
        self.path_len = torch.zeros(n, dtype=torch.float32, device=device)

    def as_struct(self):
        st = sg_gain_state()
        st.has_prev, st.has_gain = _ptr(self.has_prev), _ptr(self.has_gain)
        st.gain, st.path_len = _ptr(self.gain), _ptr(self.path_len)
        return st


def _nbytes(t):
    return t.numel() * t.element_size() if t is not None else 0


def sg_gain_gate(x_cur, x_prev, state, threshold, step_change, scores, recompute, workspace,
                 tile_thresholds=None, elems_per_tile=None):
    n = len(x_cur)
    elems = int(elems_per_tile if elems_per_tile is not None else (x_cur[0].numel() if n else 0))
    dt = _dtype_code(x_cur[0]) if n else SG_BF16
    st = state.as_struct()
    rc = load_library().sg_gain_gate(_ptr_array(x_cur), _ptr_array(x_prev), ctypes.byref(st), n, elems, dt,
                                     float(threshold), _ptr(tile_thresholds), _ptr(step_change), _ptr(scores),
                                     _ptr(recompute), _ptr(workspace), _nbytes(workspace), _stream())
    _check(rc, "sg_gain_gate")
    return step_change, scores, recompute


def sg_gain_refresh(out_cur, out_prev, latent, delta, recompute, step_change, state, workspace, elems_per_tile=None):
    n = len(out_cur)
    elems = int(elems_per_tile if elems_per_tile is not None else (out_cur[0].numel() if n else 0))
    dt = _dtype_code(out_cur[0]) if n else SG_BF16
    st = state.as_struct()
    rc = load_library().sg_gain_refresh(_ptr_array(out_cur), _ptr_array(out_prev), _ptr_array(latent), _ptr_array(delta),
                                        _ptr(recompute), _ptr(step_change), ctypes.byref(st), n, elems, dt,
                                        _ptr(workspace), _nbytes(workspace), _stream())
    _check(rc, "sg_gain_refresh")
    return out_cur


def sg_denoise_step_gain(p, grid_out, tile_x, prev_x, out_cur, out_prev, delta, state, threshold, step_change,
                         scores, recompute, workspace, latent=None, tile_thresholds=None, region=None, update=None,
                         canvas=None):
    """region: dict(track_mean, track_count, tile_std, thresholds, tau_base, alpha, mode, adjust[, sigma]);
    update: dict(latent_in, latent_out, c_latent, c_noise).  With either one the call goes to sg_refine_step.
    canvas: (q, k, v) canvas tensors; the call goes to sg_refine_step_canvas, which first gathers every
    tile's window (under p's shift) into tile_x."""
    io = sg_gain_step_io()
    keep = [_ptr_array(tile_x), _ptr_array(prev_x), _ptr_array(out_cur), _ptr_array(out_prev), _ptr_array(delta)]
    io.tile_x, io.prev_x, io.out_cur, io.out_prev, io.delta = keep
    if latent is not None:
        keep.append(_ptr_array(latent))
        io.latent = keep[-1]
    io.state = state.as_struct()
    io.threshold = float(threshold)
    io.tile_thresholds = _ptr(tile_thresholds)
    io.step_change, io.scores, io.recompute = _ptr(step_change), _ptr(scores), _ptr(recompute)
    io.grid_out = _ptr(grid_out)
    io.workspace, io.workspace_bytes = _ptr(workspace), _nbytes(workspace)
    if region is None and update is None and canvas is None:
        rc = load_library().sg_denoise_step_gain(ctypes.byref(p), ctypes.byref(io), _stream())
        _check(rc, "sg_denoise_step_gain")
        return grid_out
    rg = up = None
    if region is not None:
        rg = sg_region_control()
        rg.track_mean, rg.track_count = _ptr(region["track_mean"]), _ptr(region["track_count"])
        rg.tile_std, rg.thresholds, rg.sigma = _ptr(region["tile_std"]), _ptr(region["thresholds"]), _ptr(region.get("sigma"))
        rg.tau_base, rg.alpha = float(region["tau_base"]), float(region["alpha"])
        rg.mode, rg.adjust = int(region["mode"]), int(bool(region["adjust"]))
    if update is not None:
        up = sg_scheduler_update()
        up.latent_in, up.latent_out = _ptr(update["latent_in"]), _ptr(update["latent_out"])
        up.c_latent, up.c_noise = float(update["c_latent"]), float(update["c_noise"])
    rg_ref = ctypes.byref(rg) if rg is not None else None
    up_ref = ctypes.byref(up) if up is not None else None
    if canvas is not None:
        q, k, v = canvas
        rc = load_library().sg_refine_step_canvas(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), keep[0], ctypes.byref(io),
                                                  rg_ref, up_ref, _stream())
        _check(rc, "sg_refine_step_canvas")
    else:
        rc = load_library().sg_refine_step(ctypes.byref(p), ctypes.byref(io), rg_ref, up_ref, _stream())
        _check(rc, "sg_refine_step")
    return update["latent_out"] if update is not None else grid_out


def sg_tile_std(x, tile_std, workspace, elems_per_tile=None):
    n = len(x)
    elems = int(elems_per_tile if elems_per_tile is not None else (x[0].numel() if n else 8))
    dt = _dtype_code(x[0]) if n else SG_BF16
    rc = load_library().sg_tile_std(_ptr_array(x), n, elems, dt, _ptr(tile_std), _ptr(workspace), _nbytes(workspace),
                                    _stream())
    _check(rc, "sg_tile_std")
    return tile_std


def sg_tile_similarity(x_new, x_old, l1_rel, cos_sim, workspace, elems_per_tile=None):
    """Equation 3 per tile: relative L1 distance (x_old in the denominator) and cosine similarity."""
    n = len(x_new)
    elems = int(elems_per_tile if elems_per_tile is not None else (x_new[0].numel() if n else 0))
    dt = _dtype_code(x_new[0]) if n else SG_BF16
    rc = load_library().sg_tile_similarity(_ptr_array(x_new), _ptr_array(x_old), n, elems, dt, _ptr(l1_rel), _ptr(cos_sim),
                                           _ptr(workspace), _nbytes(workspace), _stream())
    _check(rc, "sg_tile_similarity")
    return l1_rel, cos_sim


def sg_region_thresholds(tile_std, track_mean, track_count, tau_base, alpha, mode, adjust, thresholds, sigma=None):
    """track_mean: float64 device tensor, track_count: int32 device tensor of one element."""
    n = int(tile_std.numel())
    rc = load_library().sg_region_thresholds(_ptr(tile_std), _ptr(track_mean), _ptr(track_count), n, float(tau_base),
                                             float(alpha), int(mode), int(bool(adjust)), _ptr(sigma), _ptr(thresholds),
                                             _stream())
    _check(rc, "sg_region_thresholds")
    return thresholds
