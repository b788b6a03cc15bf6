// C ABI of libsupergen_tile: host-side argument checks and the order of launches.
// Every step of the path runs in the HIP kernels of the sibling files; nothing is computed here.
#include <cmath>
#include "sg_common.h"

namespace sg {

static thread_local int g_last_hip_error = 0;

int note_hip_error(hipError_t e) {
  g_last_hip_error = (int)e;
  return SG_ERR_HIP;
}

static bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

static int validate(const sg_problem* p) {
  if (!p) return SG_ERR_INVALID_ARG;
  if (p->T <= 0 || p->H <= 0 || p->W <= 0 || p->tile_h <= 0 || p->tile_w <= 0 || p->stride_h <= 0 ||
      p->stride_w <= 0 || p->n_tile_rows <= 0 || p->n_tile_cols <= 0 || p->heads <= 0 || p->head_dim <= 0)
    return SG_ERR_INVALID_ARG;
  if (p->dtype != SG_F32 && p->dtype != SG_BF16) return SG_ERR_INVALID_ARG;
  if (!std::isfinite(p->scale) || p->scale <= 0.f) return SG_ERR_INVALID_ARG;
  if (p->stride_h > p->tile_h || p->stride_w > p->tile_w) return SG_ERR_INVALID_ARG;  // gaps between tiles
  if ((int64_t)(p->n_tile_rows - 1) * p->stride_h + p->tile_h != p->H) return SG_ERR_INVALID_ARG;
  if ((int64_t)(p->n_tile_cols - 1) * p->stride_w + p->tile_w != p->W) return SG_ERR_INVALID_ARG;
  if (p->grid_stride_token < p->head_dim || p->grid_stride_head <= 0) return SG_ERR_INVALID_ARG;
  if ((p->grid_stride_token & 7) || (p->grid_stride_head & 7)) return SG_ERR_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128) return SG_ERR_UNSUPPORTED;
  if ((int64_t)p->n_tile_rows * p->n_tile_cols > SG_MAX_TILES) return SG_ERR_UNSUPPORTED;
  if ((int64_t)p->T * p->tile_h * p->tile_w >= (1ll << 31)) return SG_ERR_UNSUPPORTED;
  if ((int64_t)p->heads * p->T >= 65536) return SG_ERR_UNSUPPORTED;
  // kernels address canvas tensors with 32-bit offsets in units of 8 elements
  const int64_t span = (int64_t)(p->heads - 1) * p->grid_stride_head +
                       ((int64_t)p->T * p->H * p->W - 1) * p->grid_stride_token + p->head_dim;
  if (span >= (1ll << 35)) return SG_ERR_UNSUPPORTED;
  if ((int64_t)p->H * p->W * (p->head_dim / 4) >= (1ll << 32)) return SG_ERR_UNSUPPORTED;
  if (p->shift_h < 0 || p->shift_h >= p->H || p->shift_w < 0 || p->shift_w >= p->W) return SG_ERR_INVALID_ARG;
  return SG_OK;
}

// Shape and strides shared by all tiles of p.
static TileView make_view(const sg_problem& p, bool wrapped) {
  TileView tv;
  tv.stride_token = p.grid_stride_token;
  tv.stride_head = p.grid_stride_head;
  tv.T = p.T; tv.H = p.H; tv.W = p.W; tv.th = p.tile_h; tv.tw = p.tile_w;
  tv.N = p.T * p.tile_h * p.tile_w;
  tv.wrapped = wrapped;
  return tv;
}

// A packed tile is a canvas that is exactly one tile.
static sg_problem packed_tile_problem(const sg_problem& p) {
  sg_problem tp = p;
  tp.H = p.tile_h; tp.W = p.tile_w; tp.n_tile_rows = tp.n_tile_cols = 1;
  tp.stride_h = p.tile_h; tp.stride_w = p.tile_w;
  tp.shift_h = tp.shift_w = 0;
  tp.grid_stride_token = p.head_dim;
  tp.grid_stride_head = (int64_t)p.T * p.tile_h * p.tile_w * p.head_dim;
  return tp;
}

static int attention_launch(const sg_problem& p, const TileView& tv, const AttnBatch& b, hipStream_t s) {
  if (p.dtype == SG_F32) return launch_attention_f32(tv, p.heads, p.head_dim, p.scale, b, s);
  return launch_attention_bf16(tv, p.heads, p.head_dim, p.scale, b, s);
}

// Attention of the listed tiles of canvas tensors q, k, v, read in place, in as few launches as possible
// (Algorithm 1: for all tiles of the partition).  Under a shifted partition the windows that cross a canvas
// edge are read through the wrapping loader and the others as ordinary windows at their shifted origin.
// tiles[i] = tile_row * n_tile_cols + tile_col;  out[i] = packed output of tiles[i].
static int attention_canvas_tiles(const sg_problem& p, const void* q, const void* k, const void* v, const int* tiles,
                                  int n, void* const* out, hipStream_t s) {
  const size_t esz = p.dtype == SG_BF16 ? 2 : 4;
  const void* qp[SG_MAX_TILES]; const void* kp[SG_MAX_TILES]; const void* vp[SG_MAX_TILES];
  void* op[SG_MAX_TILES];
  int32_t y0[SG_MAX_TILES], x0[SG_MAX_TILES];
  for (int pass = 0; pass < 2; ++pass) {   // pass 0: windows inside the canvas; pass 1: windows that wrap
    int m = 0;
    for (int i = 0; i < n; ++i) {
      const int tr = tiles[i] / p.n_tile_cols, tc = tiles[i] - tr * p.n_tile_cols;
      const int y = (int)(((int64_t)tr * p.stride_h + p.shift_h) % p.H), x = (int)(((int64_t)tc * p.stride_w + p.shift_w) % p.W);
      const bool wraps = y + p.tile_h > p.H || x + p.tile_w > p.W;
      if (wraps != (pass == 1)) continue;
      const size_t origin = wraps ? 0 : (size_t)(((int64_t)y * p.W + x) * p.grid_stride_token) * esz;
      qp[m] = (const char*)q + origin; kp[m] = (const char*)k + origin; vp[m] = (const char*)v + origin;
      op[m] = out[i];
      y0[m] = y; x0[m] = x;
      ++m;
    }
    if (!m) continue;
    const AttnBatch b = {m, qp, kp, vp, op, pass ? y0 : nullptr, pass ? x0 : nullptr, nullptr, nullptr, nullptr, 0, nullptr};
    const int st = attention_launch(p, make_view(p, pass == 1), b, s);
    if (st != SG_OK) return st;
  }
  return SG_OK;
}

// Attention of packed tile inputs x[i] = [3][heads][T][tile_h][tile_w][d] (Q, K, V) in one launch; tiles whose
// run flag (device) is 0 are skipped on the device.  With cache_x / has_cache the step's cache refresh (cache_x[i] <-
// x[i], has_cache[i] <- 1 for the tiles that run) rides on the same launch where the kernel can carry it, and is a
// launch of its own otherwise.
static int attention_packed_tiles(const sg_problem& p, const void* const* x, int n, void* const* out,
                                  const uint8_t* run_flags, hipStream_t s, void* const* cache_x = nullptr,
                                  uint8_t* has_cache = nullptr) {
  const sg_problem tp = packed_tile_problem(p);
  const size_t part = (size_t)p.heads * p.T * p.tile_h * p.tile_w * p.head_dim * (p.dtype == SG_BF16 ? 2 : 4);
  const void* qp[SG_MAX_TILES]; const void* kp[SG_MAX_TILES]; const void* vp[SG_MAX_TILES];
  for (int i = 0; i < n; ++i) {
    qp[i] = x[i];
    kp[i] = (const char*)x[i] + part;
    vp[i] = (const char*)x[i] + 2 * part;
  }
  bool refreshed = false;
  const AttnBatch b = {n, qp, kp, vp, out, nullptr, nullptr, run_flags, cache_x, has_cache,
                       cache_x ? (int64_t)(3 * part) : 0, &refreshed};
  const int st = attention_launch(tp, make_view(tp, false), b, s);
  if (st != SG_OK || !cache_x || refreshed) return st;
  return launch_cache_refresh(x, cache_x, run_flags, has_cache, n, (int64_t)(3 * part), s);
}

}  // namespace sg

using namespace sg;

extern "C" {

const char* sg_version(void) { return "0.1"; }

const char* sg_status_string(int status) {
  switch (status) {
    case SG_OK: return "ok";
    case SG_ERR_INVALID_ARG: return "invalid argument";
    case SG_ERR_UNSUPPORTED: return "unsupported problem";
    case SG_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SG_ERR_HIP: return "HIP call failed";
    default: return "unknown status";
  }
}

int sg_last_hip_error(void) { return g_last_hip_error; }

int sg_problem_validate(const sg_problem* p) { return validate(p); }

int sg_workspace_bytes(int32_t n_tiles, size_t* out_bytes) {
  if (!out_bytes || n_tiles < 0) return SG_ERR_INVALID_ARG;
  *out_bytes = gate_workspace_bytes(n_tiles);
  return SG_OK;
}

int sg_tile_attention(const sg_problem* p, const void* q, const void* k, const void* v, int32_t tile_row,
                      int32_t tile_col, void* out_tile, void* stream) {
  int st = validate(p);
  if (st != SG_OK) return st;
  if (!q || !k || !v || !out_tile) return SG_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out_tile)) return SG_ERR_INVALID_ARG;
  if (tile_row < 0 || tile_row >= p->n_tile_rows || tile_col < 0 || tile_col >= p->n_tile_cols)
    return SG_ERR_INVALID_ARG;
  const int tile = tile_row * p->n_tile_cols + tile_col;
  return attention_canvas_tiles(*p, q, k, v, &tile, 1, &out_tile, (hipStream_t)stream);
}

int sg_tile_blend(const sg_problem* p, const void* const* tile_out, void* grid_out, void* stream) {
  int st = validate(p);
  if (st != SG_OK) return st;
  if (!tile_out || !grid_out || !aligned16(grid_out)) return SG_ERR_INVALID_ARG;
  const int n_tiles = p->n_tile_rows * p->n_tile_cols;
  for (int i = 0; i < n_tiles; ++i)
    if (!tile_out[i] || !aligned16(tile_out[i])) return SG_ERR_INVALID_ARG;
  return launch_blend(*p, tile_out, grid_out, nullptr, 0.f, 0.f, (hipStream_t)stream);
}

int sg_tile_blend_update(const sg_problem* p, const void* const* tile_out, const void* latent_in, float c_latent,
                         float c_noise, void* latent_out, void* stream) {
  int st = validate(p);
  if (st != SG_OK) return st;
  if (!tile_out || !latent_in || !latent_out || !aligned16(latent_in) || !aligned16(latent_out)) return SG_ERR_INVALID_ARG;
  if (std::isnan(c_latent) || std::isnan(c_noise)) return SG_ERR_INVALID_ARG;
  const int n_tiles = p->n_tile_rows * p->n_tile_cols;
  for (int i = 0; i < n_tiles; ++i)
    if (!tile_out[i] || !aligned16(tile_out[i])) return SG_ERR_INVALID_ARG;
  return launch_blend(*p, tile_out, latent_out, latent_in, c_latent, c_noise, (hipStream_t)stream);
}

int sg_partition_tiles(sg_problem* p, int32_t tile_h, int32_t tile_w, int32_t overlap_h, int32_t overlap_w) {
  if (!p || p->H <= 0 || p->W <= 0) return SG_ERR_INVALID_ARG;
  const int32_t extent[2] = {p->H, p->W}, tile[2] = {tile_h, tile_w}, overlap[2] = {overlap_h, overlap_w};
  int32_t count[2], stride[2];
  for (int a = 0; a < 2; ++a) {
    if (tile[a] < 1 || tile[a] > extent[a] || overlap[a] < 0 || overlap[a] >= tile[a]) return SG_ERR_INVALID_ARG;
    stride[a] = tile[a] - overlap[a];
    if ((extent[a] - tile[a]) % stride[a] != 0) return SG_ERR_INVALID_ARG;   // the last tile would not end at the edge
    count[a] = (extent[a] - tile[a]) / stride[a] + 1;
  }
  if ((int64_t)count[0] * count[1] > SG_MAX_TILES) return SG_ERR_UNSUPPORTED;
  p->tile_h = tile_h; p->tile_w = tile_w;
  p->stride_h = stride[0]; p->stride_w = stride[1];
  p->n_tile_rows = count[0]; p->n_tile_cols = count[1];
  return SG_OK;
}

int sg_shift_schedule(const sg_problem* p, int32_t step, int32_t loop_step, int32_t frequency, int32_t* shift_h,
                      int32_t* shift_w) {
  sg_problem unshifted;
  if (!p || !shift_h || !shift_w) return SG_ERR_INVALID_ARG;
  unshifted = *p;                      // the schedule says where the partition goes: the caller's current shift is not an input
  unshifted.shift_h = unshifted.shift_w = 0;
  int st = validate(&unshifted);
  if (st != SG_OK) return st;
  if (step < 0 || loop_step < 1 || frequency < 1) return SG_ERR_INVALID_ARG;
  const int64_t moves = (step / frequency) % loop_step;
  *shift_h = (int32_t)(moves * p->tile_h / loop_step);   // < tile_h <= H
  *shift_w = (int32_t)(moves * p->tile_w / loop_step);
  return SG_OK;
}

int sg_tile_slice(const sg_problem* p, const void* const* src, int32_t n_src, int32_t tile_row, int32_t tile_col,
                  void* dst, void* stream) {
  int st = validate(p);
  if (st != SG_OK) return st;
  if (!src || n_src < 1 || n_src > 3 || !dst || !aligned16(dst)) return SG_ERR_INVALID_ARG;
  for (int i = 0; i < n_src; ++i)
    if (!src[i] || !aligned16(src[i])) return SG_ERR_INVALID_ARG;
  if (tile_row < 0 || tile_row >= p->n_tile_rows || tile_col < 0 || tile_col >= p->n_tile_cols)
    return SG_ERR_INVALID_ARG;
  return launch_slice(*p, src, n_src, tile_row, tile_col, dst, (hipStream_t)stream);
}

int sg_cache_gate(const void* const* x_cur, const void* const* x_cached, const uint8_t* has_cache, int32_t n_tiles,
                  int64_t elems_per_tile, int32_t dtype, float threshold, float* scores, uint8_t* recompute,
                  void* workspace, size_t workspace_bytes, void* stream) {
  if (n_tiles < 0 || elems_per_tile < 0) return SG_ERR_INVALID_ARG;
  if (dtype != SG_F32 && dtype != SG_BF16) return SG_ERR_INVALID_ARG;
  if (std::isnan(threshold)) return SG_ERR_INVALID_ARG;
  if (n_tiles == 0) return SG_OK;
  if (!x_cur || !x_cached || !has_cache || !scores || !recompute) return SG_ERR_INVALID_ARG;
  for (int i = 0; i < n_tiles; ++i) {
    if (!x_cur[i] || !aligned16(x_cur[i])) return SG_ERR_INVALID_ARG;
    if (!x_cached[i] || !aligned16(x_cached[i])) return SG_ERR_INVALID_ARG;
  }
  if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < gate_workspace_bytes(n_tiles))
    return SG_ERR_WORKSPACE;
  return launch_gate(x_cur, x_cached, has_cache, n_tiles, elems_per_tile, dtype, threshold, scores, recompute,
                     workspace, (hipStream_t)stream);
}

int sg_denoise_step_tiled(const sg_problem* p, const sg_step_io* io, void* stream) {
  int st = validate(p);
  if (st != SG_OK) return st;
  if (!io || !io->cache_out || !io->grid_out || !aligned16(io->grid_out)) return SG_ERR_INVALID_ARG;
  const int n_tiles = p->n_tile_rows * p->n_tile_cols;
  for (int i = 0; i < n_tiles; ++i)
    if (!io->cache_out[i] || !aligned16(io->cache_out[i])) return SG_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const size_t esz = p->dtype == SG_BF16 ? 2 : 4;
  const int64_t tile_elems = (int64_t)p->heads * p->T * p->tile_h * p->tile_w * p->head_dim;

  if (!io->tile_x) {  // canvas mode: every tile is recomputed from the shared canvas tensors
    if (!io->q || !io->k || !io->v) return SG_ERR_INVALID_ARG;
    if (!aligned16(io->q) || !aligned16(io->k) || !aligned16(io->v)) return SG_ERR_INVALID_ARG;
    // All tiles are read in place by one attention launch (windows of a shifted partition that cross a canvas
    // edge go through the wrapping loader).  With room for G >= 1 packed tile inputs in the workspace the tiles
    // are instead gathered G at a time (plain copies) and each group is attended in packed form by one launch:
    // a packed tile spans a fraction of the canvas' address range, which the streaming loads reward.
    const size_t packed_bytes = ((3 * (size_t)tile_elems * esz + 255) / 256) * 256;   // per tile, keeps every copy aligned
    const bool aligned_ws = io->workspace && !(((uintptr_t)io->workspace) & 255u);
    const size_t room = aligned_ws ? io->workspace_bytes / packed_bytes : 0;
    if (room == 0) {
      int tiles[SG_MAX_TILES];
      for (int i = 0; i < n_tiles; ++i) tiles[i] = i;
      st = attention_canvas_tiles(*p, io->q, io->k, io->v, tiles, n_tiles, io->cache_out, s);
      if (st != SG_OK) return st;
    } else {
      const int group = room < (size_t)n_tiles ? (int)room : n_tiles;
      const void* src[3] = {io->q, io->k, io->v};
      const void* x[SG_MAX_TILES];
      for (int t0 = 0; t0 < n_tiles; t0 += group) {
        const int n = n_tiles - t0 < group ? n_tiles - t0 : group;
        for (int i = 0; i < n; ++i) {
          char* dst = (char*)io->workspace + (size_t)i * packed_bytes;
          st = launch_slice(*p, src, 3, (t0 + i) / p->n_tile_cols, (t0 + i) % p->n_tile_cols, dst, s);
          if (st != SG_OK) return st;
          x[i] = dst;
        }
        st = attention_packed_tiles(*p, x, n, io->cache_out + t0, nullptr, s);
        if (st != SG_OK) return st;
      }
    }
    return launch_blend(*p, (const void* const*)io->cache_out, io->grid_out, nullptr, 0.f, 0.f, s);
  }

  // cached mode
  if (io->q || io->k || io->v) return SG_ERR_INVALID_ARG;
  if (!io->cache_x || !io->has_cache || !io->scores || !io->recompute) return SG_ERR_INVALID_ARG;
  if (std::isnan(io->threshold)) return SG_ERR_INVALID_ARG;
  for (int i = 0; i < n_tiles; ++i) {
    if (!io->tile_x[i] || !aligned16(io->tile_x[i])) return SG_ERR_INVALID_ARG;
    if (!io->cache_x[i] || !aligned16(io->cache_x[i])) return SG_ERR_INVALID_ARG;
  }
  if (!io->workspace || (((uintptr_t)io->workspace) & 255u) || io->workspace_bytes < gate_workspace_bytes(n_tiles))
    return SG_ERR_WORKSPACE;
  // threshold < 0: every score (>= 0 or +inf) is at or above it, so every tile recomputes
  st = launch_gate(io->tile_x, (const void* const*)io->cache_x, io->has_cache, n_tiles, 3 * tile_elems, p->dtype,
                   io->threshold, io->scores, io->recompute, io->workspace, s);
  if (st != SG_OK) return st;
  st = attention_packed_tiles(*p, io->tile_x, n_tiles, io->cache_out, io->recompute, s, io->cache_x, io->has_cache);
  if (st != SG_OK) return st;
  return launch_blend(*p, (const void* const*)io->cache_out, io->grid_out, nullptr, 0.f, 0.f, s);
}

static int check_gain_state(const sg_gain_state* st) {
  if (!st || !st->has_prev || !st->has_gain || !st->gain || !st->path_len) return SG_ERR_INVALID_ARG;
  return SG_OK;
}
static int check_ptr_array(const void* const* a, int n) {
  if (!a) return SG_ERR_INVALID_ARG;
  for (int i = 0; i < n; ++i)
    if (!a[i] || !aligned16(a[i])) return SG_ERR_INVALID_ARG;
  return SG_OK;
}

int sg_gain_gate(const void* const* x_cur, const void* const* x_prev, const sg_gain_state* state, int32_t n_tiles,
                 int64_t elems_per_tile, int32_t dtype, float threshold, const float* tile_thresholds,
                 float* step_change, float* scores, uint8_t* recompute, void* workspace, size_t workspace_bytes,
                 void* stream) {
  if (n_tiles < 0 || elems_per_tile < 0) return SG_ERR_INVALID_ARG;
  if (dtype != SG_F32 && dtype != SG_BF16) return SG_ERR_INVALID_ARG;
  if (std::isnan(threshold)) return SG_ERR_INVALID_ARG;
  if (n_tiles == 0) return SG_OK;
  if (check_gain_state(state) != SG_OK || !step_change || !scores || !recompute) return SG_ERR_INVALID_ARG;
  if (check_ptr_array(x_cur, n_tiles) != SG_OK || check_ptr_array(x_prev, n_tiles) != SG_OK) return SG_ERR_INVALID_ARG;
  if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < gate_workspace_bytes(n_tiles))
    return SG_ERR_WORKSPACE;
  return launch_gain_gate(x_cur, x_prev, *state, n_tiles, elems_per_tile, dtype, threshold, tile_thresholds,
                          step_change, scores, recompute, workspace, (hipStream_t)stream);
}

int sg_gain_refresh(void* const* out_cur, const void* const* out_prev, const void* const* latent, float* const* delta,
                    const uint8_t* recompute, const float* step_change, const sg_gain_state* state, int32_t n_tiles,
                    int64_t elems_per_tile, int32_t dtype, void* workspace, size_t workspace_bytes, void* stream) {
  if (n_tiles < 0 || elems_per_tile < 0 || (elems_per_tile & 7)) return SG_ERR_INVALID_ARG;
  if (dtype != SG_F32 && dtype != SG_BF16) return SG_ERR_INVALID_ARG;
  if (n_tiles == 0) return SG_OK;
  if (check_gain_state(state) != SG_OK || !recompute || !step_change) return SG_ERR_INVALID_ARG;
  if (check_ptr_array((const void* const*)out_cur, n_tiles) != SG_OK || check_ptr_array(out_prev, n_tiles) != SG_OK ||
      check_ptr_array(latent, n_tiles) != SG_OK || check_ptr_array((const void* const*)delta, n_tiles) != SG_OK)
    return SG_ERR_INVALID_ARG;
  if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < gate_workspace_bytes(n_tiles))
    return SG_ERR_WORKSPACE;
  return launch_gain_refresh(out_cur, out_prev, latent, delta, recompute, step_change, *state, n_tiles, elems_per_tile,
                             dtype, workspace, (hipStream_t)stream);
}

static int refine_step_check(const sg_problem* p, const sg_gain_step_io* io, const sg_region_control* region,
                             const sg_scheduler_update* update) {
  int st = validate(p);
  if (st != SG_OK) return st;
  if (!io) return SG_ERR_INVALID_ARG;
  if (update) {
    if (!update->latent_in || !update->latent_out || !aligned16(update->latent_in) || !aligned16(update->latent_out))
      return SG_ERR_INVALID_ARG;
    if (std::isnan(update->c_latent) || std::isnan(update->c_noise)) return SG_ERR_INVALID_ARG;
  } else if (!io->grid_out || !aligned16(io->grid_out)) {
    return SG_ERR_INVALID_ARG;
  }
  if (region) {
    if (!region->track_mean || !region->track_count || !region->tile_std || !region->thresholds) return SG_ERR_INVALID_ARG;
    if (region->mode != SG_REGION_MAXMIN && region->mode != SG_REGION_TOPSELECT) return SG_ERR_INVALID_ARG;
    if (std::isnan(region->tau_base) || std::isnan(region->alpha)) return SG_ERR_INVALID_ARG;
  }
  const int n_tiles = p->n_tile_rows * p->n_tile_cols;
  if (check_gain_state(&io->state) != SG_OK || !io->step_change || !io->scores || !io->recompute)
    return SG_ERR_INVALID_ARG;
  if (std::isnan(io->threshold)) return SG_ERR_INVALID_ARG;
  if (check_ptr_array(io->tile_x, n_tiles) != SG_OK || check_ptr_array(io->prev_x, n_tiles) != SG_OK ||
      check_ptr_array((const void* const*)io->out_cur, n_tiles) != SG_OK ||
      check_ptr_array(io->out_prev, n_tiles) != SG_OK || check_ptr_array((const void* const*)io->delta, n_tiles) != SG_OK)
    return SG_ERR_INVALID_ARG;
  if (io->latent && check_ptr_array(io->latent, n_tiles) != SG_OK) return SG_ERR_INVALID_ARG;
  if (!io->workspace || (((uintptr_t)io->workspace) & 255u) || io->workspace_bytes < gate_workspace_bytes(n_tiles))
    return SG_ERR_WORKSPACE;
  return SG_OK;
}

static int refine_step(const sg_problem* p, const sg_gain_step_io* io, const sg_region_control* region,
                       const sg_scheduler_update* update, void* stream) {
  int st = refine_step_check(p, io, region, update);
  if (st != SG_OK) return st;
  const int n_tiles = p->n_tile_rows * p->n_tile_cols;
  hipStream_t s = (hipStream_t)stream;
  const int64_t tile_elems = (int64_t)p->heads * p->T * p->tile_h * p->tile_w * p->head_dim;

  st = launch_gain_gate(io->tile_x, io->prev_x, io->state, n_tiles, 3 * tile_elems, p->dtype, io->threshold,
                        region ? region->thresholds : io->tile_thresholds, io->step_change, io->scores, io->recompute,
                        io->workspace, s);
  if (st != SG_OK) return st;
  st = attention_packed_tiles(*p, io->tile_x, n_tiles, io->out_cur, io->recompute, s);
  if (st != SG_OK) return st;
  // the residual is taken against the Q part of the packed input unless the caller names a latent
  st = launch_gain_refresh(io->out_cur, io->out_prev, io->latent ? io->latent : io->tile_x, io->delta, io->recompute,
                           io->step_change, io->state, n_tiles, tile_elems, p->dtype, io->workspace, s);
  if (st != SG_OK) return st;
  if (region) {   // StdTracker.Update on this step's outputs, thresholds for the next step
    st = launch_tile_std((const void* const*)io->out_cur, n_tiles, tile_elems, p->dtype, region->tile_std, io->workspace, s);
    if (st != SG_OK) return st;
    st = launch_region_thresholds(region->tile_std, region->track_mean, region->track_count, n_tiles, region->tau_base,
                                  region->alpha, region->mode, region->adjust != 0, region->sigma, region->thresholds, s);
    if (st != SG_OK) return st;
  }
  if (update)
    return launch_blend(*p, (const void* const*)io->out_cur, update->latent_out, update->latent_in, update->c_latent,
                        update->c_noise, s);
  return launch_blend(*p, (const void* const*)io->out_cur, io->grid_out, nullptr, 0.f, 0.f, s);
}

int sg_denoise_step_gain(const sg_problem* p, const sg_gain_step_io* io, void* stream) {
  return refine_step(p, io, nullptr, nullptr, stream);
}

int sg_refine_step(const sg_problem* p, const sg_gain_step_io* io, const sg_region_control* region,
                   const sg_scheduler_update* update, void* stream) {
  return refine_step(p, io, region, update, stream);
}

int sg_refine_step_canvas(const sg_problem* p, const void* q, const void* k, const void* v, void* const* tile_x,
                          const sg_gain_step_io* io, const sg_region_control* region,
                          const sg_scheduler_update* update, void* stream) {
  int st = validate(p);
  if (st != SG_OK) return st;
  if (!q || !k || !v || !aligned16(q) || !aligned16(k) || !aligned16(v) || !tile_x || !io || !io->tile_x)
    return SG_ERR_INVALID_ARG;
  const int n_tiles = p->n_tile_rows * p->n_tile_cols;
  for (int i = 0; i < n_tiles; ++i)
    if (!tile_x[i] || !aligned16(tile_x[i]) || io->tile_x[i] != tile_x[i]) return SG_ERR_INVALID_ARG;
  // every check of the step itself runs before the first launch: a rejected call leaves tile_x untouched
  st = refine_step_check(p, io, region, update);
  if (st != SG_OK) return st;
  const void* src[3] = {q, k, v};
  for (int tr = 0; tr < p->n_tile_rows; ++tr)
    for (int tc = 0; tc < p->n_tile_cols; ++tc) {
      st = launch_slice(*p, src, 3, tr, tc, tile_x[tr * p->n_tile_cols + tc], (hipStream_t)stream);
      if (st != SG_OK) return st;
    }
  return refine_step(p, io, region, update, stream);
}

int sg_tile_std(const void* const* x, int32_t n_tiles, int64_t elems_per_tile, int32_t dtype, float* tile_std,
                void* workspace, size_t workspace_bytes, void* stream) {
  if (n_tiles < 0 || elems_per_tile <= 0 || (elems_per_tile & 7)) return SG_ERR_INVALID_ARG;
  if (dtype != SG_F32 && dtype != SG_BF16) return SG_ERR_INVALID_ARG;
  if (n_tiles == 0) return SG_OK;
  if (!tile_std || check_ptr_array(x, n_tiles) != SG_OK) return SG_ERR_INVALID_ARG;
  if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < gate_workspace_bytes(n_tiles))
    return SG_ERR_WORKSPACE;
  return launch_tile_std(x, n_tiles, elems_per_tile, dtype, tile_std, workspace, (hipStream_t)stream);
}

int sg_tile_similarity(const void* const* x_new, const void* const* x_old, int32_t n_tiles, int64_t elems_per_tile,
                       int32_t dtype, float* l1_rel, float* cos_sim, void* workspace, size_t workspace_bytes, void* stream) {
  if (n_tiles < 0 || elems_per_tile < 0) return SG_ERR_INVALID_ARG;
  if (dtype != SG_F32 && dtype != SG_BF16) return SG_ERR_INVALID_ARG;
  if (n_tiles == 0) return SG_OK;
  if (!l1_rel || !cos_sim || check_ptr_array(x_new, n_tiles) != SG_OK || check_ptr_array(x_old, n_tiles) != SG_OK)
    return SG_ERR_INVALID_ARG;
  if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < gate_workspace_bytes(n_tiles))
    return SG_ERR_WORKSPACE;
  return launch_similarity(x_new, x_old, n_tiles, elems_per_tile, dtype, l1_rel, cos_sim, workspace, (hipStream_t)stream);
}

int sg_region_thresholds(const float* tile_std, double* track_mean, int32_t* track_count, int32_t n_tiles,
                         float tau_base, float alpha, int32_t mode, int32_t adjust, float* sigma, float* thresholds,
                         void* stream) {
  if (n_tiles < 0) return SG_ERR_INVALID_ARG;
  if (mode != SG_REGION_MAXMIN && mode != SG_REGION_TOPSELECT) return SG_ERR_INVALID_ARG;
  if (std::isnan(tau_base) || std::isnan(alpha)) return SG_ERR_INVALID_ARG;
  if (n_tiles == 0) return SG_OK;
  if (!tile_std || !track_mean || !track_count || !thresholds) return SG_ERR_INVALID_ARG;
  return launch_region_thresholds(tile_std, track_mean, track_count, n_tiles, tau_base, alpha, mode, adjust != 0, sigma,
                                  thresholds, (hipStream_t)stream);
}

}  // extern "C"
