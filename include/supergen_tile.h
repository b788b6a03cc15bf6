/*
 * supergen_tile.h - C ABI of the tile-based denoising hot path on one MI355X (gfx950).
 *
 * The library computes, for a latent canvas of T x H x W tokens that is partitioned into
 * overlapping tiles along H and W only (every tile keeps all T frames; paper Section 4.2,
 * Algorithm 1 stage 2: PartitionTiles / SliceTile):
 *
 *   sg_tile_attention       3D full self-attention over one tile's tokens (paper Section 2.1
 *                           "full attention"; Section 3: no Q/K/V exchange across tiles)
 *   sg_tile_blend           Fuse: merge all tile outputs into the full canvas (Algorithm 1
 *                           "Fuse"; Section 4.2; Tile Fuser of Section 5)
 *   sg_cache_gate           per-tile cache decision from the relative L1 change of the tile
 *                           input (Equation 3) against a threshold (Equation 7)
 *   sg_denoise_step_tiled   one stage-2 step: gate -> attention on the tiles to recompute ->
 *                           cache refresh -> Fuse (Algorithm 1 loop body; Section 5.1 pipeline)
 *
 * Conventions shared by every entry point
 *   - "device" pointers are HIP device memory on the current device; "host" pointers are
 *     ordinary process memory.  Every buffer is owned by the caller; the library allocates
 *     nothing and keeps no state between calls (scratch comes from the caller's workspace;
 *     sg_cache_gate_static alone uses a fixed device array of the library's own).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it and the calls return without waiting; no host readback takes place.
 *   - Every call is a fixed sequence of kernel launches, so it can be captured in a HIP graph and
 *     replayed.  The first bf16 attention launch on a device raises that kernel's dynamic-LDS limit
 *     (a one-time function attribute): make one call outside of capture first.
 *   - Inputs are never written.  Outputs must not alias inputs (exceptions are stated per call).
 *   - Argument checks run on the host before anything is launched; a failed check launches
 *     nothing.  Return value: SG_OK (0) or a negative sg_status.
 *   - Element types: SG_F32 (IEEE binary32) or SG_BF16 (bfloat16, round-to-nearest-even on
 *     store).  bf16 problems multiply in bf16 on the matrix cores and accumulate in fp32;
 *     f32 problems compute in fp32 throughout.
 *   - Token order: a canvas token (t, y, x) has linear index n = (t*H + y)*W + x; element c of
 *     head a of token n of a canvas tensor lives at
 *         base + a*grid_stride_head + n*grid_stride_token + c          (in elements),
 *     so [heads][T][H][W][d] (grid_stride_token = d, grid_stride_head = T*H*W*d) and
 *     [T][H][W][heads][d] (grid_stride_token = heads*d, grid_stride_head = d) are both
 *     expressible.  Canvas base pointers must be 16-byte aligned and both strides multiples of
 *     8 elements.
 *   - A packed tile is [heads][T][tile_h][tile_w][d], contiguous; tile tokens are ordered
 *     (t, i, j) with j fastest.  Tile (tile_row, tile_col) has its top-left token at canvas
 *     row tile_row*stride_h, column tile_col*stride_w; tiles are listed row-major.
 */
#ifndef SUPERGEN_TILE_H
#define SUPERGEN_TILE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SG_F32 = 0, SG_BF16 = 1 } sg_dtype;

typedef enum {
  SG_OK = 0,
  SG_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, tiles not covering the canvas, ... */
  SG_ERR_UNSUPPORTED = -2, /* a valid problem this build has no kernel for (head_dim, dtype, tile count) */
  SG_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or smaller than sg_workspace_bytes() */
  SG_ERR_HIP = -4          /* a HIP call failed; see sg_last_hip_error() */
} sg_status;

/* Largest number of tiles per canvas (their pointers travel as kernel arguments). */
#define SG_MAX_TILES 256

/* Problem statement: canvas, tiling, attention shape.  Plain data, passed by pointer (host). */
typedef struct sg_problem {
  int32_t T, H, W;                  /* canvas size in tokens                                   */
  int32_t tile_h, tile_w;           /* tile size in tokens (a tile spans all T)                */
  int32_t stride_h, stride_w;       /* spacing of tile origins; overlap = tile - stride >= 0   */
  int32_t n_tile_rows, n_tile_cols; /* (n-1)*stride + tile must equal H (resp. W)              */
  int32_t heads, head_dim;          /* head_dim: 64 or 128 (either dtype)                      */
  int32_t dtype;                    /* sg_dtype of every tensor of the problem                 */
  float scale;                      /* softmax scale applied to Q.K^T, > 0 (1/sqrt(head_dim))  */
  int64_t grid_stride_token;        /* canvas tensors: elements between consecutive tokens     */
  int64_t grid_stride_head;         /* canvas tensors: elements between consecutive heads      */
  int32_t shift_h, shift_w;         /* tile shifting (Algorithm 1 "Shift"): offset of the whole partition on
                                       the canvas, wrapping around: token (i, j) of tile (r, c) sits at canvas
                                       row (r*stride_h + i + shift_h) mod H, column (c*stride_w + j + shift_w)
                                       mod W.  0 <= shift_h < H, 0 <= shift_w < W; 0 = the fixed partition. */
} sg_problem;

/* Library version, "major.minor". */
const char* sg_version(void);
/* Static text for a status code. */
const char* sg_status_string(int status);
/* Numeric hipError_t of the last failed HIP call made by the calling thread (0 if none). */
int sg_last_hip_error(void);

/* Checks a problem statement (host only, launches nothing). */
int sg_problem_validate(const sg_problem* p);

/* Bytes of device scratch that sg_cache_gate / sg_denoise_step_tiled need for `n_tiles` tiles.
 * The workspace must be 256-byte aligned device memory; its contents need no initialisation
 * and it may be reused by the next call on the same stream. */
int sg_workspace_bytes(int32_t n_tiles, size_t* out_bytes);

/*
 * Tile attention (paper Sections 2.1 and 3; Algorithm 1 "SliceTile" + the self-attention of
 * "Model.DiT").  For tile (tile_row, tile_col), per head a and tile token n:
 *     O[a][n][:] = sum_m softmax_m( scale * <Q[a][n], K[a][m]> ) * V[a][m][:]
 * over all N = T*tile_h*tile_w tokens m of the same tile: bidirectional, no mask, no bias.
 *   q, k, v   device, canvas tensors (layout above); the tile is read in place, never copied
 *   out_tile  device, packed tile [heads][T][tile_h][tile_w][head_dim], 16-byte aligned
 * A packed tile is attended by describing it as a canvas that is one tile (H = tile_h,
 * W = tile_w, 1 x 1 tiles).  Under a shifted partition (shift_h or shift_w non-zero) the tile's
 * window is read at its shifted position, wrapping around the canvas edges where it crosses them
 * (a window that wraps is read row by row and runs somewhat slower than one that does not; gathering
 * it with sg_tile_slice and attending the packed copy is the faster route for large tiles).
 * Q is multiplied by scale * log2(e) and rounded to bf16 once more before the products of a bf16
 * problem (the score then leaves the matrix cores as the exponent): one extra bf16 rounding of the
 * scores' left factor on top of "multiply in bf16, accumulate in fp32".
 */
int sg_tile_attention(const sg_problem* p, const void* q, const void* k, const void* v,
                      int32_t tile_row, int32_t tile_col, void* out_tile, void* stream);

/*
 * Fuse / overlap blend (Algorithm 1 "Fuse"; Section 4.2).  For every canvas token g, head and
 * channel:
 *     out[g] = sum_{tiles covering g} w(g) * O_tile(g)  /  sum_{tiles covering g} w(g)
 *     w = w_h(i) * w_w(j),  w_axis(i) = min(1, (i+1)/(o+1), (L-i)/(o+1)),
 * i, j = the token's row/column inside the tile, L = tile length and o = L - stride along that
 * axis; the T axis carries weight 1.  With o = 0 this is the paper's non-overlapping placement.
 * Under a shifted partition (shift_h, shift_w) tile tokens land at their wrapped canvas positions.
 * Weights and sums are fp32; one rounding to the output type.
 *   tile_out  host array of n_tile_rows*n_tile_cols device pointers to packed tiles (row-major)
 *   grid_out  device, canvas tensor with the problem's strides
 */
int sg_tile_blend(const sg_problem* p, const void* const* tile_out, void* grid_out, void* stream);

/*
 * Fuse followed by the scheduler update in one pass (Algorithm 1: n = Fuse(N); L = Model.Denoise(L, n);
 * Section 4.2: the tile predictions are aggregated before the update so the canvas follows one
 * trajectory).  Every first-order sampler step is affine in the latent and the fused prediction:
 *     latent_out = c_latent * latent_in + c_noise * Fuse(tile_out)
 * (flow-matching Euler: c_latent = 1, c_noise = sigma_next - sigma).  The fused prediction is never
 * written to memory.  latent_in and latent_out are canvas tensors with the problem's strides;
 * latent_out may be latent_in (update in place).  One rounding to the tensors' type.
 */
int sg_tile_blend_update(const sg_problem* p, const void* const* tile_out, const void* latent_in, float c_latent,
                         float c_noise, void* latent_out, void* stream);

/*
 * PartitionTiles (Algorithm 1, stage 2; Section 4.2: the canvas is cut along height and width only).  Host only.
 * Fills p->tile_h, tile_w, stride_h, stride_w, n_tile_rows, n_tile_cols for tiles of tile_h x tile_w tokens whose
 * neighbours share overlap_h / overlap_w tokens (0 = the paper's non-overlapping tiles) on the canvas p->H x p->W,
 * which must be set; the other fields of *p are neither read nor written.  Tiles sit at multiples of
 * stride = tile - overlap and the last one has to end at the canvas edge: if no such partition exists, or more than
 * SG_MAX_TILES tiles result, nothing is written (SG_ERR_INVALID_ARG / SG_ERR_UNSUPPORTED).
 */
int sg_partition_tiles(sg_problem* p, int32_t tile_h, int32_t tile_w, int32_t overlap_h, int32_t overlap_w);

/*
 * Where the partition sits at a denoising step (Algorithm 1 "ShiftThisStep" / "Shift"; Section 4.2: deterministic
 * shifts along both directions with a fixed stride; Section 8 "Workloads": loop step 16, i.e. a stride of 1/16 of the
 * tile size, shifting every step; appendix: loop step = 1 / shift stride, a frequency of x shifts every x steps).
 * Host only; nothing is launched.  With moves = (step / frequency) mod loop_step (integer division):
 *     *shift_h = floor(moves * tile_h / loop_step),   *shift_w = floor(moves * tile_w / loop_step)
 * - after loop_step moves the partition has travelled one whole tile, which for equal non-overlapping tiles on the
 * wrapping canvas is the partition it started from.  The results are valid sg_problem.shift_h / shift_w values.
 *   step >= 0: 0 for the first denoising step;  loop_step >= 1;  frequency >= 1 (anything else: SG_ERR_INVALID_ARG)
 */
int sg_shift_schedule(const sg_problem* p, int32_t step, int32_t loop_step, int32_t frequency, int32_t* shift_h,
                      int32_t* shift_w);

/*
 * SliceTile into packed form (Algorithm 1 "SliceTile"; with shift_h / shift_w the shifted, wrapping
 * partition of "Shift").  Gathers the window of tile (tile_row, tile_col) out of n_src (1..3) canvas
 * tensors into dst = [n_src][heads][T][tile_h][tile_w][d]; with q, k, v as the sources dst is the
 * packed tile input of sg_denoise_step_tiled's cached mode.
 *   src   host array of n_src device pointers to canvas tensors;  dst: device, 16-byte aligned
 */
int sg_tile_slice(const sg_problem* p, const void* const* src, int32_t n_src, int32_t tile_row, int32_t tile_col,
                  void* dst, void* stream);

/*
 * Cache gate (Equation 3 relative L1 with the cached tensor as denominator; Equation 7:
 * strictly below the threshold reuses, at or above recomputes).  Per tile i:
 *     score[i]     = sum|x_cur[i] - x_cached[i]| / sum|x_cached[i]|      (+inf if the sum is 0)
 *     recompute[i] = !has_cache[i] || score[i] >= threshold
 * A tile without a cache gets score +inf and its buffers are not read.
 *   x_cur, x_cached  host arrays of n_tiles device pointers, each `elems_per_tile` elements of
 *                    `dtype`, 16-byte aligned; any elems_per_tile >= 0 (a ragged tail is summed too)
 *   has_cache        device, n_tiles bytes (0/1)
 *   scores           device, n_tiles floats (out);  recompute: device, n_tiles bytes (out)
 *   workspace        device scratch of at least sg_workspace_bytes(n_tiles)
 * Partial sums are fp32 per thread and fp64 across threads in a fixed order, so results are
 * bit-reproducible from run to run.
 */
int sg_cache_gate(const void* const* x_cur, const void* const* x_cached, const uint8_t* has_cache,
                  int32_t n_tiles, int64_t elems_per_tile, int32_t dtype, float threshold,
                  float* scores, uint8_t* recompute, void* workspace, size_t workspace_bytes,
                  void* stream);

/*
 * sg_cache_gate for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * sg_cache_gate, but without a workspace: the partial sums live in a fixed 1 MiB device array inside
 * the library (one copy per device, held until the process ends).  The call allocates and frees
 * nothing.  At most SG_STATIC_GATE_MAX_TILES tiles per call; more returns SG_ERR_WORKSPACE and
 * launches nothing.  Every call on a device shares that device's array: calls that may overlap on one
 * device (different streams, different threads) race and must be ordered by the caller; calls on one
 * stream are ordered by the stream.  Nothing needs clearing between calls.  The first call on a
 * device looks the array's address up; make it outside of graph capture.
 */
#define SG_STATIC_GATE_MAX_TILES 64
int sg_cache_gate_static(const void* const* x_cur, const void* const* x_cached, const uint8_t* has_cache,
                         int32_t n_tiles, int64_t elems_per_tile, int32_t dtype, float threshold,
                         float* scores, uint8_t* recompute, void* stream);

/*
 * Similarity of a tile tensor across adjacent denoising steps (Equation 3, both measures), per tile i:
 *     l1_rel[i]  = sum|x_new[i] - x_old[i]| / sum|x_old[i]|      (+inf if the sum is 0; sg_cache_gate's score)
 *     cos_sim[i] = <x_new[i], x_old[i]> / (||x_new[i]||_2 ||x_old[i]||_2)   (0 if either norm is 0)
 * the pair the paper profiles predicted noise and cache residuals with (Section 3; Section 5.1).  One read of
 * both tensors; sums in fp32 per thread, fp64 across threads in a fixed order.
 *   x_new, x_old   host arrays of n_tiles device pointers, elems_per_tile elements of `dtype`, 16-byte aligned
 *   l1_rel, cos_sim  device, n_tiles floats each (out);  workspace: as sg_cache_gate
 */
int sg_tile_similarity(const void* const* x_new, const void* const* x_old, int32_t n_tiles, int64_t elems_per_tile,
                       int32_t dtype, float* l1_rel, float* cos_sim, void* workspace, size_t workspace_bytes, void* stream);

/* Buffers of one tiled step.  All arrays of pointers are host arrays of device pointers. */
typedef struct sg_step_io {
  /* Canvas mode (gate off): q, k, v are canvas tensors and every tile is recomputed.        */
  const void* q;
  const void* k;
  const void* v;
  /* Cached mode: tile_x[i] is tile i's packed input [3][heads][T][tile_h][tile_w][d] (Q, K, V
   * one after the other); q, k, v must then be NULL.                                        */
  const void* const* tile_x;
  void* const* cache_x;   /* cached mode: per-tile cached input, same shape as tile_x[i]; refreshed on recompute */
  void* const* cache_out; /* both modes: per-tile packed attention output; the blend reads these                */
  uint8_t* has_cache;     /* cached mode: device, n_tiles bytes, in/out (set to 1 on recompute)                 */
  float threshold;        /* cached mode: cache threshold; < 0 switches the gate off (all tiles recompute)      */
  float* scores;          /* cached mode: device, n_tiles floats (out)                                          */
  uint8_t* recompute;     /* cached mode: device, n_tiles bytes (out)                                           */
  void* grid_out;         /* device, canvas tensor (out)                                                        */
  void* workspace;        /* cached mode: device scratch, sg_workspace_bytes(n_tiles); canvas mode: optional,   */
                          /* room for one or more packed tile inputs (see sg_denoise_step_tiled)                */
  size_t workspace_bytes;
} sg_step_io;

/*
 * One stage-2 step over all tiles (Algorithm 1 loop body; Section 5.1: Tile Dispatcher ->
 * Threshold Comparator -> recompute or reuse -> Tile Fuser).
 *   canvas mode: cache_out[i] = attention(tile i of q, k, v) for every tile; grid_out = Fuse.  All
 *     tiles are read in place and attended by one launch (two under a shifted partition: the windows
 *     that wrap around a canvas edge and those that do not).  If `workspace` (256-byte aligned) holds
 *     G >= 1 packed tile inputs (each 3 * heads * T * tile_h * tile_w * head_dim elements, rounded up
 *     to 256 bytes), the tiles are instead gathered into it G at a time (sg_tile_slice) and every group
 *     is attended in packed form by one launch; with room for all tiles this is the fastest form.
 *   cached mode: gate every tile on tile_x[i] against cache_x[i]; for the tiles to recompute
 *     cache_out[i] = attention(tile_x[i]), cache_x[i] = tile_x[i], has_cache[i] = 1; reused
 *     tiles keep their cache entries untouched (drift stays measured from the last recomputed
 *     step); grid_out = Fuse of all cache_out.
 * The decisions stay on the device and nothing is read back: one attention launch covers all tiles
 * and numbers only the work of the tiles to recompute; for bf16 problems the same launch also carries
 * the cache refresh, on the compute units its last, partial round of workgroups leaves idle.
 */
int sg_denoise_step_tiled(const sg_problem* p, const sg_step_io* io, void* stream);

/* ------------------------------------------------------------------------------------------
 * Inter-step tile-wise cache policy of the paper (Section 5.1).  Where sg_cache_gate compares the
 * tile input with the cached input directly, this policy keeps per tile
 *     delta_c   the cache residual O_c - I_c of the last recomputed step c (fp32, device buffer),
 *     g_c       the gain ||O_t - O_{t-1}|| / ||I_t - I_{t-1}|| measured when step c ran (Equation 5),
 *     L         the latent path length sum ||I_z - I_{z-1}|| since step c (Equation 6),
 * reuses a tile while g_c * L < tau_i with O_t = I_t + delta_c (Residual Approximation), and
 * otherwise recomputes it and sets c = t (Equation 7).  The paper does not name the norm; every
 * ||X_z - X_{z-1}|| here is the relative L1 change sum|X_z - X_{z-1}| / sum|X_{z-1}| of Equation 3
 * (+inf if the denominator is 0), which makes the thresholds dimensionless like the paper's.
 * While g_c is unknown (it needs two consecutive outputs) the tile recomputes: a tile's first two
 * steps always run the engine.  On reused steps O_{t-1} is the approximated output.
 * The caller double-buffers inputs and outputs: this step's x_cur / out_cur are the next step's
 * x_prev / out_prev. */
typedef struct sg_gain_state {   /* device arrays of n_tiles entries, read and updated by the calls below */
  uint8_t* has_prev;   /* 1 once the tile has a previous step (x_prev / out_prev valid); start at 0 */
  uint8_t* has_gain;   /* 1 once g_c is known; start at 0                                           */
  float* gain;         /* g_c                                                                       */
  float* path_len;     /* L; start at 0                                                             */
} sg_gain_state;

/*
 * Error Calculator and Threshold Comparator (Equations 6 and 7).  Per tile i:
 *     d = has_prev ? ||x_cur - x_prev|| : 0;   L += d;   score = has_gain ? g_c * L : +inf;
 *     recompute = !(has_gain && score < tau_i)         (a NaN score recomputes)
 *   x_cur, x_prev    host arrays of n_tiles device pointers, elems_per_tile elements each (as sg_cache_gate)
 *   threshold        tau for every tile, unless tile_thresholds (device, n_tiles floats) is not NULL
 *   step_change      device, n_tiles floats (out): d, consumed by sg_gain_refresh
 *   scores, recompute, workspace: as sg_cache_gate
 */
int sg_gain_gate(const void* const* x_cur, const void* const* x_prev, const sg_gain_state* state,
                 int32_t n_tiles, int64_t elems_per_tile, int32_t dtype, float threshold,
                 const float* tile_thresholds, float* step_change, float* scores, uint8_t* recompute,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cache Store update after the engine has written out_cur[i] for the tiles to recompute.  Per tile:
 *   recomputed: delta[i] = out_cur[i] - latent[i]; if has_prev and 0 < d < inf:
 *               g_c = ||out_cur - out_prev|| / d, has_gain = 1 (else g_c keeps its state); L = 0;
 *   reused:     out_cur[i] = latent[i] + delta[i]   (one rounding to the tensors' type);
 *   every tile: has_prev = 1.
 *   out_cur, out_prev, latent  host arrays of device pointers, elems_per_tile elements of `dtype`
 *                              (latent[i] = the tensor I_t the residual is taken against)
 *   delta                      host array of device pointers, elems_per_tile floats each
 *   elems_per_tile             a multiple of 8
 */
int sg_gain_refresh(void* const* out_cur, const void* const* out_prev, const void* const* latent,
                    float* const* delta, const uint8_t* recompute, const float* step_change,
                    const sg_gain_state* state, int32_t n_tiles, int64_t elems_per_tile, int32_t dtype,
                    void* workspace, size_t workspace_bytes, void* stream);

/* Buffers of one step under this policy; arrays of pointers are host arrays of device pointers. */
typedef struct sg_gain_step_io {
  const void* const* tile_x;   /* this step's packed tile inputs [3][heads][T][tile_h][tile_w][d] (Q, K, V) */
  const void* const* prev_x;   /* the previous step's (not read while has_prev = 0)                          */
  const void* const* latent;   /* I_t per tile, packed tile shape; NULL: the Q part of tile_x                */
  void* const* out_cur;        /* this step's tile outputs (written for every tile; the blend reads these)   */
  const void* const* out_prev; /* the previous step's                                                        */
  float* const* delta;         /* cache residuals                                                            */
  sg_gain_state state;
  float threshold;
  const float* tile_thresholds; /* device or NULL */
  float* step_change;           /* device, n_tiles (out) */
  float* scores;                /* device, n_tiles (out) */
  uint8_t* recompute;           /* device, n_tiles (out) */
  void* grid_out;
  void* workspace;
  size_t workspace_bytes;
} sg_gain_step_io;

/* One stage-2 step: sg_gain_gate on the packed inputs -> attention of the tiles to recompute into
 * out_cur -> sg_gain_refresh -> Fuse of out_cur into grid_out.  Nothing is read back. */
int sg_denoise_step_gain(const sg_problem* p, const sg_gain_step_io* io, void* stream);

/* ------------------------------------------------------------------------------------------
 * Intra-step region-aware cache control of the paper (Section 5.2; Appendix Algorithm 2): tiles
 * whose predicted noise has a high standard deviation (slowly updating regions) get a larger
 * threshold, so they skip more steps.  The paper leaves the tracker and the normalisation open;
 * here the tracker is, per tile, the running mean over the steps seen of the population standard
 * deviation of that step's tile output, Normalized() is min-max scaling across tiles (both
 * policies use only the order of the normalised values), and ties go to the lowest tile index. */
typedef enum { SG_REGION_MAXMIN = 0, SG_REGION_TOPSELECT = 1 } sg_region_mode;

/* tile_std[i] = sqrt(mean(x_i^2) - mean(x_i)^2) over the elems_per_tile elements of tile i.
 *   x          host array of n_tiles device pointers (16-byte aligned); elems_per_tile a multiple of 8
 *   tile_std   device, n_tiles floats (out);  workspace: as sg_cache_gate */
int sg_tile_std(const void* const* x, int32_t n_tiles, int64_t elems_per_tile, int32_t dtype, float* tile_std,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * StdTracker.Update with this step's tile_std, and, when `adjust` is non-zero (the caller sets it every
 * Delta steps), tau_i = tau_base * (1 + delta_i) with delta = 0 except
 *     SG_REGION_MAXMIN:    delta[argmax] = alpha, then delta[argmin] = -alpha/2
 *     SG_REGION_TOPSELECT: delta[largest] = alpha, delta[second largest] = alpha/2
 * over the tracked means.  The first call (track_count = 0) sets every threshold to tau_base if it
 * does not adjust; other calls without `adjust` leave the thresholds as they are.
 *   tile_std     device, n_tiles floats (in)
 *   track_mean   device, n_tiles doubles (in/out);  track_count: device, one int32 (in/out, start at 0)
 *   sigma        device, n_tiles floats (out, the normalised means; written only when adjusting) or NULL
 *   thresholds   device, n_tiles floats (in/out): what sg_gain_gate takes as tile_thresholds
 */
int sg_region_thresholds(const float* tile_std, double* track_mean, int32_t* track_count, int32_t n_tiles,
                         float tau_base, float alpha, int32_t mode, int32_t adjust, float* sigma,
                         float* thresholds, void* stream);

/* ------------------------------------------------------------------------------------------
 * One refinement step of stage 2 with everything the paper attaches to it, in one call and with
 * nothing read back (Algorithm 1 loop body with the cache of Section 5 and Algorithm 2's control):
 *     gate with per-tile thresholds -> attention of the tiles to recompute -> cache store update /
 *     residual reuse -> [StdTracker.Update and, when region->adjust, new thresholds] ->
 *     Fuse [-> scheduler update]
 * io        as for sg_denoise_step_gain; with `region` the gate reads region->thresholds (the
 *           values left by the previous call; on a tile's first two steps they are not consulted)
 * region    NULL, or Algorithm 2's state: see sg_tile_std / sg_region_thresholds for the fields
 * update    NULL: the fused prediction is written to io->grid_out.  Otherwise
 *           latent_out = c_latent * latent_in + c_noise * Fuse (sg_tile_blend_update) and
 *           io->grid_out is not used. */
typedef struct sg_region_control {
  double* track_mean;    /* device, n_tiles (in/out)                                    */
  int32_t* track_count;  /* device, one int32 (in/out, start at 0)                      */
  float* tile_std;       /* device, n_tiles (out): this step's standard deviations      */
  float* thresholds;     /* device, n_tiles (in/out): tau_i                             */
  float* sigma;          /* device, n_tiles (out when adjusting) or NULL                */
  float tau_base, alpha;
  int32_t mode;          /* sg_region_mode                                              */
  int32_t adjust;        /* non-zero on the steps where s mod Delta = 0                 */
} sg_region_control;

typedef struct sg_scheduler_update {
  const void* latent_in; /* device, canvas tensor                                       */
  void* latent_out;      /* device, canvas tensor; may be latent_in                     */
  float c_latent, c_noise;
} sg_scheduler_update;

int sg_refine_step(const sg_problem* p, const sg_gain_step_io* io, const sg_region_control* region,
                   const sg_scheduler_update* update, void* stream);

/* The whole loop body of Algorithm 1 from canvas tensors: Shift (the partition sits at
 * p->shift_h, p->shift_w, wrapping) and SliceTile of every tile, then sg_refine_step.
 *   q, k, v   device, canvas tensors (addressed through p's strides); read only
 *   tile_x    host array of n_tiles device pointers to WRITABLE buffers of
 *             3 * heads * T * tile_h * tile_w * head_dim elements: tile i's window of q, k and v is
 *             gathered into tile_x[i] before anything else; io->tile_x must name the same buffers
 *             (SG_ERR_INVALID_ARG otherwise) and io->prev_x the ones the previous call filled, so a
 *             caller alternates two sets of buffers.  Must not alias q, k, v or any output.
 * io, region, update, errors: as sg_refine_step. */
int sg_refine_step_canvas(const sg_problem* p, const void* q, const void* k, const void* v, void* const* tile_x,
                          const sg_gain_step_io* io, const sg_region_control* region,
                          const sg_scheduler_update* update, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SUPERGEN_TILE_H */
