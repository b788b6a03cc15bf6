// Shared by the tile-attention kernels (paper Sections 2.1 and 3; Algorithm 1 "SliceTile" / "Shift"):
// the table of tiles one launch works on, the mapping of workgroups to (tile, head, query block) that skips
// reused tiles on the device, and the addressing of a tile's tokens inside a canvas tensor.
#pragma once
#include "sg_common.h"

namespace sg {

// vector types of the bf16 matrix-core kernels
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#define SG_LDS __attribute__((address_space(3)))

// ---------------------------------------------------------------------------------------------------
// One launch attends up to kAttnTilesPerLaunch tiles of the same shape (Algorithm 1: for all tiles of the
// partition).  Per tile the table holds the tensors its offsets are relative to, the packed output and,
// for a shifted (wrapping) partition, the canvas position of its first token.
constexpr int kAttnTilesPerLaunch = 32;
struct AttnTable {
  const void* q[kAttnTilesPerLaunch];
  const void* k[kAttnTilesPerLaunch];
  const void* v[kAttnTilesPerLaunch];
  void* out[kAttnTilesPerLaunch];
  int32_t y0[kAttnTilesPerLaunch], x0[kAttnTilesPerLaunch];   // wrapped windows only
  void* refresh[kAttnTilesPerLaunch];   // cache refresh fused into the launch (packed tiles): copy of the tile's input, or unused
};

// Tiles whose run flag is 0 (the cache gate reuses them) are skipped on the device: the workgroups number
// only the work of the active tiles, so that work is spread evenly whichever tiles run, and the rest of the
// grid exits at once.  Returns the 32-bit mask of active tiles among the launch's n_tiles.
__device__ __forceinline__ uint32_t attn_active_mask(const uint8_t* __restrict__ run_flags, int n_tiles) {
  const int lane = threadIdx.x & 63;
  if (!run_flags) return n_tiles >= 32 ? 0xffffffffu : ((1u << n_tiles) - 1u);
  const bool on = lane < n_tiles && run_flags[lane] != 0;
  return (uint32_t)__ballot(on);
}
// index of the a-th set bit of mask (a < popcount(mask))
__device__ __forceinline__ int attn_nth_tile(uint32_t mask, int a) {
  for (int i = 0; i < a; ++i) mask &= mask - 1;
  return __builtin_ctz(mask);
}

// ---------------------------------------------------------------------------------------------------
// Tile addressing on the device in units of 16 bytes, so that offsets inside one head fit 32 bits.
// Offsets are relative to the tile's table pointers: the host folds the tile origin of a fixed partition
// into them; a wrapped window keeps the canvas pointers and carries its origin in the table.
struct View16 {
  uint32_t st16;          // 16-byte units per canvas token
  uint32_t row_skip16;    // (W - tw) * st16: jump at the end of a tile row
  uint32_t frame_skip16;  // (H - th) * W * st16: jump at the end of a tile frame
  int32_t th, tw, N;
  uint32_t head16;        // 16-byte units per head
  int32_t H, W;           // canvas size: used by wrapped windows only
};

struct RowCursor {  // a tile token (i, j of the current frame) and its offset
  int32_t i, j;
  uint32_t off16;
};

__device__ __forceinline__ RowCursor cursor_at(const View16& vw, int n) {
  const int plane = vw.th * vw.tw;
  const int t = n / plane, r = n - t * plane;
  RowCursor c;
  c.i = r / vw.tw;
  c.j = r - c.i * vw.tw;
  // canvas token index = (t*H + i)*W + j = n + (t*th + i)*(W - tw) + t*(H - th)*W
  c.off16 = (uint32_t)n * vw.st16 + (uint32_t)(t * vw.th + c.i) * vw.row_skip16 + (uint32_t)t * vw.frame_skip16;
  return c;
}
__device__ __forceinline__ void cursor_advance(const View16& vw, RowCursor& c, int step) {
  c.j += step;
  c.off16 += (uint32_t)step * vw.st16;
  while (c.j >= vw.tw) {
    c.j -= vw.tw;
    c.off16 += vw.row_skip16;
    if (++c.i == vw.th) { c.i = 0; c.off16 += vw.frame_skip16; }
  }
}

// Wrapped window of a shifted partition (Algorithm 1 "Shift"): tile token (t, i, j) sits at canvas row
// (y0 + i) mod H, column (x0 + j) mod W, so a tile row may consist of two runs and the offset is formed
// from the coordinates each time.
struct WrapCursor {
  int32_t t, i, j;
};
__device__ __forceinline__ WrapCursor wrap_cursor_at(const View16& vw, int n) {
  const int plane = vw.th * vw.tw;
  WrapCursor c;
  c.t = n / plane;
  const int r = n - c.t * plane;
  c.i = r / vw.tw;
  c.j = r - c.i * vw.tw;
  return c;
}
__device__ __forceinline__ void wrap_cursor_advance(const View16& vw, WrapCursor& c, int step) {
  c.j += step;
  while (c.j >= vw.tw) {
    c.j -= vw.tw;
    if (++c.i == vw.th) { c.i = 0; ++c.t; }
  }
}
__device__ __forceinline__ uint32_t wrap_offset16(const View16& vw, const WrapCursor& c, int y0, int x0) {
  int y = y0 + c.i, x = x0 + c.j;
  y -= (y >= vw.H) ? vw.H : 0;
  x -= (x >= vw.W) ? vw.W : 0;
  return (uint32_t)((c.t * vw.H + y) * vw.W + x) * vw.st16;
}

// Host side: the device view of a tile shape.
inline View16 make_view16(const TileView& tv) {
  View16 vw;
  vw.st16 = (uint32_t)(tv.stride_token / 8);
  vw.row_skip16 = (uint32_t)(tv.W - tv.tw) * vw.st16;
  vw.frame_skip16 = (uint32_t)((int64_t)(tv.H - tv.th) * tv.W) * vw.st16;
  vw.th = tv.th; vw.tw = tv.tw; vw.N = tv.N;
  vw.head16 = (uint32_t)(tv.stride_head / 8);
  vw.H = tv.H; vw.W = tv.W;
  return vw;
}

}  // namespace sg
