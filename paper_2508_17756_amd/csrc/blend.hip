// Fuse / overlap blend of tile outputs into the canvas (paper Algorithm 1 "Fuse", Section 4.2).
//
// Gather form of the weighted scatter-accumulate-and-normalise: every canvas element pulls the
// contributions of the tiles that cover it, with the separable ramp weights recomputed
// analytically, and divides by the weight sum.  No accumulator or weight buffers, no atomics:
// each tile-output element is read once and each canvas element written once, which is the
// algorithmic HBM traffic.  One thread owns one 16-byte vector position of the canvas.
#include "sg_common.h"

namespace sg {
namespace {

constexpr int kThreads = 256;

struct BlendArgs {
  const void* tile[SG_MAX_TILES];
  int32_t T, H, W, th, tw, sh, sw, n_rows, n_cols, heads, d;
  int32_t vec_per_token_log2;  // log2(d / elements per 16-byte vector)
  int32_t shift_h, shift_w;    // partition offset on the canvas, wrapping
  float inv_oh1, inv_ow1;      // 1/(o+1) per axis
  float c_latent, c_noise;     // scheduler update: out = c_latent * latent + c_noise * fused
  const void* latent;          // canvas tensor read by the update (may be the output itself)
  int64_t stride_token, stride_head;
  uint32_t plane_vecs;         // H*W*vec_per_token
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float ramp(int i, int L, float inv_o1) {
  // min(1, (i+1)/(o+1), (L-i)/(o+1))
  return fminf(1.0f, fminf((float)(i + 1) * inv_o1, (float)(L - i) * inv_o1));
}

template <int DT>
__device__ __forceinline__ void fma_vec(const u32x4 val, const float w, float (&acc)[8]) {
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (DT == SG_BF16) {
      acc[2 * c] += w * bf16_bits_to_f32(val[c] & 0xffffu);
      acc[2 * c + 1] += w * __uint_as_float(val[c] & 0xffff0000u);
    } else {
      acc[c] += w * __uint_as_float(val[c]);
    }
  }
}
template <int DT>
__device__ __forceinline__ u32x4 pack_vec(const float (&acc)[8], const float inv) {
  u32x4 o;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (DT == SG_BF16) o[c] = pack_bf16x2(acc[2 * c] * inv, acc[2 * c + 1] * inv);
    else o[c] = __float_as_uint(acc[c] * inv);
  }
  return o;
}
// scheduler update on the fused value: c_latent * latent + c_noise * (acc * inv), one rounding
template <int DT>
__device__ __forceinline__ u32x4 pack_update(const float (&acc)[8], const float inv, const u32x4 lat, const float cl,
                                             const float cn) {
  u32x4 o;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (DT == SG_BF16)
      o[c] = pack_bf16x2(cl * bf16_bits_to_f32(lat[c] & 0xffffu) + cn * (acc[2 * c] * inv),
                         cl * __uint_as_float(lat[c] & 0xffff0000u) + cn * (acc[2 * c + 1] * inv));
    else
      o[c] = __float_as_uint(cl * __uint_as_float(lat[c]) + cn * (acc[c] * inv));
  }
  return o;
}

// A thread owns one 16-byte vector position (y, x, channel group) of the canvas plane and produces it for
// kPlanes consecutive (head, frame) planes: the covering tiles, their weights and the reciprocal weight sum
// depend on (y, x) only and are worked out once, and the loads of all planes are in flight together.
// RC x CC = the largest number of tiles that can cover a token (rows x columns); every candidate has a
// fixed register slot, absent ones carry weight 0 and are not loaded.
constexpr int kPlanes = 2;

template <int DT, int RC, int CC, bool UPD>
__global__ __launch_bounds__(kThreads) void blend_kernel(const BlendArgs a, void* grid_out) {
  constexpr int kPerVec = (DT == SG_BF16) ? 8 : 4;
  const uint32_t v = blockIdx.x * kThreads + threadIdx.x;  // vector inside one (head, frame) plane
  if (v >= a.plane_vecs) return;
  const uint32_t token = v >> a.vec_per_token_log2;
  const int cv = v & ((1u << a.vec_per_token_log2) - 1);
  const int yc = token / (uint32_t)a.W, xc = token - yc * a.W;   // canvas position written
  // position in the unshifted partition (the partition sits at (shift_h, shift_w) on the canvas, wrapping)
  int y = yc - a.shift_h; if (y < 0) y += a.H;
  int x = xc - a.shift_w; if (x < 0) x += a.W;

  // tiles covering row y: tr*sh <= y < tr*sh + th, i.e. tr in [ceil((y-th+1)/sh), floor(y/sh)]
  int tr_hi = y / a.sh; if (tr_hi > a.n_rows - 1) tr_hi = a.n_rows - 1;
  int tr_lo = (y - a.th + a.sh) / a.sh; if (y - a.th + a.sh < 0) tr_lo = 0;
  int tc_hi = x / a.sw; if (tc_hi > a.n_cols - 1) tc_hi = a.n_cols - 1;
  int tc_lo = (x - a.tw + a.sw) / a.sw; if (x - a.tw + a.sw < 0) tc_lo = 0;

  const u32x4* src[RC * CC];
  float w[RC * CC];
  float wsum = 0.f;
#pragma unroll
  for (int ir = 0; ir < RC; ++ir) {
    const int tr = tr_lo + ir;
    const int i = y - tr * a.sh;
    const float wh = (tr <= tr_hi) ? ramp(i, a.th, a.inv_oh1) : 0.f;
#pragma unroll
    for (int ic = 0; ic < CC; ++ic) {
      const int tc = tc_lo + ic;
      const int j = x - tc * a.sw;
      const bool on = (tr <= tr_hi) && (tc <= tc_hi);
      w[ir * CC + ic] = on ? wh * ramp(j, a.tw, a.inv_ow1) : 0.f;
      wsum += w[ir * CC + ic];
      src[ir * CC + ic] = on ? (const u32x4*)a.tile[tr * a.n_cols + tc] + ((((int64_t)i * a.tw + j) << a.vec_per_token_log2) + cv)
                             : nullptr;
    }
  }
  const float inv = 1.0f / wsum;
  const int64_t tile_plane_vecs = ((int64_t)a.th * a.tw) << a.vec_per_token_log2;
  const int plane0 = blockIdx.y * kPlanes, n_planes = a.heads * a.T;

  float acc[kPlanes][8];
#pragma unroll
  for (int pl = 0; pl < kPlanes; ++pl)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[pl][c] = 0.f;
#pragma unroll
  for (int k = 0; k < RC * CC; ++k) {
    if (w[k] != 0.f) {
      u32x4 val[kPlanes];
#pragma unroll
      for (int pl = 0; pl < kPlanes; ++pl)
        val[pl] = (plane0 + pl < n_planes) ? __builtin_nontemporal_load(src[k] + (int64_t)(plane0 + pl) * tile_plane_vecs)
                                           : u32x4{0, 0, 0, 0};
#pragma unroll
      for (int pl = 0; pl < kPlanes; ++pl) fma_vec<DT>(val[pl], w[k], acc[pl]);
    }
  }
#pragma unroll
  for (int pl = 0; pl < kPlanes; ++pl) {
    const int plane = plane0 + pl;  // head * T + t
    if (plane < n_planes) {
      const int head = plane / a.T, t = plane - head * a.T;
      const int64_t n = ((int64_t)t * a.H + yc) * a.W + xc;
      const int64_t off = (int64_t)head * a.stride_head + n * a.stride_token + (int64_t)cv * kPerVec;
      u32x4* dst = (u32x4*)((char*)grid_out + off * (DT == SG_BF16 ? 2 : 4));
      if (UPD) {
        const u32x4 lat = __builtin_nontemporal_load((const u32x4*)((const char*)a.latent + off * (DT == SG_BF16 ? 2 : 4)));
        __builtin_nontemporal_store(pack_update<DT>(acc[pl], inv, lat, a.c_latent, a.c_noise), dst);
      } else {
        __builtin_nontemporal_store(pack_vec<DT>(acc[pl], inv), dst);
      }
    }
  }
}

// Any coverage: the same computation with loops over the covering tiles, one plane per thread.
template <int DT, bool UPD>
__global__ __launch_bounds__(kThreads) void blend_any_kernel(const BlendArgs a, void* grid_out) {
  constexpr int kPerVec = (DT == SG_BF16) ? 8 : 4;
  const uint32_t v = blockIdx.x * kThreads + threadIdx.x;
  if (v >= a.plane_vecs) return;
  const int plane = blockIdx.y;  // head * T + t
  const int head = plane / a.T, t = plane - head * a.T;
  const uint32_t token = v >> a.vec_per_token_log2;
  const int cv = v & ((1u << a.vec_per_token_log2) - 1);
  const int yc = token / (uint32_t)a.W, xc = token - yc * a.W;
  int y = yc - a.shift_h; if (y < 0) y += a.H;
  int x = xc - a.shift_w; if (x < 0) x += a.W;
  int tr_hi = y / a.sh; if (tr_hi > a.n_rows - 1) tr_hi = a.n_rows - 1;
  int tr_lo = (y - a.th + a.sh) / a.sh; if (y - a.th + a.sh < 0) tr_lo = 0;
  int tc_hi = x / a.sw; if (tc_hi > a.n_cols - 1) tc_hi = a.n_cols - 1;
  int tc_lo = (x - a.tw + a.sw) / a.sw; if (x - a.tw + a.sw < 0) tc_lo = 0;
  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.f;
  float wsum = 0.f;
  for (int tr = tr_lo; tr <= tr_hi; ++tr) {
    const int i = y - tr * a.sh;
    const float wh = ramp(i, a.th, a.inv_oh1);
    for (int tc = tc_lo; tc <= tc_hi; ++tc) {
      const int j = x - tc * a.sw;
      const float w = wh * ramp(j, a.tw, a.inv_ow1);
      const int64_t tok = ((int64_t)(plane * a.th + i)) * a.tw + j;  // packed tile token index incl. head
      const u32x4* src = (const u32x4*)a.tile[tr * a.n_cols + tc] + ((tok << a.vec_per_token_log2) + cv);
      wsum += w;
      fma_vec<DT>(__builtin_nontemporal_load(src), w, acc);
    }
  }
  const int64_t n = ((int64_t)t * a.H + yc) * a.W + xc;
  const int64_t off = (int64_t)head * a.stride_head + n * a.stride_token + (int64_t)cv * kPerVec;
  u32x4* dst = (u32x4*)((char*)grid_out + off * (DT == SG_BF16 ? 2 : 4));
  if (UPD) {
    const u32x4 lat = __builtin_nontemporal_load((const u32x4*)((const char*)a.latent + off * (DT == SG_BF16 ? 2 : 4)));
    __builtin_nontemporal_store(pack_update<DT>(acc, 1.0f / wsum, lat, a.c_latent, a.c_noise), dst);
  } else {
    __builtin_nontemporal_store(pack_vec<DT>(acc, 1.0f / wsum), dst);
  }
}

// SliceTile under a (possibly shifted, wrapping) partition: gathers the window of tile (tile_row, tile_col)
// out of up to three canvas tensors into one packed buffer [n_src][heads][T][tile_h][tile_w][d].  A plain
// copy, one 16-byte vector per thread, the packed side fully coalesced.
struct SliceArgs {
  const void* src[3];
  int32_t n_src, T, H, W, th, tw, r0, c0;     // r0, c0: canvas position of the tile's token (0, 0), before wrapping
  int32_t vec_per_token_log2;
  int64_t stride_token, stride_head;          // canvas strides in elements
  int32_t elem_bytes;
  uint32_t tile_plane_vecs;                   // th * tw * vectors per token
  int32_t heads;
};
__global__ __launch_bounds__(kThreads) void slice_kernel(const SliceArgs a, u32x4* __restrict__ dst) {
  const uint32_t v = blockIdx.x * kThreads + threadIdx.x;
  if (v >= a.tile_plane_vecs) return;
  const int plane = blockIdx.y;                 // head * T + t
  const int which = blockIdx.z;
  const int head = plane / a.T, t = plane - head * a.T;
  const uint32_t token = v >> a.vec_per_token_log2;
  const int cv = v & ((1u << a.vec_per_token_log2) - 1);
  const int i = token / (uint32_t)a.tw, j = token - i * a.tw;
  int y = a.r0 + i; if (y >= a.H) y -= a.H;
  int x = a.c0 + j; if (x >= a.W) x -= a.W;
  const int64_t n = ((int64_t)t * a.H + y) * a.W + x;
  const int64_t off_bytes = ((int64_t)head * a.stride_head + n * a.stride_token) * a.elem_bytes + (int64_t)cv * 16;
  const u32x4 val = __builtin_nontemporal_load((const u32x4*)((const char*)a.src[which] + off_bytes));
  const int64_t planes = (int64_t)a.heads * a.T;
  __builtin_nontemporal_store(val, dst + ((int64_t)which * planes + plane) * a.tile_plane_vecs + v);
}

}  // namespace

template <int DT, bool UPD>
static void launch_blend_cover(const BlendArgs& a, void* grid_out, int rc, int cc, dim3 grid_pl, dim3 grid_any, hipStream_t s) {
  if (rc <= 1 && cc <= 1) blend_kernel<DT, 1, 1, UPD><<<grid_pl, kThreads, 0, s>>>(a, grid_out);
  else if (rc <= 2 && cc <= 2) blend_kernel<DT, 2, 2, UPD><<<grid_pl, kThreads, 0, s>>>(a, grid_out);
  else if (rc <= 3 && cc <= 3) blend_kernel<DT, 3, 3, UPD><<<grid_pl, kThreads, 0, s>>>(a, grid_out);
  else blend_any_kernel<DT, UPD><<<grid_any, kThreads, 0, s>>>(a, grid_out);
}

// latent == nullptr: plain Fuse; otherwise grid_out = c_latent * latent + c_noise * Fuse
int launch_blend(const sg_problem& p, const void* const* tile_out, void* grid_out, const void* latent, float c_latent,
                 float c_noise, hipStream_t s) {
  BlendArgs a;
  const int n_tiles = p.n_tile_rows * p.n_tile_cols;
  for (int i = 0; i < SG_MAX_TILES; ++i) a.tile[i] = i < n_tiles ? tile_out[i] : nullptr;
  a.T = p.T; a.H = p.H; a.W = p.W; a.th = p.tile_h; a.tw = p.tile_w; a.sh = p.stride_h; a.sw = p.stride_w;
  a.n_rows = p.n_tile_rows; a.n_cols = p.n_tile_cols; a.heads = p.heads; a.d = p.head_dim;
  a.shift_h = p.shift_h; a.shift_w = p.shift_w;
  a.latent = latent; a.c_latent = c_latent; a.c_noise = c_noise;
  const int per_vec = (p.dtype == SG_BF16) ? 8 : 4;
  const int vpt = p.head_dim / per_vec;
  int lg = 0; while ((1 << lg) < vpt) ++lg;
  a.vec_per_token_log2 = lg;
  a.inv_oh1 = 1.0f / (float)(p.tile_h - p.stride_h + 1);
  a.inv_ow1 = 1.0f / (float)(p.tile_w - p.stride_w + 1);
  a.stride_token = p.grid_stride_token; a.stride_head = p.grid_stride_head;
  a.plane_vecs = (uint32_t)((int64_t)p.H * p.W * vpt);
  const uint32_t gx = (a.plane_vecs + kThreads - 1) / kThreads;
  const int n_planes = p.heads * p.T;
  // most tiles that can cover one token, per axis
  const int rc = (p.tile_h + p.stride_h - 1) / p.stride_h, cc = (p.tile_w + p.stride_w - 1) / p.stride_w;
  const dim3 grid_pl(gx, (n_planes + kPlanes - 1) / kPlanes), grid_any(gx, n_planes);
  const bool bf = p.dtype == SG_BF16;
  if (latent) {
    if (bf) launch_blend_cover<SG_BF16, true>(a, grid_out, rc, cc, grid_pl, grid_any, s);
    else launch_blend_cover<SG_F32, true>(a, grid_out, rc, cc, grid_pl, grid_any, s);
  } else {
    if (bf) launch_blend_cover<SG_BF16, false>(a, grid_out, rc, cc, grid_pl, grid_any, s);
    else launch_blend_cover<SG_F32, false>(a, grid_out, rc, cc, grid_pl, grid_any, s);
  }
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

int launch_slice(const sg_problem& p, const void* const* src, int n_src, int tile_row, int tile_col, void* dst,
                 hipStream_t s) {
  SliceArgs a;
  for (int i = 0; i < 3; ++i) a.src[i] = i < n_src ? src[i] : nullptr;
  a.n_src = n_src; a.T = p.T; a.H = p.H; a.W = p.W; a.th = p.tile_h; a.tw = p.tile_w; a.heads = p.heads;
  a.r0 = (tile_row * p.stride_h + p.shift_h) % p.H;
  a.c0 = (tile_col * p.stride_w + p.shift_w) % p.W;
  a.elem_bytes = (p.dtype == SG_BF16) ? 2 : 4;
  const int vpt = p.head_dim * a.elem_bytes / 16;
  int lg = 0; while ((1 << lg) < vpt) ++lg;
  a.vec_per_token_log2 = lg;
  a.stride_token = p.grid_stride_token; a.stride_head = p.grid_stride_head;
  a.tile_plane_vecs = (uint32_t)((int64_t)p.tile_h * p.tile_w * vpt);
  dim3 grid((a.tile_plane_vecs + kThreads - 1) / kThreads, p.heads * p.T, n_src);
  slice_kernel<<<grid, kThreads, 0, s>>>(a, (u32x4*)dst);
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

}  // namespace sg
