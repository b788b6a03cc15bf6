// Internal declarations shared by the HIP translation units of libsupergen_tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "supergen_tile.h"

namespace sg {

// Records a failed HIP call for sg_last_hip_error() and maps it to SG_ERR_HIP.
int note_hip_error(hipError_t e);
#define SG_HIP_TRY(expr)                                  \
  do {                                                    \
    hipError_t sg_e_ = (expr);                            \
    if (sg_e_ != hipSuccess) return sg::note_hip_error(sg_e_); \
  } while (0)

// Shape and canvas addressing shared by the tiles of one attention call, in elements, resolved on the host.
struct TileView {
  int64_t stride_token;  // elements between canvas tokens
  int64_t stride_head;
  int32_t T, H, W;       // canvas
  int32_t th, tw;        // tile
  int32_t N;             // T*th*tw tokens
  bool wrapped;          // shifted partition: windows wrap around the canvas edges
};

// The tiles of one attention call.  For a fixed partition q[i], k[i], v[i] point at tile i's first token
// (the tile origin is folded into the pointer); for wrapped windows they are the canvas tensors and
// (y0[i], x0[i]) is the canvas position of tile i's first token.
struct AttnBatch {
  int n_tiles;
  const void* const* q;      // host arrays of n_tiles device pointers
  const void* const* k;
  const void* const* v;
  void* const* out;          // packed tile outputs
  const int32_t* y0;         // host arrays, wrapped windows only (else nullptr)
  const int32_t* x0;
  const uint8_t* run_flags;  // device, n_tiles bytes: tiles with a 0 are skipped; nullptr = all tiles run
  // Cache refresh of the tiled step, carried out by the same launch where the kernel supports it (*refreshed is
  // then set): for every tile that runs, refresh_dst[i] <- the refresh_bytes at q[i] (a packed tile input: Q, K, V
  // one after the other) and has_cache[i] <- 1.  All nullptr / 0 when no refresh is asked for.
  void* const* refresh_dst;  // host array of n_tiles device pointers
  uint8_t* has_cache;        // device, n_tiles bytes
  int64_t refresh_bytes;     // a multiple of 16
  bool* refreshed;           // host, out
};

// Launchers (each validates nothing: the API layer has already done so).
int launch_attention_f32(const TileView& tv, int heads, int head_dim, float scale, const AttnBatch& b, hipStream_t s);
int launch_attention_bf16(const TileView& tv, int heads, int head_dim, float scale, const AttnBatch& b, hipStream_t s);
int launch_attention_bf16_generic(const TileView& tv, int heads, int head_dim, float scale, const AttnBatch& b,
                                  hipStream_t s);
int launch_blend(const sg_problem& p, const void* const* tile_out, void* grid_out, const void* latent, float c_latent,
                 float c_noise, hipStream_t s);
int launch_slice(const sg_problem& p, const void* const* src, int n_src, int tile_row, int tile_col, void* dst,
                 hipStream_t s);
int launch_gate(const void* const* x_cur, const void* const* x_cached, const uint8_t* has_cache,
                int n_tiles, int64_t elems, int dtype, float threshold, float* scores,
                uint8_t* recompute, void* ws, hipStream_t s);
int launch_gain_gate(const void* const* x_cur, const void* const* x_prev, const sg_gain_state& gs, int n_tiles,
                     int64_t elems, int dtype, float threshold, const float* tile_thresholds, float* step_change,
                     float* scores, uint8_t* recompute, void* ws, hipStream_t s);
int launch_gain_refresh(void* const* out_cur, const void* const* out_prev, const void* const* latent,
                        float* const* delta, const uint8_t* recompute, const float* step_change,
                        const sg_gain_state& gs, int n_tiles, int64_t elems, int dtype, void* ws, hipStream_t s);
int launch_tile_std(const void* const* x, int n_tiles, int64_t elems, int dtype, float* tile_std, void* ws, hipStream_t s);
int launch_similarity(const void* const* x_new, const void* const* x_old, int n_tiles, int64_t elems, int dtype,
                      float* l1_rel, float* cos_sim, void* ws, hipStream_t s);
int launch_region_thresholds(const float* tile_std, double* track_mean, int32_t* track_count, int n_tiles,
                             float tau_base, float alpha, int mode, int adjust, float* sigma, float* thresholds,
                             hipStream_t s);
int launch_cache_refresh(const void* const* src, void* const* dst, const uint8_t* recompute,
                         uint8_t* has_cache, int n_tiles, int64_t bytes_per_tile, hipStream_t s);

// Gate scratch: per tile kGateSlots (num, den) fp64 pairs, one per workgroup of the partial-sum kernel.
constexpr int kGateSlots = 1024;
inline size_t gate_workspace_bytes(int n_tiles) {
  return (size_t)(n_tiles > 0 ? n_tiles : 1) * kGateSlots * 2 * sizeof(double);
}

// bf16 <-> fp32 on the device.
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {  // round to nearest even
  __bf16 b = (__bf16)f;
  return (uint32_t)__builtin_bit_cast(unsigned short, b);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

}  // namespace sg
