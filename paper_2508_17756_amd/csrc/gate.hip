// Cache gate: relative L1 change of each tile's input against its cached input
// (paper Equation 3, cached tensor in the denominator) compared with the threshold
// (Equation 7: score >= threshold recomputes).
//
// Pure HBM streaming: each input element is read once.  Stage 1 runs one workgroup per compute
// unit; a thread sums |a-b| and |b| in fp32 over its 16-byte vectors, the workgroup adds its
// threads in fp64 and stores one (num, den) pair per tile.  Stage 2 adds the pairs of a tile in
// a fixed order in fp64, so the score is bit-reproducible run to run on a given device.
#include "sg_common.h"

namespace sg {
namespace {

constexpr int kThreads = 256;
constexpr int kFinalThreads = 128;
constexpr int kTilesPerLaunch = 64;

struct GatePtrs {
  const void* cur[kTilesPerLaunch];
  const void* cached[kTilesPerLaunch];
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ void accum_vec(const u32x4 a, const u32x4 b, float& num, float& den) {
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (DT == SG_BF16) {
      float a0 = bf16_bits_to_f32(a[c] & 0xffffu), a1 = __uint_as_float(a[c] & 0xffff0000u);
      float b0 = bf16_bits_to_f32(b[c] & 0xffffu), b1 = __uint_as_float(b[c] & 0xffff0000u);
      num += fabsf(a0 - b0) + fabsf(a1 - b1);
      den += fabsf(b0) + fabsf(b1);
    } else {
      float af = __uint_as_float(a[c]), bf = __uint_as_float(b[c]);
      num += fabsf(af - bf);
      den += fabsf(bf);
    }
  }
}

// One resident workgroup per compute unit walks the tiles of the launch one after the other; within a tile
// workgroup b streams the b-th of gridDim.x equal contiguous slabs of both buffers.  Every workgroup
// therefore carries the same load, no tail of late workgroups forms, and each buffer is read as
// gridDim.x long sequential streams.
template <int DT>
__global__ __launch_bounds__(kThreads) void gate_partial_kernel(GatePtrs ptrs, const uint8_t* __restrict__ has_cache,
                                                                int tile0, int n_tiles, int64_t elems,
                                                                double* __restrict__ partial) {
  constexpr int kPerVec = (DT == SG_BF16) ? 8 : 4;
  const int blk = blockIdx.x, n_blk = gridDim.x;
  const int64_t n_vec = elems / kPerVec;
  const int64_t per_blk = (n_vec + n_blk - 1) / n_blk;
  const int64_t v0 = (int64_t)blk * per_blk;
  const int64_t v1 = (v0 + per_blk < n_vec) ? v0 + per_blk : n_vec;
  __shared__ double s_num[2][kThreads / 64], s_den[2][kThreads / 64];
  for (int tile = 0; tile < n_tiles; ++tile) {
    double* out = partial + ((size_t)(tile0 + tile) * kGateSlots + blk) * 2;
    if (!has_cache[tile0 + tile]) {  // no cached input: nothing to compare, buffers are not read
      if (threadIdx.x == 0) { out[0] = 0.0; out[1] = 0.0; }
      continue;
    }
    const u32x4* __restrict__ a = (const u32x4*)ptrs.cur[tile];
    const u32x4* __restrict__ b = (const u32x4*)ptrs.cached[tile];
    float num0 = 0.f, den0 = 0.f, num1 = 0.f, den1 = 0.f;
    int64_t i = v0 + threadIdx.x;
    for (; i + 3 * kThreads < v1; i += 4 * kThreads) {
      u32x4 a0 = __builtin_nontemporal_load(a + i), b0 = __builtin_nontemporal_load(b + i);
      u32x4 a1 = __builtin_nontemporal_load(a + i + kThreads), b1 = __builtin_nontemporal_load(b + i + kThreads);
      u32x4 a2 = __builtin_nontemporal_load(a + i + 2 * kThreads), b2 = __builtin_nontemporal_load(b + i + 2 * kThreads);
      u32x4 a3 = __builtin_nontemporal_load(a + i + 3 * kThreads), b3 = __builtin_nontemporal_load(b + i + 3 * kThreads);
      accum_vec<DT>(a0, b0, num0, den0);
      accum_vec<DT>(a1, b1, num1, den1);
      accum_vec<DT>(a2, b2, num0, den0);
      accum_vec<DT>(a3, b3, num1, den1);
    }
    for (; i < v1; i += kThreads) accum_vec<DT>(__builtin_nontemporal_load(a + i), __builtin_nontemporal_load(b + i), num0, den0);
    double num = (double)num0 + (double)num1, den = (double)den0 + (double)den1;
    // ragged tail (elems not a multiple of the vector width): last workgroup, scalar
    if (blk == n_blk - 1) {
      for (int64_t e = n_vec * kPerVec + threadIdx.x; e < elems; e += kThreads) {
        float af, bf;
        if (DT == SG_BF16) {
          af = bf16_bits_to_f32(((const uint16_t*)ptrs.cur[tile])[e]);
          bf = bf16_bits_to_f32(((const uint16_t*)ptrs.cached[tile])[e]);
        } else {
          af = ((const float*)ptrs.cur[tile])[e];
          bf = ((const float*)ptrs.cached[tile])[e];
        }
        num += (double)fabsf(af - bf);
        den += (double)fabsf(bf);
      }
    }
    // fixed-order tree over the workgroup: wavefront shuffles, then one value per wavefront via LDS
    // (two LDS slots alternate between tiles, so one barrier per tile suffices)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      num += __shfl_down(num, off, 64);
      den += __shfl_down(den, off, 64);
    }
    const int par = tile & 1;
    if ((threadIdx.x & 63) == 0) { s_num[par][threadIdx.x >> 6] = num; s_den[par][threadIdx.x >> 6] = den; }
    __syncthreads();
    if (threadIdx.x == 0) {
      double n = 0.0, d = 0.0;
      for (int w = 0; w < kThreads / 64; ++w) { n += s_num[par][w]; d += s_den[par][w]; }
      out[0] = n;
      out[1] = d;
    }
  }
}

// Adds the `n_slots` workgroup partials of a tile in a fixed order and takes the decision.
__global__ __launch_bounds__(kFinalThreads) void gate_finalize_kernel(const double* __restrict__ partial, int n_slots,
                                                                     const uint8_t* __restrict__ has_cache, float threshold,
                                                                     float* __restrict__ scores, uint8_t* __restrict__ recompute) {
  const int tile = blockIdx.x;
  __shared__ double s_num[kFinalThreads], s_den[kFinalThreads];
  double n = 0.0, d = 0.0;
  for (int sl = threadIdx.x; sl < n_slots; sl += kFinalThreads) {
    n += partial[((size_t)tile * kGateSlots + sl) * 2];
    d += partial[((size_t)tile * kGateSlots + sl) * 2 + 1];
  }
  s_num[threadIdx.x] = n;
  s_den[threadIdx.x] = d;
  __syncthreads();
  for (int off = kFinalThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      s_num[threadIdx.x] += s_num[threadIdx.x + off];
      s_den[threadIdx.x] += s_den[threadIdx.x + off];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const bool cached = has_cache[tile] != 0;
    float score = __builtin_inff();
    if (cached && s_den[0] > 0.0) score = (float)(s_num[0] / s_den[0]);
    scores[tile] = score;
    recompute[tile] = (!cached || score >= threshold) ? 1 : 0;
  }
}

// cache_x[i] <- tile_x[i] for the tiles flagged for recomputation, has_cache[i] <- 1.
struct RefreshPtrs {
  const void* src[kTilesPerLaunch];
  void* dst[kTilesPerLaunch];
};
__global__ __launch_bounds__(kThreads) void cache_refresh_kernel(RefreshPtrs ptrs, const uint8_t* __restrict__ recompute,
                                                                 uint8_t* __restrict__ has_cache, int tile0, int64_t n_vec,
                                                                 int64_t tail_bytes) {
  const int tile = blockIdx.y;
  if (!recompute[tile0 + tile]) return;
  const u32x4* __restrict__ s = (const u32x4*)ptrs.src[tile];
  u32x4* __restrict__ d = (u32x4*)ptrs.dst[tile];
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n_vec; i += (int64_t)gridDim.x * kThreads)
    __builtin_nontemporal_store(__builtin_nontemporal_load(s + i), d + i);
  if (blockIdx.x == 0) {
    for (int64_t e = threadIdx.x; e < tail_bytes; e += kThreads)
      ((uint8_t*)ptrs.dst[tile])[n_vec * 16 + e] = ((const uint8_t*)ptrs.src[tile])[n_vec * 16 + e];
    if (threadIdx.x == 0) has_cache[tile0 + tile] = 1;
  }
}

}  // namespace

int launch_gate(const void* const* x_cur, const void* const* x_cached, const uint8_t* has_cache, int n_tiles,
                int64_t elems, int dtype, float threshold, float* scores, uint8_t* recompute, void* ws, hipStream_t s) {
  if (n_tiles == 0) return SG_OK;
  double* partial = (double*)ws;
  // one workgroup per compute unit; the partial-sum layout (and with it the summation order) depends only
  // on the device's compute-unit count
  int dev = 0, n_cu = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
  SG_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  const int n_blk = n_cu < 1 ? 1 : (n_cu > kGateSlots ? kGateSlots : n_cu);
  for (int t0 = 0; t0 < n_tiles; t0 += kTilesPerLaunch) {
    const int n = (n_tiles - t0 < kTilesPerLaunch) ? n_tiles - t0 : kTilesPerLaunch;
    GatePtrs ptrs;
    for (int i = 0; i < n; ++i) { ptrs.cur[i] = x_cur[t0 + i]; ptrs.cached[i] = x_cached[t0 + i]; }
    for (int i = n; i < kTilesPerLaunch; ++i) { ptrs.cur[i] = nullptr; ptrs.cached[i] = nullptr; }
    if (dtype == SG_BF16)
      gate_partial_kernel<SG_BF16><<<n_blk, kThreads, 0, s>>>(ptrs, has_cache, t0, n, elems, partial);
    else
      gate_partial_kernel<SG_F32><<<n_blk, kThreads, 0, s>>>(ptrs, has_cache, t0, n, elems, partial);
    SG_HIP_TRY(hipGetLastError());
  }
  gate_finalize_kernel<<<n_tiles, kFinalThreads, 0, s>>>(partial, n_blk, has_cache, threshold, scores, recompute);
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

int launch_cache_refresh(const void* const* src, void* const* dst, const uint8_t* recompute, uint8_t* has_cache,
                         int n_tiles, int64_t bytes_per_tile, hipStream_t s) {
  const int64_t n_vec = bytes_per_tile / 16;
  for (int t0 = 0; t0 < n_tiles; t0 += kTilesPerLaunch) {
    const int n = (n_tiles - t0 < kTilesPerLaunch) ? n_tiles - t0 : kTilesPerLaunch;
    RefreshPtrs ptrs;
    for (int i = 0; i < kTilesPerLaunch; ++i) { ptrs.src[i] = i < n ? src[t0 + i] : nullptr; ptrs.dst[i] = i < n ? dst[t0 + i] : nullptr; }
    dim3 grid(1024, n);   // grid-stride copy; 1024 workgroups per tile measured fastest for a plain copy
    cache_refresh_kernel<<<grid, kThreads, 0, s>>>(ptrs, recompute, has_cache, t0, n_vec, bytes_per_tile - n_vec * 16);
    SG_HIP_TRY(hipGetLastError());
  }
  return SG_OK;
}

}  // namespace sg
