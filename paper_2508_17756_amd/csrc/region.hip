// Intra-step region-aware cache control (paper Section 5.2; Appendix Algorithm 2): the standard
// deviation of each tile's predicted noise, an online tracker of it, and every Delta steps the
// per-tile thresholds tau_i = tau_base * (1 + delta_i) of the "MaxMin" or "TopSelect" policy.
//
// The standard deviation is one streaming read of the tile outputs (HBM-bound, same layout as the
// cache gate: one resident workgroup per compute unit, equal contiguous slabs per tile); the
// tracker and the policy are a few operations per tile and run in a single workgroup, so that
// nothing has to be read back between the steps.
#include "sg_common.h"

namespace sg {
namespace {

constexpr int kThreads = 256;
constexpr int kFinalThreads = 128;
constexpr int kTilesPerLaunch = 64;
constexpr int kMomentsUnroll = 16;   // 16-byte loads in flight per thread: 64 KiB per compute unit (8: 6.6 TB/s, 16: 7.0, 24: 6.9, 32: 6.6)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct StdPtrs { const void* x[kTilesPerLaunch]; };

template <int DT>
__device__ __forceinline__ void moments_vec(const u32x4 a, const float pivot, float& s1, float& s2) {
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (DT == SG_BF16) {
      const float x0 = bf16_bits_to_f32(a[c] & 0xffffu) - pivot, x1 = __uint_as_float(a[c] & 0xffff0000u) - pivot;
      s1 += x0 + x1;
      s2 += x0 * x0 + x1 * x1;
    } else {
      const float x0 = __uint_as_float(a[c]) - pivot;
      s1 += x0;
      s2 += x0 * x0;
    }
  }
}

// Sums of (x - pivot) and (x - pivot)^2 per tile and workgroup; pivot = the tile's first element, which
// keeps the variance free of cancellation when the mean is large against the spread.
template <int DT>
__global__ __launch_bounds__(kThreads) void tile_moments_kernel(StdPtrs ptrs, int tile0, int n_tiles, int64_t elems,
                                                                double* __restrict__ partial) {
  constexpr int kPerVec = (DT == SG_BF16) ? 8 : 4;
  const int blk = blockIdx.x, n_blk = gridDim.x;
  const int64_t n_vec = elems / kPerVec;
  const int64_t per_blk = (n_vec + n_blk - 1) / n_blk;
  const int64_t v0 = (int64_t)blk * per_blk;
  const int64_t v1 = (v0 + per_blk < n_vec) ? v0 + per_blk : n_vec;
  for (int tile = 0; tile < n_tiles; ++tile) {
    const u32x4* __restrict__ x = (const u32x4*)ptrs.x[tile];
    float pivot;
    if (DT == SG_BF16) pivot = bf16_bits_to_f32(((const uint16_t*)ptrs.x[tile])[0]);
    else pivot = ((const float*)ptrs.x[tile])[0];
    float a0 = 0.f, b0 = 0.f, a1 = 0.f, b1 = 0.f;
    int64_t i = v0 + threadIdx.x;
    for (; i + (kMomentsUnroll - 1) * kThreads < v1; i += kMomentsUnroll * kThreads) {
      u32x4 xv[kMomentsUnroll];
#pragma unroll
      for (int u = 0; u < kMomentsUnroll; ++u) xv[u] = __builtin_nontemporal_load(x + i + u * kThreads);
#pragma unroll
      for (int u = 0; u < kMomentsUnroll; u += 2) {
        moments_vec<DT>(xv[u], pivot, a0, b0);
        moments_vec<DT>(xv[u + 1], pivot, a1, b1);
      }
    }
    for (; i < v1; i += kThreads) moments_vec<DT>(__builtin_nontemporal_load(x + i), pivot, a0, b0);
    double s1 = (double)a0 + (double)a1, s2 = (double)b0 + (double)b1;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      s1 += __shfl_down(s1, off, 64);
      s2 += __shfl_down(s2, off, 64);
    }
    // one partial pair per wavefront: no workgroup barrier between tiles
    if ((threadIdx.x & 63) == 0) {
      double* out = partial + ((size_t)(tile0 + tile) * kGateSlots + blk * (kThreads / 64) + (threadIdx.x >> 6)) * 2;
      out[0] = s1;
      out[1] = s2;
    }
  }
}

__global__ __launch_bounds__(kFinalThreads) void tile_std_finalize_kernel(const double* __restrict__ partial, int n_slots,
                                                                          int64_t elems, float* __restrict__ tile_std) {
  const int tile = blockIdx.x;
  __shared__ double s_a[kFinalThreads], s_b[kFinalThreads];
  double a = 0.0, b = 0.0;
  for (int sl = threadIdx.x; sl < n_slots; sl += kFinalThreads) {
    a += partial[((size_t)tile * kGateSlots + sl) * 2];
    b += partial[((size_t)tile * kGateSlots + sl) * 2 + 1];
  }
  s_a[threadIdx.x] = a;
  s_b[threadIdx.x] = b;
  __syncthreads();
  for (int off = kFinalThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      s_a[threadIdx.x] += s_a[threadIdx.x + off];
      s_b[threadIdx.x] += s_b[threadIdx.x + off];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double m = s_a[0] / (double)elems;
    const double var = s_b[0] / (double)elems - m * m;
    tile_std[tile] = (float)sqrt(var > 0.0 ? var : 0.0);
  }
}

// StdTracker.Update, and when `adjust` is set StdTracker.Normalized and the policy.  One workgroup.
// Ties go to the lowest tile index; with "MaxMin" the minimum is assigned after the maximum.
__global__ __launch_bounds__(kThreads) void region_threshold_kernel(const float* __restrict__ tile_std,
                                                                    double* __restrict__ track_mean,
                                                                    int32_t* __restrict__ track_count, int n_tiles,
                                                                    float tau_base, float alpha, int mode, int adjust,
                                                                    float* __restrict__ sigma, float* __restrict__ thresholds) {
  const int count = *track_count + 1;
  for (int i = threadIdx.x; i < n_tiles; i += kThreads) {
    const double m = (count == 1) ? 0.0 : track_mean[i];
    track_mean[i] = m + ((double)tile_std[i] - m) / (double)count;
    if (count == 1 && !adjust) thresholds[i] = tau_base;   // the thresholds start at tau_base
  }
  __syncthreads();
  if (threadIdx.x == 0) *track_count = count;
  if (!adjust) return;
  __shared__ int s_sel[2];
  __shared__ double s_lo, s_hi;
  if (threadIdx.x == 0) {
    int i_max = 0, i_min = 0, i_second = -1;
    for (int i = 1; i < n_tiles; ++i) {
      if (track_mean[i] > track_mean[i_max]) i_max = i;
      if (track_mean[i] < track_mean[i_min]) i_min = i;
    }
    for (int i = 0; i < n_tiles; ++i)
      if (i != i_max && (i_second < 0 || track_mean[i] > track_mean[i_second])) i_second = i;
    s_sel[0] = i_max;
    s_sel[1] = (mode == SG_REGION_MAXMIN) ? i_min : i_second;
    s_lo = track_mean[i_min];
    s_hi = track_mean[i_max];
  }
  __syncthreads();
  const double lo = s_lo, hi = s_hi;
  for (int i = threadIdx.x; i < n_tiles; i += kThreads) {
    float delta = 0.f;
    if (i == s_sel[0]) delta = alpha;
    if (i == s_sel[1]) delta = (mode == SG_REGION_MAXMIN) ? -0.5f * alpha : 0.5f * alpha;
    thresholds[i] = tau_base * (1.0f + delta);
    if (sigma) sigma[i] = (hi == lo) ? 0.f : (float)((track_mean[i] - lo) / (hi - lo));
  }
}

}  // namespace

int launch_tile_std(const void* const* x, int n_tiles, int64_t elems, int dtype, float* tile_std, void* ws, hipStream_t s) {
  if (n_tiles == 0) return SG_OK;
  double* partial = (double*)ws;
  int dev = 0, n_cu = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
  SG_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  constexpr int kWavesPerBlock = kThreads / 64;   // one partial slot per wavefront
  const int n_blk = n_cu < 1 ? 1 : (n_cu > kGateSlots / kWavesPerBlock ? kGateSlots / kWavesPerBlock : n_cu);
  for (int t0 = 0; t0 < n_tiles; t0 += kTilesPerLaunch) {
    const int n = (n_tiles - t0 < kTilesPerLaunch) ? n_tiles - t0 : kTilesPerLaunch;
    StdPtrs ptrs;
    for (int i = 0; i < kTilesPerLaunch; ++i) ptrs.x[i] = i < n ? x[t0 + i] : nullptr;
    if (dtype == SG_BF16) tile_moments_kernel<SG_BF16><<<n_blk, kThreads, 0, s>>>(ptrs, t0, n, elems, partial);
    else tile_moments_kernel<SG_F32><<<n_blk, kThreads, 0, s>>>(ptrs, t0, n, elems, partial);
    SG_HIP_TRY(hipGetLastError());
  }
  tile_std_finalize_kernel<<<n_tiles, kFinalThreads, 0, s>>>(partial, n_blk * kWavesPerBlock, elems, tile_std);
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

int launch_region_thresholds(const float* tile_std, double* track_mean, int32_t* track_count, int n_tiles,
                             float tau_base, float alpha, int mode, int adjust, float* sigma, float* thresholds,
                             hipStream_t s) {
  if (n_tiles == 0) return SG_OK;
  region_threshold_kernel<<<1, kThreads, 0, s>>>(tile_std, track_mean, track_count, n_tiles, tau_base, alpha, mode, adjust,
                                                 sigma, thresholds);
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

}  // namespace sg
