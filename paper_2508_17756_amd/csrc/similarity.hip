// Similarity of a tile tensor across adjacent denoising steps (paper Equation 3): the relative L1 distance
// ||x_new - x_old||_1 / ||x_old||_1 (the earlier step's tensor in the denominator) and the cosine similarity
// <x_new, x_old> / (||x_new||_2 ||x_old||_2).  The paper profiles predicted noise and cache residuals with this
// pair to choose what to cache and where to put the thresholds (Section 3; Section 5.1).
//
// One streaming read of both tensors (HBM-bound, the cache gate's layout: one resident workgroup per compute
// unit, equal contiguous slabs per tile).  A thread keeps the five sums in fp32 over its 16-byte vectors, the
// wavefronts add them in fp64, the four wavefronts of a workgroup meet in LDS, and the finalize kernel adds the
// workgroups' partials in a fixed order: bit-reproducible from run to run on a given device.
#include "sg_common.h"

namespace sg {
namespace {

constexpr int kThreads = 256;
constexpr int kSimUnroll = 8;   // vectors per input and thread in flight: 16 loads of 16 bytes (4: 6.9 TB/s, 8: 7.05, 12 and 16: 7.0)
constexpr int kFinalThreads = 128;
constexpr int kTilesPerLaunch = 64;
constexpr int kSums = 5;   // sum|a-b|, sum|b|, sum a b, sum a^2, sum b^2
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct SimPtrs {
  const void* a[kTilesPerLaunch];
  const void* b[kTilesPerLaunch];
};

__device__ __forceinline__ void sim_pair(const float a, const float b, float (&s)[kSums]) {
  s[0] += fabsf(a - b);
  s[1] += fabsf(b);
  s[2] += a * b;
  s[3] += a * a;
  s[4] += b * b;
}
template <int DT>
__device__ __forceinline__ void sim_vec(const u32x4 a, const u32x4 b, float (&s)[kSums]) {
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (DT == SG_BF16) {
      sim_pair(bf16_bits_to_f32(a[c] & 0xffffu), bf16_bits_to_f32(b[c] & 0xffffu), s);
      sim_pair(__uint_as_float(a[c] & 0xffff0000u), __uint_as_float(b[c] & 0xffff0000u), s);
    } else {
      sim_pair(__uint_as_float(a[c]), __uint_as_float(b[c]), s);
    }
  }
}

// partial: per tile kGateSlots * 2 doubles; workgroup blk of a tile writes its five sums at [blk * kSums, +kSums)
template <int DT>
__global__ __launch_bounds__(kThreads) void similarity_partial_kernel(SimPtrs ptrs, int tile0, int n_tiles, int64_t elems,
                                                                      double* __restrict__ partial) {
  constexpr int kPerVec = (DT == SG_BF16) ? 8 : 4;
  __shared__ double s_part[kThreads / 64][kSums];
  const int blk = blockIdx.x, n_blk = gridDim.x;
  const int64_t n_vec = elems / kPerVec;
  const int64_t per_blk = (n_vec + n_blk - 1) / n_blk;
  const int64_t v0 = (int64_t)blk * per_blk;
  const int64_t v1 = (v0 + per_blk < n_vec) ? v0 + per_blk : n_vec;
  for (int tile = 0; tile < n_tiles; ++tile) {
    const u32x4* __restrict__ a = (const u32x4*)ptrs.a[tile];
    const u32x4* __restrict__ b = (const u32x4*)ptrs.b[tile];
    float s0[kSums] = {0.f, 0.f, 0.f, 0.f, 0.f}, s1[kSums] = {0.f, 0.f, 0.f, 0.f, 0.f};
    int64_t i = v0 + threadIdx.x;
    for (; i + (kSimUnroll - 1) * kThreads < v1; i += kSimUnroll * kThreads) {
      u32x4 av[kSimUnroll], bv[kSimUnroll];
#pragma unroll
      for (int u = 0; u < kSimUnroll; ++u) { av[u] = __builtin_nontemporal_load(a + i + u * kThreads); bv[u] = __builtin_nontemporal_load(b + i + u * kThreads); }
#pragma unroll
      for (int u = 0; u < kSimUnroll; u += 2) { sim_vec<DT>(av[u], bv[u], s0); sim_vec<DT>(av[u + 1], bv[u + 1], s1); }
    }
    for (; i < v1; i += kThreads) sim_vec<DT>(__builtin_nontemporal_load(a + i), __builtin_nontemporal_load(b + i), s0);
    double d[kSums];
#pragma unroll
    for (int j = 0; j < kSums; ++j) d[j] = (double)s0[j] + (double)s1[j];
    if (blk == n_blk - 1) {   // ragged tail (elems not a multiple of the vector width): last workgroup, scalar
      for (int64_t e = n_vec * kPerVec + threadIdx.x; e < elems; e += kThreads) {
        float af, bf;
        if (DT == SG_BF16) {
          af = bf16_bits_to_f32(((const uint16_t*)ptrs.a[tile])[e]);
          bf = bf16_bits_to_f32(((const uint16_t*)ptrs.b[tile])[e]);
        } else {
          af = ((const float*)ptrs.a[tile])[e];
          bf = ((const float*)ptrs.b[tile])[e];
        }
        d[0] += (double)fabsf(af - bf); d[1] += (double)fabsf(bf);
        d[2] += (double)af * (double)bf; d[3] += (double)af * (double)af; d[4] += (double)bf * (double)bf;
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
#pragma unroll
      for (int j = 0; j < kSums; ++j) d[j] += __shfl_down(d[j], off, 64);
    if ((threadIdx.x & 63) == 0)
#pragma unroll
      for (int j = 0; j < kSums; ++j) s_part[threadIdx.x >> 6][j] = d[j];
    __syncthreads();
    if (threadIdx.x < kSums) {
      double t = 0.0;
      for (int w = 0; w < kThreads / 64; ++w) t += s_part[w][threadIdx.x];
      partial[(size_t)(tile0 + tile) * kGateSlots * 2 + (size_t)blk * kSums + threadIdx.x] = t;
    }
    __syncthreads();   // s_part is reused by the next tile
  }
}

__global__ __launch_bounds__(kFinalThreads) void similarity_finalize_kernel(const double* __restrict__ partial, int n_blk,
                                                                            float* __restrict__ l1_rel, float* __restrict__ cos_sim) {
  const int tile = blockIdx.x;
  __shared__ double s_sum[kSums][kFinalThreads];
  double t[kSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  for (int w = threadIdx.x; w < n_blk; w += kFinalThreads)
#pragma unroll
    for (int j = 0; j < kSums; ++j) t[j] += partial[(size_t)tile * kGateSlots * 2 + (size_t)w * kSums + j];
#pragma unroll
  for (int j = 0; j < kSums; ++j) s_sum[j][threadIdx.x] = t[j];
  __syncthreads();
  for (int off = kFinalThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off)
#pragma unroll
      for (int j = 0; j < kSums; ++j) s_sum[j][threadIdx.x] += s_sum[j][threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double num = s_sum[0][0], den = s_sum[1][0], dot = s_sum[2][0], aa = s_sum[3][0], bb = s_sum[4][0];
    l1_rel[tile] = (den == 0.0) ? __builtin_inff() : (float)(num / den);
    // the direction of a zero tensor is not defined: its cosine is reported as 0
    cos_sim[tile] = (aa == 0.0 || bb == 0.0) ? 0.f : (float)(dot / (sqrt(aa) * sqrt(bb)));
  }
}

}  // namespace

int launch_similarity(const void* const* x_new, const void* const* x_old, int n_tiles, int64_t elems, int dtype,
                      float* l1_rel, float* cos_sim, void* ws, hipStream_t s) {
  if (n_tiles == 0) return SG_OK;
  double* partial = (double*)ws;
  int dev = 0, n_cu = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
  SG_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  constexpr int kMaxBlk = kGateSlots * 2 / kSums;   // the tile's share of the workspace holds this many workgroups' sums
  const int n_blk = n_cu < 1 ? 1 : (n_cu > kMaxBlk ? kMaxBlk : n_cu);
  for (int t0 = 0; t0 < n_tiles; t0 += kTilesPerLaunch) {
    const int n = (n_tiles - t0 < kTilesPerLaunch) ? n_tiles - t0 : kTilesPerLaunch;
    SimPtrs ptrs;
    for (int i = 0; i < kTilesPerLaunch; ++i) { ptrs.a[i] = i < n ? x_new[t0 + i] : nullptr; ptrs.b[i] = i < n ? x_old[t0 + i] : nullptr; }
    if (dtype == SG_BF16) similarity_partial_kernel<SG_BF16><<<n_blk, kThreads, 0, s>>>(ptrs, t0, n, elems, partial);
    else similarity_partial_kernel<SG_F32><<<n_blk, kThreads, 0, s>>>(ptrs, t0, n, elems, partial);
    SG_HIP_TRY(hipGetLastError());
  }
  similarity_finalize_kernel<<<n_tiles, kFinalThreads, 0, s>>>(partial, n_blk, l1_rel, cos_sim);
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

}  // namespace sg
