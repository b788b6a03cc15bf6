// Cache gate: relative L1 change of each tile's input against its cached input
// (paper Equation 3, cached tensor in the denominator) compared with the threshold
// (Equation 7: score >= threshold recomputes).
//
// Pure HBM streaming: each input element is read once.  Stage 1 runs one workgroup per compute
// unit; a thread sums |a-b| and |b| in fp32 over its 16-byte vectors, each wavefront adds its
// threads in fp64 and stores one (num, den) pair per tile.  Stage 2 adds the pairs of a tile in
// a fixed order in fp64, so the score is bit-reproducible run to run on a given device.
#include "sg_common.h"

namespace sg {
namespace {

constexpr int kThreads = 256;
constexpr int kGateUnroll = 4;   // vectors per input and thread in flight in the gate's partial sums (6, 8, 12 are 2 % slower)
constexpr int kWavesPerBlock = kThreads / 64;   // every wavefront owns one partial slot per tile
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
  for (int tile = 0; tile < n_tiles; ++tile) {
    double* out = partial + ((size_t)(tile0 + tile) * kGateSlots + blk * kWavesPerBlock) * 2;
    if (!has_cache[tile0 + tile]) {  // no cached input: nothing to compare, buffers are not read
      if ((threadIdx.x & 63) == 0) { out[2 * (threadIdx.x >> 6)] = 0.0; out[2 * (threadIdx.x >> 6) + 1] = 0.0; }
      continue;
    }
    const u32x4* __restrict__ a = (const u32x4*)ptrs.cur[tile];
    const u32x4* __restrict__ b = (const u32x4*)ptrs.cached[tile];
    float num0 = 0.f, den0 = 0.f, num1 = 0.f, den1 = 0.f;
    int64_t i = v0 + threadIdx.x;
    for (; i + (kGateUnroll - 1) * kThreads < v1; i += kGateUnroll * kThreads) {
      u32x4 av[kGateUnroll], bv[kGateUnroll];
#pragma unroll
      for (int u = 0; u < kGateUnroll; ++u) {
        av[u] = __builtin_nontemporal_load(a + i + u * kThreads);
        bv[u] = __builtin_nontemporal_load(b + i + u * kThreads);
      }
#pragma unroll
      for (int u = 0; u < kGateUnroll; u += 2) {
        accum_vec<DT>(av[u], bv[u], num0, den0);
        accum_vec<DT>(av[u + 1], bv[u + 1], num1, den1);
      }
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
    // fixed-order tree over the wavefront
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      num += __shfl_down(num, off, 64);
      den += __shfl_down(den, off, 64);
    }
    if ((threadIdx.x & 63) == 0) {   // one partial pair per wavefront: no workgroup barrier between tiles
      out[2 * (threadIdx.x >> 6)] = num;
      out[2 * (threadIdx.x >> 6) + 1] = den;
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
    // Equation 7 reuses a tile only while its score is strictly below the threshold; the comparison is made
    // in fp64 on the unrounded ratio, so a NaN score (NaN or Inf in the inputs) recomputes rather than
    // reusing a stale cache.  The fp32 score is stored for reporting only.
    const bool cached = has_cache[tile] != 0;
    double ratio = (double)__builtin_inff();
    if (cached && !(s_den[0] == 0.0)) ratio = s_num[0] / s_den[0];
    scores[tile] = (float)ratio;
    recompute[tile] = (cached && ratio < (double)threshold) ? 0 : 1;
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

// ---------------------------------------------------------------------------------------------------
// Inter-step tile-wise cache policy (paper Section 5.1): cache residual delta_c = O_c - I_c, gain g_c
// (Equation 5), latent path length L_{c->t} (Equation 6), rule g_c L >= tau recomputes (Equation 7).
// Every ||X_z - X_{z-1}|| is the relative L1 change with the older tensor as denominator (Equation 3's
// distance), computed by the two-stage reduction above.

// Error Calculator + Threshold Comparator, one workgroup per tile.
__global__ __launch_bounds__(kFinalThreads) void gain_gate_finalize_kernel(
    const double* __restrict__ partial, int n_slots, const uint8_t* __restrict__ has_prev,
    const uint8_t* __restrict__ has_gain, const float* __restrict__ gain, float* __restrict__ path_len, float threshold,
    const float* __restrict__ tile_thresholds, float* __restrict__ step_change, float* __restrict__ scores,
    uint8_t* __restrict__ recompute) {
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
    float change = 0.f;   // first step of a tile: nothing to compare with
    if (has_prev[tile]) change = s_den[0] > 0.0 ? (float)(s_num[0] / s_den[0]) : __builtin_inff();
    const float L = path_len[tile] + change;
    path_len[tile] = L;
    step_change[tile] = change;
    const bool known = has_gain[tile] != 0;
    const float score = known ? gain[tile] * L : __builtin_inff();
    const float thr = tile_thresholds ? tile_thresholds[tile] : threshold;
    scores[tile] = score;
    recompute[tile] = (known && score < thr) ? 0 : 1;   // a NaN score recomputes
  }
}

constexpr int kRefreshTilesPerLaunch = 32;
// Measured on the 4K sizes: unroll 1-8 and 1-4 workgroups per compute unit all land within 4.4-5.1 TB/s (the
// pass writes 40-25 % of its bytes and runs at the device's copy rate); 2 and 1 were the best pair.
// Measured at the 4K sizes (20 tiles, half recomputed): equal contiguous slabs per workgroup with strided 16-byte
// halves 4.9 TB/s; chunks dealt round-robin 5.1; round-robin chunks with the lanes exchanging halves (below) 5.35,
// the plain copy rate of the same device.  Unroll 1 / 4 and 2 - 4 workgroups per compute unit are no faster.
constexpr int kRefreshUnroll = 2;
constexpr int kRefreshBlocksPerCu = 1;

// The eight fp32 residuals of a thread's 16-byte bf16 vector are 32 contiguous bytes, so a wavefront's 64 vectors
// map to one 2 KiB run of delta.  Accessed as "every lane its own two 16-byte halves" each instruction would touch
// only half of every line (measured: 6 % more bytes written than the algorithmic amount).  Instead the lanes
// exchange halves through the cross-lane network so that one instruction covers the first contiguous KiB of the run
// (lane L: 16-byte slot L) and the other the second (slot 64 + L).  Slot s holds half (s & 1) of lane s >> 1.
__device__ __forceinline__ u32x4 lane_gather(const u32x4 v, const int src_lane) {
  u32x4 r;
#pragma unroll
  for (int c = 0; c < 4; ++c) r[c] = (uint32_t)__builtin_amdgcn_ds_bpermute(src_lane << 2, (int)v[c]);
  return r;
}
// own halves (d0, d1) -> the two contiguous slots this lane stores (slot L and slot 64 + L)
__device__ __forceinline__ void halves_to_slots(const u32x4 d0, const u32x4 d1, u32x4& lo, u32x4& hi) {
  const int lane = threadIdx.x & 63;
  const u32x4 a0 = lane_gather(d0, lane >> 1), a1 = lane_gather(d1, lane >> 1);
  const u32x4 b0 = lane_gather(d0, 32 + (lane >> 1)), b1 = lane_gather(d1, 32 + (lane >> 1));
  lo = (lane & 1) ? a1 : a0;
  hi = (lane & 1) ? b1 : b0;
}
// the two contiguous slots this lane loaded (slot L and slot 64 + L) -> own halves (slots 2L and 2L + 1)
__device__ __forceinline__ void slots_to_halves(const u32x4 lo, const u32x4 hi, u32x4& d0, u32x4& d1) {
  const int lane = threadIdx.x & 63;
  const int s0 = (2 * lane) & 63, s1 = (2 * lane + 1) & 63;
  const u32x4 l0 = lane_gather(lo, s0), h0 = lane_gather(hi, s0);
  const u32x4 l1 = lane_gather(lo, s1), h1 = lane_gather(hi, s1);
  d0 = (lane < 32) ? l0 : h0;
  d1 = (lane < 32) ? l1 : h1;
}

// one 16-byte vector of outputs: O = I + delta (delta in fp32: two vectors for bf16 tensors, one for fp32)
template <int DT>
__device__ __forceinline__ u32x4 residual_apply(const u32x4 l, const u32x4 d0, const u32x4 d1) {
  u32x4 o;
  if (DT == SG_BF16) {
    o[0] = pack_bf16x2(bf16_bits_to_f32(l[0] & 0xffffu) + __uint_as_float(d0[0]), __uint_as_float(l[0] & 0xffff0000u) + __uint_as_float(d0[1]));
    o[1] = pack_bf16x2(bf16_bits_to_f32(l[1] & 0xffffu) + __uint_as_float(d0[2]), __uint_as_float(l[1] & 0xffff0000u) + __uint_as_float(d0[3]));
    o[2] = pack_bf16x2(bf16_bits_to_f32(l[2] & 0xffffu) + __uint_as_float(d1[0]), __uint_as_float(l[2] & 0xffff0000u) + __uint_as_float(d1[1]));
    o[3] = pack_bf16x2(bf16_bits_to_f32(l[3] & 0xffffu) + __uint_as_float(d1[2]), __uint_as_float(l[3] & 0xffff0000u) + __uint_as_float(d1[3]));
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) o[c] = __float_as_uint(__uint_as_float(l[c]) + __uint_as_float(d0[c]));
  }
  return o;
}
// delta = O - I for one 16-byte vector of outputs
template <int DT>
__device__ __forceinline__ void residual_take(const u32x4 a, const u32x4 l, u32x4& d0, u32x4& d1) {
  if (DT == SG_BF16) {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      d0[2 * c] = __float_as_uint(bf16_bits_to_f32(a[c] & 0xffffu) - bf16_bits_to_f32(l[c] & 0xffffu));
      d0[2 * c + 1] = __float_as_uint(__uint_as_float(a[c] & 0xffff0000u) - __uint_as_float(l[c] & 0xffff0000u));
      d1[2 * c] = __float_as_uint(bf16_bits_to_f32(a[c + 2] & 0xffffu) - bf16_bits_to_f32(l[c + 2] & 0xffffu));
      d1[2 * c + 1] = __float_as_uint(__uint_as_float(a[c + 2] & 0xffff0000u) - __uint_as_float(l[c + 2] & 0xffff0000u));
    }
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) d0[c] = __float_as_uint(__uint_as_float(a[c]) - __uint_as_float(l[c]));
    d1 = d0;
  }
}
struct GainPtrs {
  void* out_cur[kRefreshTilesPerLaunch];
  const void* out_prev[kRefreshTilesPerLaunch];
  const void* latent[kRefreshTilesPerLaunch];
  float* delta[kRefreshTilesPerLaunch];
};

// One pass over every tile's output after the Denoising Engine ran on the tiles to recompute:
//   recomputed tile: delta_c = O_t - I_t (fp32) is stored and, if a previous output exists, the sums of
//                    ||O_t - O_{t-1}||_1 and ||O_{t-1}||_1 are taken in the same pass (O_t is read once);
//   reused tile:     O_t = I_t + delta_c is written (Residual Approximation).
// One workgroup per compute unit; the workgroups walk each tile's buffers together, chunk by chunk.
// delta is kept in fp32: its magnitude follows the latent's and can exceed the output's by orders, so
// the output's storage type would lose O_c.
template <int DT>
__global__ __launch_bounds__(kThreads) void gain_refresh_kernel(GainPtrs ptrs, const uint8_t* __restrict__ recompute,
                                                                const uint8_t* __restrict__ has_prev, int tile0, int n_tiles,
                                                                int64_t elems, double* __restrict__ partial) {
  constexpr int kPerVec = (DT == SG_BF16) ? 8 : 4;
  const int blk = blockIdx.x, n_blk = gridDim.x;
  const int64_t n_vec = elems / kPerVec;
  // chunks of kRefreshUnroll * kThreads vectors are dealt round-robin to the workgroups, so at any moment the
  // whole device works on one contiguous window of every stream; the ragged rest (fewer vectors than a chunk)
  // goes to one workgroup, vector by vector without the lane exchange
  constexpr int64_t kChunk = (int64_t)kRefreshUnroll * kThreads;
  const int64_t n_chunks = n_vec / kChunk, main_end = n_chunks * kChunk;
  const int64_t first = (int64_t)blk * kChunk + threadIdx.x, step = (int64_t)n_blk * kChunk;
  const int64_t tail_first = (blk == (int)(n_chunks % n_blk)) ? main_end + threadIdx.x : n_vec, tail_end = n_vec;
  auto main_ok = [&](int64_t i) __attribute__((always_inline)) { return i - threadIdx.x < main_end; };
  auto tail_begin = [&](int64_t) __attribute__((always_inline)) { return tail_first; };
  for (int tile = 0; tile < n_tiles; ++tile) {
    double* out = partial + ((size_t)(tile0 + tile) * kGateSlots + blk * kWavesPerBlock) * 2;
    u32x4* __restrict__ oc = (u32x4*)ptrs.out_cur[tile];
    const u32x4* __restrict__ lat = (const u32x4*)ptrs.latent[tile];
    u32x4* __restrict__ dl = (u32x4*)ptrs.delta[tile];
    if (!recompute[tile0 + tile]) {   // reuse: O_t = I_t + delta_c
      int64_t i = first;
      for (; main_ok(i); i += step) {
        u32x4 l[kRefreshUnroll], d0[kRefreshUnroll], d1[kRefreshUnroll];
#pragma unroll
        for (int u = 0; u < kRefreshUnroll; ++u) {
          const int64_t j = i + u * kThreads;
          l[u] = __builtin_nontemporal_load(lat + j);
          if (DT == SG_BF16) {   // j - lane is the wavefront's first vector: its delta run starts at 2 (j - lane)
            const int64_t w0 = 2 * (j - (threadIdx.x & 63)) + (threadIdx.x & 63);
            d0[u] = __builtin_nontemporal_load(dl + w0);
            d1[u] = __builtin_nontemporal_load(dl + w0 + 64);
          } else {
            d0[u] = __builtin_nontemporal_load(dl + j);
          }
        }
#pragma unroll
        for (int u = 0; u < kRefreshUnroll; ++u) {
          if (DT == SG_BF16) {
            u32x4 h0, h1;
            slots_to_halves(d0[u], d1[u], h0, h1);
            d0[u] = h0; d1[u] = h1;
          }
          __builtin_nontemporal_store(residual_apply<DT>(l[u], d0[u], d1[u]), oc + i + u * kThreads);
        }
      }
      for (i = tail_begin(i); i < tail_end; i += kThreads) {
        const u32x4 l = __builtin_nontemporal_load(lat + i);
        u32x4 d0, d1 = {0, 0, 0, 0};
        if (DT == SG_BF16) { d0 = __builtin_nontemporal_load(dl + 2 * i); d1 = __builtin_nontemporal_load(dl + 2 * i + 1); }
        else d0 = __builtin_nontemporal_load(dl + i);
        __builtin_nontemporal_store(residual_apply<DT>(l, d0, d1), oc + i);
      }
      if ((threadIdx.x & 63) == 0) { out[2 * (threadIdx.x >> 6)] = 0.0; out[2 * (threadIdx.x >> 6) + 1] = 0.0; }
      continue;
    }
    // recompute: store the residual; relative change of the output against the previous step's
    const bool sums = has_prev[tile0 + tile] != 0;
    const u32x4* __restrict__ op = (const u32x4*)ptrs.out_prev[tile];
    float num0 = 0.f, den0 = 0.f, num1 = 0.f, den1 = 0.f;
    int64_t i = first;
    for (; main_ok(i); i += step) {
      u32x4 a[kRefreshUnroll], l[kRefreshUnroll], b[kRefreshUnroll];
#pragma unroll
      for (int u = 0; u < kRefreshUnroll; ++u) {
        const int64_t j = i + u * kThreads;
        a[u] = __builtin_nontemporal_load((const u32x4*)oc + j);
        l[u] = __builtin_nontemporal_load(lat + j);
        if (sums) b[u] = __builtin_nontemporal_load(op + j);
      }
#pragma unroll
      for (int u = 0; u < kRefreshUnroll; ++u) {
        const int64_t j = i + u * kThreads;
        if (sums) { if (u & 1) accum_vec<DT>(a[u], b[u], num1, den1); else accum_vec<DT>(a[u], b[u], num0, den0); }
        u32x4 d0, d1;
        residual_take<DT>(a[u], l[u], d0, d1);
        if (DT == SG_BF16) {
          u32x4 lo, hi;
          halves_to_slots(d0, d1, lo, hi);
          const int64_t w0 = 2 * (j - (threadIdx.x & 63)) + (threadIdx.x & 63);
          __builtin_nontemporal_store(lo, dl + w0);
          __builtin_nontemporal_store(hi, dl + w0 + 64);
        } else {
          __builtin_nontemporal_store(d0, dl + j);
        }
      }
    }
    for (i = tail_begin(i); i < tail_end; i += kThreads) {
      const u32x4 a = __builtin_nontemporal_load((const u32x4*)oc + i);
      const u32x4 l = __builtin_nontemporal_load(lat + i);
      if (sums) accum_vec<DT>(a, __builtin_nontemporal_load(op + i), num0, den0);
      u32x4 d0, d1;
      residual_take<DT>(a, l, d0, d1);
      if (DT == SG_BF16) { __builtin_nontemporal_store(d0, dl + 2 * i); __builtin_nontemporal_store(d1, dl + 2 * i + 1); }
      else __builtin_nontemporal_store(d0, dl + i);
    }
    double num = (double)num0 + (double)num1, den = (double)den0 + (double)den1;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      num += __shfl_down(num, off, 64);
      den += __shfl_down(den, off, 64);
    }
    if ((threadIdx.x & 63) == 0) {   // one partial pair per wavefront: no workgroup barrier between tiles
      out[2 * (threadIdx.x >> 6)] = num;
      out[2 * (threadIdx.x >> 6) + 1] = den;
    }
  }
}

// Cache Store update, one workgroup per tile: a recomputed tile gets g_c = ||O_t - O_{t-1}|| / d_t when a
// previous output exists and d_t is finite and positive (otherwise g_c keeps its state) and L = 0; every
// tile now has a previous step.
__global__ __launch_bounds__(kFinalThreads) void gain_refresh_finalize_kernel(
    const double* __restrict__ partial, int n_slots, const uint8_t* __restrict__ recompute,
    const float* __restrict__ step_change, uint8_t* __restrict__ has_prev, uint8_t* __restrict__ has_gain,
    float* __restrict__ gain, float* __restrict__ path_len) {
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
    if (recompute[tile]) {
      const float dt = step_change[tile];
      if (has_prev[tile] && dt > 0.f && dt < __builtin_inff()) {
        const double r = s_den[0] > 0.0 ? s_num[0] / s_den[0] : (double)__builtin_inff();
        gain[tile] = (float)(r / (double)dt);
        has_gain[tile] = 1;
      }
      path_len[tile] = 0.f;
    }
    has_prev[tile] = 1;
  }
}

}  // namespace

// Stage 1 for `n_tiles` pairs of buffers: per tile and workgroup one (sum|a-b|, sum|b|) pair in `partial`;
// tiles whose `active` byte is 0 are not read and get zero sums.  Returns the number of workgroups
// (= partial pairs per tile) in *n_slots.
static int launch_partials(const void* const* a, const void* const* b, const uint8_t* active, int n_tiles,
                           int64_t elems, int dtype, double* partial, int* n_slots, hipStream_t s) {
  // one workgroup per compute unit; the partial-sum layout (and with it the summation order) depends only
  // on the device's compute-unit count
  int dev = 0, n_cu = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
  SG_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  const int n_blk = n_cu < 1 ? 1 : (n_cu > kGateSlots / kWavesPerBlock ? kGateSlots / kWavesPerBlock : n_cu);
  *n_slots = n_blk * kWavesPerBlock;
  for (int t0 = 0; t0 < n_tiles; t0 += kTilesPerLaunch) {
    const int n = (n_tiles - t0 < kTilesPerLaunch) ? n_tiles - t0 : kTilesPerLaunch;
    GatePtrs ptrs;
    for (int i = 0; i < n; ++i) { ptrs.cur[i] = a[t0 + i]; ptrs.cached[i] = b[t0 + i]; }
    for (int i = n; i < kTilesPerLaunch; ++i) { ptrs.cur[i] = nullptr; ptrs.cached[i] = nullptr; }
    if (dtype == SG_BF16)
      gate_partial_kernel<SG_BF16><<<n_blk, kThreads, 0, s>>>(ptrs, active, t0, n, elems, partial);
    else
      gate_partial_kernel<SG_F32><<<n_blk, kThreads, 0, s>>>(ptrs, active, t0, n, elems, partial);
    SG_HIP_TRY(hipGetLastError());
  }
  return SG_OK;
}

int launch_gate(const void* const* x_cur, const void* const* x_cached, const uint8_t* has_cache, int n_tiles,
                int64_t elems, int dtype, float threshold, float* scores, uint8_t* recompute, void* ws, hipStream_t s) {
  if (n_tiles == 0) return SG_OK;
  double* partial = (double*)ws;
  int n_blk = 0;
  const int st = launch_partials(x_cur, x_cached, has_cache, n_tiles, elems, dtype, partial, &n_blk, s);
  if (st != SG_OK) return st;
  gate_finalize_kernel<<<n_tiles, kFinalThreads, 0, s>>>(partial, n_blk, has_cache, threshold, scores, recompute);
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

int launch_gain_gate(const void* const* x_cur, const void* const* x_prev, const sg_gain_state& gs, int n_tiles,
                     int64_t elems, int dtype, float threshold, const float* tile_thresholds, float* step_change,
                     float* scores, uint8_t* recompute, void* ws, hipStream_t s) {
  if (n_tiles == 0) return SG_OK;
  double* partial = (double*)ws;
  int n_blk = 0;
  const int st = launch_partials(x_cur, x_prev, gs.has_prev, n_tiles, elems, dtype, partial, &n_blk, s);
  if (st != SG_OK) return st;
  gain_gate_finalize_kernel<<<n_tiles, kFinalThreads, 0, s>>>(partial, n_blk, gs.has_prev, gs.has_gain, gs.gain,
                                                              gs.path_len, threshold, tile_thresholds, step_change,
                                                              scores, recompute);
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

int launch_gain_refresh(void* const* out_cur, const void* const* out_prev, const void* const* latent,
                        float* const* delta, const uint8_t* recompute, const float* step_change,
                        const sg_gain_state& gs, int n_tiles, int64_t elems, int dtype, void* ws, hipStream_t s) {
  if (n_tiles == 0) return SG_OK;
  double* partial = (double*)ws;
  int dev = 0, n_cu = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
  SG_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  int n_blk = (n_cu < 1 ? 1 : n_cu) * kRefreshBlocksPerCu;
  if (n_blk > kGateSlots / kWavesPerBlock) n_blk = kGateSlots / kWavesPerBlock;
  for (int t0 = 0; t0 < n_tiles; t0 += kRefreshTilesPerLaunch) {
    const int n = (n_tiles - t0 < kRefreshTilesPerLaunch) ? n_tiles - t0 : kRefreshTilesPerLaunch;
    GainPtrs ptrs;
    for (int i = 0; i < kRefreshTilesPerLaunch; ++i) {
      ptrs.out_cur[i] = i < n ? out_cur[t0 + i] : nullptr;
      ptrs.out_prev[i] = i < n ? out_prev[t0 + i] : nullptr;
      ptrs.latent[i] = i < n ? latent[t0 + i] : nullptr;
      ptrs.delta[i] = i < n ? delta[t0 + i] : nullptr;
    }
    if (dtype == SG_BF16)
      gain_refresh_kernel<SG_BF16><<<n_blk, kThreads, 0, s>>>(ptrs, recompute, gs.has_prev, t0, n, elems, partial);
    else
      gain_refresh_kernel<SG_F32><<<n_blk, kThreads, 0, s>>>(ptrs, recompute, gs.has_prev, t0, n, elems, partial);
    SG_HIP_TRY(hipGetLastError());
  }
  gain_refresh_finalize_kernel<<<n_tiles, kFinalThreads, 0, s>>>(partial, n_blk * kWavesPerBlock, recompute, step_change, gs.has_prev,
                                                                 gs.has_gain, gs.gain, gs.path_len);
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
