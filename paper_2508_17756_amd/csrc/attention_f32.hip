// Tile attention, fp32 throughout (paper Section 2.1 "full attention" restricted to one tile).
// Plain vector-ALU kernel for SG_F32 problems, where fp32 accuracy matters more than speed:
// a workgroup owns 64 query rows; its 4 wavefronts split the keys (each wavefront takes every
// fourth 32-key chunk), one thread per query row and wavefront with q and o in registers, keys
// and values staged through LDS and read back as wave-wide broadcasts, softmax in the online
// (running max / running sum) form, which is algebraically the two-pass softmax.  The four
// partial states (m, l, o) of a query are merged through LDS at the end.
#include <atomic>
#include "attention_common.h"

namespace sg {
namespace {

constexpr int kQ = 64;       // queries per workgroup
constexpr int kSplit = 4;    // wavefronts per workgroup, each on its own share of the keys
constexpr int kKC = 32;      // keys per wavefront and LDS chunk

// element offset of tile token n from the tile's pointers (head 0); a wrapped window (shifted partition)
// starts at canvas position (y0, x0) and wraps around both canvas edges
__device__ __forceinline__ int64_t token_offset(const TileView& tv, int n, int y0, int x0) {
  const int plane = tv.th * tv.tw;
  const int t = n / plane, r = n - t * plane;
  int i = r / tv.tw, j = r - i * tv.tw;
  if (tv.wrapped) {
    i += y0; j += x0;
    i -= (i >= tv.H) ? tv.H : 0;
    j -= (j >= tv.W) ? tv.W : 0;
  }
  return (((int64_t)t * tv.H + i) * tv.W + j) * tv.stride_token;
}

// grid: (query blocks, heads, tiles of the launch); a tile whose run flag is 0 is skipped
template <int D>
__global__ __launch_bounds__(kQ * kSplit) void attention_f32_kernel(const TileView tv, const float scale, const AttnTable tab,
                                                                    const uint8_t* __restrict__ run_flags) {
  const int tile = blockIdx.z;
  if (run_flags && !run_flags[tile]) return;
  const float* __restrict__ q = (const float*)tab.q[tile];
  const float* __restrict__ k = (const float*)tab.k[tile];
  const float* __restrict__ v = (const float*)tab.v[tile];
  float* __restrict__ out = (float*)tab.out[tile];
  const int y0 = tab.y0[tile], x0 = tab.x0[tile];
  // [wavefront][key][d] chunks of K and V; after the key loop the same memory holds the partial outputs
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float (*sK)[kKC][D] = (float (*)[kKC][D])smem;
  float (*sV)[kKC][D] = (float (*)[kKC][D])(smem + kSplit * kKC * D);
  const int head = blockIdx.y;
  const int lane = threadIdx.x & (kQ - 1), wave = threadIdx.x / kQ;
  const int n = blockIdx.x * kQ + lane;
  const bool valid = n < tv.N;
  const int64_t hoff = (int64_t)head * tv.stride_head;

  float qr[D], o[D];
  {
    const float4* src = (const float4*)(q + hoff + token_offset(tv, valid ? n : tv.N - 1, y0, x0));
#pragma unroll
    for (int c = 0; c < D / 4; ++c) {
      float4 x = src[c];
      qr[4 * c] = x.x * scale; qr[4 * c + 1] = x.y * scale; qr[4 * c + 2] = x.z * scale; qr[4 * c + 3] = x.w * scale;
    }
  }
#pragma unroll
  for (int c = 0; c < D; ++c) o[c] = 0.f;
  float m = -__builtin_inff(), l = 0.f;
  constexpr float kLog2e = 1.4426950408889634f;

  // every wavefront loads and consumes its own chunk: no workgroup barrier inside the loop
  for (int m0 = wave * kKC; m0 < tv.N; m0 += kSplit * kKC) {
    const int cnt = (tv.N - m0 < kKC) ? tv.N - m0 : kKC;
    for (int e = lane; e < kKC * (D / 4); e += kQ) {
      const int row = e / (D / 4), c4 = e - row * (D / 4);
      if (row < cnt) {
        const int64_t off = hoff + token_offset(tv, m0 + row, y0, x0);
        ((float4*)sK[wave][row])[c4] = ((const float4*)(k + off))[c4];
        ((float4*)sV[wave][row])[c4] = ((const float4*)(v + off))[c4];
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float s[kKC];
    float cmax = -__builtin_inff();
#pragma unroll
    for (int r = 0; r < kKC; ++r) {
      float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
      if (r < cnt) {
#pragma unroll
        for (int c = 0; c < D / 4; ++c) {
          const float4 kk = ((const float4*)sK[wave][r])[c];
          a0 = fmaf(qr[4 * c], kk.x, a0); a1 = fmaf(qr[4 * c + 1], kk.y, a1);
          a2 = fmaf(qr[4 * c + 2], kk.z, a2); a3 = fmaf(qr[4 * c + 3], kk.w, a3);
        }
        s[r] = (a0 + a1) + (a2 + a3);
        cmax = fmaxf(cmax, s[r]);
      } else {
        s[r] = -__builtin_inff();
      }
    }
    const float m_new = fmaxf(m, cmax);
    const float alpha = exp2f((m - m_new) * kLog2e);  // m = -inf on the first chunk gives 0
    l *= alpha;
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] *= alpha;
#pragma unroll
    for (int r = 0; r < kKC; ++r) {
      if (r < cnt) {
        const float p = exp2f((s[r] - m_new) * kLog2e);
        l += p;
#pragma unroll
        for (int c = 0; c < D / 4; ++c) {
          const float4 vv = ((const float4*)sV[wave][r])[c];
          o[4 * c] = fmaf(p, vv.x, o[4 * c]); o[4 * c + 1] = fmaf(p, vv.y, o[4 * c + 1]);
          o[4 * c + 2] = fmaf(p, vv.z, o[4 * c + 2]); o[4 * c + 3] = fmaf(p, vv.w, o[4 * c + 3]);
        }
      }
    }
    m = m_new;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();   // the chunk is consumed before the next one overwrites it
  }

  // ---- merge the kSplit partial states of every query: a wavefront that saw no key has m = -inf, l = 0
  __syncthreads();
  float* sM = smem;                          // [kSplit][kQ]
  float* sL = smem + kSplit * kQ;            // [kSplit][kQ]
  float* sO = smem + 2 * kSplit * kQ;        // [kSplit][D][kQ]  (query fastest: conflict-free)
  sM[wave * kQ + lane] = m;
  sL[wave * kQ + lane] = l;
#pragma unroll
  for (int c = 0; c < D; ++c) sO[(wave * D + c) * kQ + lane] = o[c];
  __syncthreads();
  if (wave == 0 && valid) {
    float mt = sM[lane];
#pragma unroll
    for (int w = 1; w < kSplit; ++w) mt = fmaxf(mt, sM[w * kQ + lane]);
    float lt = 0.f;
    float wgt[kSplit];
#pragma unroll
    for (int w = 0; w < kSplit; ++w) {
      const float mw = sM[w * kQ + lane];
      wgt[w] = (mw == -__builtin_inff()) ? 0.f : exp2f((mw - mt) * kLog2e);
      lt += wgt[w] * sL[w * kQ + lane];
    }
    const float inv = 1.0f / lt;
    float4* dst = (float4*)(out + ((int64_t)head * tv.N + n) * D);
#pragma unroll
    for (int c = 0; c < D / 4; ++c) {
      float r4[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float acc = 0.f;
#pragma unroll
        for (int w = 0; w < kSplit; ++w) acc += wgt[w] * sO[(w * D + 4 * c + e) * kQ + lane];
        r4[e] = acc * inv;
      }
      dst[c] = make_float4(r4[0], r4[1], r4[2], r4[3]);
    }
  }
}

}  // namespace

int launch_attention_f32(const TileView& tv, int heads, int head_dim, float scale, const AttnBatch& b, hipStream_t s) {
  if (head_dim != 64 && head_dim != 128) return SG_ERR_UNSUPPORTED;
  if (b.n_tiles <= 0) return SG_OK;
  // K and V chunks of the 4 wavefronts (2 * 4 * 32 * D floats); the merge reuses them for the partial
  // outputs (4 * D * 64 floats, the same amount) and needs 2 * 4 * 64 floats more for the (m, l) pairs
  const size_t lds = ((size_t)2 * kSplit * kKC * head_dim + 2 * kSplit * kQ) * sizeof(float);
  static_assert(2 * kKC == kQ, "the merge buffer is sized by the chunk buffers");
  constexpr int kMaxDevices = 64;
  static std::atomic<bool> attr_set[kMaxDevices][2];   // zero-initialised; set twice by racing threads is harmless
  int dev = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
  const int slot = head_dim == 64 ? 0 : 1;
  const void* kern = head_dim == 64 ? (const void*)attention_f32_kernel<64> : (const void*)attention_f32_kernel<128>;
  if (dev < 0 || dev >= kMaxDevices || !attr_set[dev][slot].load(std::memory_order_acquire)) {
    SG_HIP_TRY(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    if (dev >= 0 && dev < kMaxDevices) attr_set[dev][slot].store(true, std::memory_order_release);
  }
  for (int t0 = 0; t0 < b.n_tiles; t0 += kAttnTilesPerLaunch) {
    const int n = (b.n_tiles - t0 < kAttnTilesPerLaunch) ? b.n_tiles - t0 : kAttnTilesPerLaunch;
    AttnTable tab;
    for (int i = 0; i < kAttnTilesPerLaunch; ++i) {
      const bool in = i < n;
      tab.q[i] = in ? b.q[t0 + i] : nullptr;
      tab.k[i] = in ? b.k[t0 + i] : nullptr;
      tab.v[i] = in ? b.v[t0 + i] : nullptr;
      tab.out[i] = in ? b.out[t0 + i] : nullptr;
      tab.y0[i] = (in && b.y0) ? b.y0[t0 + i] : 0;
      tab.x0[i] = (in && b.x0) ? b.x0[t0 + i] : 0;
      tab.refresh[i] = nullptr;   // the cache refresh is not carried by this kernel
    }
    const dim3 grid((tv.N + kQ - 1) / kQ, heads, n);
    const uint8_t* flags = b.run_flags ? b.run_flags + t0 : nullptr;
    if (head_dim == 64) attention_f32_kernel<64><<<grid, kQ * kSplit, lds, s>>>(tv, scale, tab, flags);
    else attention_f32_kernel<128><<<grid, kQ * kSplit, lds, s>>>(tv, scale, tab, flags);
    SG_HIP_TRY(hipGetLastError());
  }
  return SG_OK;
}

}  // namespace sg
