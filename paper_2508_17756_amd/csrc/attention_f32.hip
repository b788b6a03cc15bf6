// Tile attention, fp32 throughout (paper Section 2.1 "full attention" restricted to one tile).
// Plain vector-ALU kernel for SG_F32 problems, where fp32 accuracy matters more than speed:
// one thread owns one query row (q and o live in registers), keys and values are staged
// through LDS 32 at a time and read back as wave-wide broadcasts, softmax is the online
// (running max / running sum) form, which is algebraically the two-pass softmax.
#include "sg_common.h"

namespace sg {
namespace {

constexpr int kQ = 64;   // queries per workgroup = threads
constexpr int kKC = 32;  // keys per LDS chunk

__device__ __forceinline__ int64_t token_offset(const TileView& tv, int n) {
  const int plane = tv.th * tv.tw;
  const int t = n / plane, r = n - t * plane;
  const int i = r / tv.tw, j = r - i * tv.tw;
  return tv.base + (((int64_t)t * tv.H + i) * tv.W + j) * tv.stride_token;
}

template <int D>
__global__ __launch_bounds__(kQ) void attention_f32_kernel(const TileView tv, const float scale, const float* __restrict__ q,
                                                           const float* __restrict__ k, const float* __restrict__ v,
                                                           float* __restrict__ out, const uint8_t* __restrict__ run_flag) {
  if (run_flag && !*run_flag) return;
  __shared__ __attribute__((aligned(16))) float sK[kKC][D];
  __shared__ __attribute__((aligned(16))) float sV[kKC][D];
  const int head = blockIdx.y;
  const int n = blockIdx.x * kQ + threadIdx.x;
  const bool valid = n < tv.N;
  const int64_t hoff = (int64_t)head * tv.stride_head;

  float qr[D], o[D];
  {
    const float4* src = (const float4*)(q + hoff + token_offset(tv, valid ? n : tv.N - 1));
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

  for (int m0 = 0; m0 < tv.N; m0 += kKC) {
    const int cnt = (tv.N - m0 < kKC) ? tv.N - m0 : kKC;
    __syncthreads();
    for (int e = threadIdx.x; e < kKC * (D / 4); e += kQ) {
      const int row = e / (D / 4), c4 = e - row * (D / 4);
      if (row < cnt) {
        const int64_t off = hoff + token_offset(tv, m0 + row);
        ((float4*)sK[row])[c4] = ((const float4*)(k + off))[c4];
        ((float4*)sV[row])[c4] = ((const float4*)(v + off))[c4];
      }
    }
    __syncthreads();
    float s[kKC];
    float cmax = -__builtin_inff();
#pragma unroll
    for (int r = 0; r < kKC; ++r) {
      float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
      if (r < cnt) {
#pragma unroll
        for (int c = 0; c < D / 4; ++c) {
          const float4 kk = ((const float4*)sK[r])[c];
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
          const float4 vv = ((const float4*)sV[r])[c];
          o[4 * c] = fmaf(p, vv.x, o[4 * c]); o[4 * c + 1] = fmaf(p, vv.y, o[4 * c + 1]);
          o[4 * c + 2] = fmaf(p, vv.z, o[4 * c + 2]); o[4 * c + 3] = fmaf(p, vv.w, o[4 * c + 3]);
        }
      }
    }
    m = m_new;
  }
  if (valid) {
    const float inv = 1.0f / l;
    float4* dst = (float4*)(out + ((int64_t)head * tv.N + n) * D);
#pragma unroll
    for (int c = 0; c < D / 4; ++c) dst[c] = make_float4(o[4 * c] * inv, o[4 * c + 1] * inv, o[4 * c + 2] * inv, o[4 * c + 3] * inv);
  }
}

}  // namespace

int launch_attention_f32(const TileView& tv, int heads, int head_dim, float scale, const float* q, const float* k,
                         const float* v, float* out, const uint8_t* run_flag, hipStream_t s) {
  dim3 grid((tv.N + kQ - 1) / kQ, heads);
  if (head_dim == 64) attention_f32_kernel<64><<<grid, kQ, 0, s>>>(tv, scale, q, k, v, out, run_flag);
  else if (head_dim == 128) attention_f32_kernel<128><<<grid, kQ, 0, s>>>(tv, scale, q, k, v, out, run_flag);
  else return SG_ERR_UNSUPPORTED;
  SG_HIP_TRY(hipGetLastError());
  return SG_OK;
}

}  // namespace sg
