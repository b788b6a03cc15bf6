// Tile attention on the matrix cores, general-addressing variant (paper Section 2.1 "full
// attention" over one tile's T x tile_h x tile_w tokens; Section 3: tiles exchange no Q/K/V).
// Used for canvases whose per-head extent exceeds the 32-bit byte offsets of the streaming kernel
// in attention_bf16.hip, and for head_dim 64 (the streaming kernel is laid out for head_dim 128);
// slower (register-staged loads, in-step barriers), same mathematics.
//
// Flash-style: a workgroup owns 256 query rows of one head (8 wavefronts x 32 rows) and streams
// the tile's keys and values through LDS 64 at a time; the N x N score matrix is never stored.
// All products are bf16 MFMA (32x32x16) with fp32 accumulation, softmax statistics are fp32.
//
// The kernel works on transposed products so that no value ever changes lanes between the two
// GEMMs:  S^T = K Q^T  puts one query per lane column (lane l holds query l%32, 16 keys in its
// accumulator registers), so the row max / row sum are in-lane reductions plus one exchange
// between the two lane halves, and the exponentials, packed to bf16, already sit in the
// B-operand layout of  O^T = V^T P^T.  V^T fragments come out of LDS through the transposing
// read (ds_read_b64_tr_b16); K and V rows are stored with XOR-swizzled 16-byte chunks so that
// both fragment reads are bank-conflict free.
#include <atomic>
#include "attention_common.h"

namespace sg {
namespace {


constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kQB = 1;                    // 32-query sub-blocks per wavefront
constexpr int kBR = kWaves * kQB * 32;    // 256 query rows per workgroup
constexpr int kBC = 64;                   // keys per LDS stage
constexpr int kXcd = 8;

// LDS stage: K[64][128] then V[64][128] bf16, rows of 256 bytes = 16 chunks of 16 bytes.
// K chunk c of row r is stored at chunk c ^ (r & 15); V chunk c of row r at c ^ ((r & 3) << 2).
// With head_dim 64 a row has 8 chunks and keeps its 256-byte slot: the XOR still sends them to distinct
// positions below 16.
constexpr int kRowBytes = 256;
constexpr int kStageBytes = 2 * kBC * kRowBytes;  // 32 KiB

__device__ __forceinline__ uint32_t k_slot(int row, int chunk) { return row * kRowBytes + ((chunk ^ (row & 15)) << 4); }
__device__ __forceinline__ uint32_t v_slot(int row, int chunk) { return kBC * kRowBytes + row * kRowBytes + ((chunk ^ ((row & 3) << 2)) << 4); }

// Value held by the lane 32 positions away (the other half of the wavefront).
__device__ __forceinline__ float other_half(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);  // r[0] = {lo, lo}, r[1] = {hi, hi}
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

struct Softmax {  // running statistics of one query (replicated in lanes l and l^32)
  float m;        // running max of the raw (unscaled) scores
  float l;        // this lane's share of the running sum
};

// One 64-key x 32-query block of scores for this lane's query (s[kb][r]: key = key0 + 32*kb +
// 8*(r>>2) + 4*half + (r&3)): update (m, l), return the rescale factor alpha for the output
// accumulators and the exponentials packed to bf16 in B-operand order (p[2*kb + h] = registers
// 8h..8h+7 of sub-block kb).
template <bool MASK>
__device__ __forceinline__ float softmax_block(f32x16 (&s)[2], Softmax& st, const float c /* scale*log2(e) */,
                                               const int key0, const int n_keys, bf16x8 (&p)[4]) {
  const int half = (threadIdx.x & 63) >> 5;
  if (MASK) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + 32 * kb + 8 * (r >> 2) + 4 * half + (r & 3);
        if (key >= n_keys) s[kb][r] = -__builtin_inff();
      }
  }
  float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s[0][r], s[1][r]));
  mx = fmaxf(mx, other_half(mx));
  const float m_new = fmaxf(st.m, mx);
  const float mc = m_new * c;
  const float alpha = __builtin_amdgcn_exp2f(st.m * c - mc);  // first block: exp2(-inf) = 0
  float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float e[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) e[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][8 * h + r], c, -mc));
#pragma unroll
      for (int r = 0; r < 8; r += 2) { sum0 += e[r]; sum1 += e[r + 1]; }
#pragma unroll
      for (int r = 0; r < 8; ++r) p[2 * kb + h][r] = (__bf16)e[r];
    }
  st.l = st.l * alpha + (sum0 + sum1);
  st.m = m_new;
  return alpha;
}

enum { kCursor = 0, kLinearRows = 1, kWrappedRows = 2 };   // how the loader finds a tile token

template <int D, int MODE>
__global__ __launch_bounds__(kThreads) void attention_bf16_generic_kernel(const View16 vw, const float c_log2, const int heads,
                                                                  const int n_qblocks, const int n_tiles, const AttnTable tab,
                                                                  const uint8_t* __restrict__ run_flags) {
  static_assert((D == 128 || D == 64) && kQB == 1 && kBC == 64, "head_dim 64 or 128, one 32-query block per wavefront, 64-key stages");
  constexpr bool LINEAR = MODE == kLinearRows;
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  SG_LDS uint8_t* const lds = (SG_LDS uint8_t*)smem;

  // Work = (active tile, head, query block), query block fastest; workgroups are dealt round-robin to the
  // 8 XCDs and renumbered so that each XCD walks a contiguous range and streams the same head's K/V through
  // its own L2.  Tiles whose run flag is 0 are not numbered; the rest of the grid exits here.
  const uint32_t active = attn_active_mask(run_flags, n_tiles);
  const int per_tile = heads * n_qblocks;
  const int total = __builtin_popcount(active) * per_tile;
  const int per_xcd = (total + kXcd - 1) / kXcd;
  const int xcd = blockIdx.x % kXcd, slot = blockIdx.x / kXcd;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int nth = logical / per_tile, in_tile = logical - nth * per_tile;
  const int tile = __builtin_amdgcn_readfirstlane(attn_nth_tile(active, nth));
  const int head = in_tile / n_qblocks, qblk = in_tile - head * n_qblocks;
  const u32x4* const qg = (const u32x4*)tab.q[tile];
  const u32x4* const kg = (const u32x4*)tab.k[tile];
  const u32x4* const vg = (const u32x4*)tab.v[tile];
  uint16_t* const out = (uint16_t*)tab.out[tile];
  const int wy0 = (MODE == kWrappedRows) ? tab.y0[tile] : 0, wx0 = (MODE == kWrappedRows) ? tab.x0[tile] : 0;
  auto token_off16 = [&](int n) __attribute__((always_inline)) -> uint32_t {
    if (MODE == kWrappedRows) return wrap_offset16(vw, wrap_cursor_at(vw, n), wy0, wx0);
    return cursor_at(vw, n).off16;
  };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, half = lane >> 5;
  const int N = vw.N;
  const uint32_t head_off16 = (uint32_t)head * vw.head16;
  const u32x4* __restrict__ kh = kg + head_off16;
  const u32x4* __restrict__ vh = vg + head_off16;

  // ---- Q fragments (B operand of S^T = K Q^T): query = q0 + 32*qb + lq, d = 16*kk + 8*half + 0..7
  const int q0 = qblk * kBR + wave * (kQB * 32);
  bf16x8 qf[kQB][D / 16];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    int n = q0 + 32 * qb + lq;
    if (n > N - 1) n = N - 1;
    const u32x4* src = qg + head_off16 + token_off16(n);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) qf[qb][kk] = __builtin_bit_cast(bf16x8, src[2 * kk + half]);
  }

  // ---- K/V loader: a row has D/8 chunks of 16 bytes; thread owns chunk (tid % kChunks) of rows
  // (tid / kChunks) + kLdRows*u, u < kLdSlots, of every stage
  constexpr int kChunks = D / 8;
  const int ld_chunk = tid % kChunks, ld_row = tid / kChunks;
  constexpr int kLdRows = kThreads / kChunks, kLdSlots = kBC / kLdRows;
  static_assert(kLdSlots >= 1 && kLdRows * kLdSlots == kBC, "the workgroup's threads tile a stage exactly");
  RowCursor cur[kLdSlots];
  WrapCursor wcur[kLdSlots];
  const uint32_t last16 = token_off16(N - 1);
#pragma unroll
  for (int u = 0; u < kLdSlots; ++u) {
    const int row = ld_row + kLdRows * u;
    if (LINEAR) { cur[u].i = 0; cur[u].j = 0; cur[u].off16 = (uint32_t)row * vw.st16; }
    else if (MODE == kWrappedRows) { wcur[u] = wrap_cursor_at(vw, row < N ? row : N - 1); cur[u].off16 = wrap_offset16(vw, wcur[u], wy0, wx0); }
    else cur[u] = cursor_at(vw, row < N ? row : N - 1);
  }
  u32x4 kreg[kLdSlots], vreg[kLdSlots];
  auto load_stage = [&](int blk) {
#pragma unroll
    for (int u = 0; u < kLdSlots; ++u) {
      const int n = blk * kBC + ld_row + kLdRows * u;
      const uint32_t off = ((n < N) ? cur[u].off16 : last16) + ld_chunk;
      kreg[u] = kh[off];
      vreg[u] = vh[off];
      if (LINEAR) cur[u].off16 += kBC * vw.st16;
      else if (n + kBC < N) {
        if (MODE == kWrappedRows) { wrap_cursor_advance(vw, wcur[u], kBC); cur[u].off16 = wrap_offset16(vw, wcur[u], wy0, wx0); }
        else cursor_advance(vw, cur[u], kBC);
      }
    }
  };
  auto store_stage = [&](int buf) {
    SG_LDS uint8_t* base = lds + buf * kStageBytes;
#pragma unroll
    for (int u = 0; u < kLdSlots; ++u) {
      const int row = ld_row + kLdRows * u;
      *(SG_LDS u32x4*)(base + k_slot(row, ld_chunk)) = kreg[u];
      *(SG_LDS u32x4*)(base + v_slot(row, ld_chunk)) = vreg[u];
    }
  };

  f32x16 oacc[D / 32][kQB];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
  Softmax st[kQB];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) { st[qb].m = -__builtin_inff(); st[qb].l = 0.f; }

  // V^T fragment addressing for the transposing read: within a 16-lane group, lane s reads 4
  // consecutive d of key row (s >> 2); the hardware hands lane i the 4 keys of d column i.
  const int grp = lane >> 4, gi = lane & 15;
  const int vt_row = 4 * (grp >> 1) + (gi >> 2);        // + 32*kb + 16*kk2 (+8 for the second read)
  const int vt_dbyte = (16 * (grp & 1) + 4 * (gi & 3)) * 2;  // + 64*db bytes

  auto compute = [&](int buf, int blk, auto mask_tag) {
    constexpr bool MASK = decltype(mask_tag)::value;
    const SG_LDS uint8_t* base = lds + buf * kStageBytes;
    // S^T = K Q^T for the stage's two 32-key sub-blocks: two independent accumulator chains
    f32x16 s[2];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      const bf16x8 a0 = __builtin_bit_cast(bf16x8, *(const SG_LDS u32x4*)(base + k_slot(lq, 2 * kk + half)));
      const bf16x8 a1 = __builtin_bit_cast(bf16x8, *(const SG_LDS u32x4*)(base + k_slot(32 + lq, 2 * kk + half)));
      if (kk == 0) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[0][kk], zero, 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[0][kk], zero, 0, 0, 0);
      } else {
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[0][kk], s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[0][kk], s[1], 0, 0, 0);
      }
    }
    bf16x8 p[4];
    const float alpha = softmax_block<MASK>(s, st[0], c_log2, blk * kBC, N, p);
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int db = 0; db < D / 32; ++db) oacc[db][0] *= alpha;
    }
    // O^T += V^T P^T: four independent accumulator chains (one per 32 rows of d)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {  // 16 keys each
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const int row0 = 16 * ks + vt_row;
        const int chunk_byte = 64 * db + vt_dbyte;  // byte offset inside the 256-byte row
        const uint32_t a0 = v_slot(row0, chunk_byte >> 4) + (chunk_byte & 15);
        const uint32_t a1 = v_slot(row0 + 8, chunk_byte >> 4) + (chunk_byte & 15);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SG_LDS s16x4*)(base + a0));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SG_LDS s16x4*)(base + a1));
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), p[ks], oacc[db][0], 0, 0, 0);
      }
    }
  };

  // Software pipeline over 64-key stages: global loads of stage b+1 are in flight while stage b
  // is consumed from LDS; the last stage (the only one that can hold keys >= N) is peeled.
  const int n_blocks = (N + kBC - 1) / kBC;
  load_stage(0);
  store_stage(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): Q fragments have landed before the loop starts
  __syncthreads();
  for (int blk = 0; blk < n_blocks - 1; ++blk) {
    load_stage(blk + 1);
    compute(blk & 1, blk, std::false_type{});
    store_stage((blk + 1) & 1);
    __syncthreads();
  }
  if ((N % kBC) != 0) compute((n_blocks - 1) & 1, n_blocks - 1, std::true_type{});
  else compute((n_blocks - 1) & 1, n_blocks - 1, std::false_type{});

  // ---- epilogue: O^T accumulators -> packed tile [head][n][d]; lane holds query lq of each sub-block,
  // register r of block db is d = 32*db + 8*(r>>2) + 4*half + (r&3): 4 consecutive d = one 8-byte store
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const int n = q0 + 32 * qb + lq;
    float l = st[qb].l;
    l += other_half(l);
    const float inv = 1.0f / l;
    if (n < N) {
      uint16_t* dst = out + ((size_t)head * N + n) * D;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w;
          w[0] = pack_bf16x2(oacc[db][qb][4 * g] * inv, oacc[db][qb][4 * g + 1] * inv);
          w[1] = pack_bf16x2(oacc[db][qb][4 * g + 2] * inv, oacc[db][qb][4 * g + 3] * inv);
          *(u32x2*)(dst + 32 * db + 8 * g + 4 * half) = w;
        }
    }
  }
}

}  // namespace

int launch_attention_bf16_generic(const TileView& tv, int heads, int head_dim, float scale, const AttnBatch& b, hipStream_t s) {
  if (head_dim != 128 && head_dim != 64) return SG_ERR_UNSUPPORTED;
  if (b.n_tiles <= 0) return SG_OK;
  const View16 vw = make_view16(tv);
  const int mode = tv.wrapped ? kWrappedRows : ((tv.W == tv.tw && tv.H == tv.th) ? kLinearRows : kCursor);
  const int n_qblocks = (tv.N + kBR - 1) / kBR;
  const float c_log2 = scale * 1.4426950408889634f;
  const size_t lds = 2 * kStageBytes;
  // the dynamic-LDS size is declared once per device and kernel (not per launch, so not inside a later capture)
  constexpr int kMaxDevices = 64;
  static std::atomic<bool> attr_set[kMaxDevices][6];   // zero-initialised; set twice by racing threads is harmless
  int dev = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
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
    const int64_t total = (int64_t)n * heads * n_qblocks;
    if (total > (1ll << 31) - 2 * kXcd) return SG_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)(((total + kXcd - 1) / kXcd) * kXcd));
    const uint8_t* flags = b.run_flags ? b.run_flags + t0 : nullptr;
    auto launch = [&](auto kern, int slot) -> int {
      if (dev < 0 || dev >= kMaxDevices || !attr_set[dev][slot].load(std::memory_order_acquire)) {
        SG_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        if (dev >= 0 && dev < kMaxDevices) attr_set[dev][slot].store(true, std::memory_order_release);
      }
      kern<<<grid, kThreads, lds, s>>>(vw, c_log2, heads, n_qblocks, n, tab, flags);
      return SG_OK;
    };
    int st;
    if (head_dim == 128) {
      if (mode == kLinearRows) st = launch(attention_bf16_generic_kernel<128, kLinearRows>, 0);
      else if (mode == kWrappedRows) st = launch(attention_bf16_generic_kernel<128, kWrappedRows>, 1);
      else st = launch(attention_bf16_generic_kernel<128, kCursor>, 2);
    } else {
      if (mode == kLinearRows) st = launch(attention_bf16_generic_kernel<64, kLinearRows>, 3);
      else if (mode == kWrappedRows) st = launch(attention_bf16_generic_kernel<64, kWrappedRows>, 4);
      else st = launch(attention_bf16_generic_kernel<64, kCursor>, 5);
    }
    if (st != SG_OK) return st;
    SG_HIP_TRY(hipGetLastError());
  }
  return SG_OK;
}

}  // namespace sg
