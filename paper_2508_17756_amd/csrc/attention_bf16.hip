// Tile attention on the matrix cores (paper Section 2.1 "full attention" over one tile's
// T x tile_h x tile_w tokens; Section 3: tiles exchange no Q/K/V).
//
// Flash-style: a workgroup of 8 wavefronts owns 256 query rows of one head (32 per wavefront) and
// streams the tile's keys and values through a 4-stage LDS ring, 64 keys per stage, filled by
// direct global->LDS transfers; the N x N score matrix is never stored.  All products are bf16
// MFMA (32x32x16) with fp32 accumulation, softmax statistics are fp32.
//
// Transposed products keep every value in its lane between the two GEMMs:  S^T = K Q^T  puts one
// query per lane column (lane l holds query l%32, 16 keys of a 32-key block in its accumulator
// registers), so the exponentials, packed to bf16, already sit in the B-operand layout of
// O^T = V^T P^T.  V^T fragments come out of LDS through the transposing read (ds_read_b64_tr_b16);
// K and V rows are stored with XOR-swizzled 16-byte chunks so both fragment reads are free of bank
// conflicts.
//
// Vector work beside the MFMAs costs issue slots and, on a power-limited part, clock, so the softmax is
// cut to one exponential, one add and half a convert per score:  Q is pre-multiplied by log2(e)*scale (one bf16 rounding)
// and the score accumulators start at -M, the softmax reference, so the MFMA result is the
// exponent itself.  M is an online-softmax running maximum refreshed lazily (see Softmax below).
// A SIMD overlaps MFMA and vector work only across wavefronts, never inside one, so the two
// wavefronts of each SIMD run half an iteration apart (see "Schedule" in the kernel).
//
// Built with -fno-honor-nans: a NaN in Q, K or V gives unspecified (not necessarily NaN) output.
#include <type_traits>
#include <atomic>
#include "attention_common.h"

namespace sg {
namespace {

#define SG_INLINE __attribute__((always_inline))   // on the kernel's lambdas: a lambda left as a call pins every captured array in memory

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kBR = kWaves * 32;   // query rows per workgroup
constexpr int kBC = 64;            // keys per stage
constexpr int kStages = 4;
constexpr int kXcd = 8;
constexpr int kRowBytes = 256;
constexpr int kTileBytes = kBC * kRowBytes;          // one K (or V) stage: 16 KiB
constexpr int kVRegion = kStages * kTileBytes;       // V stages start at 64 KiB
constexpr int kLdsBytes = 2 * kStages * kTileBytes;  // 128 KiB

// 16 bytes per lane from global memory straight into LDS: lane i fills bytes [16 i, 16 i + 16) of the
// 1 KiB block at LDS byte address `lds_dst` (wave-uniform).  Address = sbase + voff (32-bit byte offset).
// Inline assembly keeps the compiler from ordering later LDS reads behind the transfer; completion is
// awaited explicitly with wait_vmcnt.  The statement overwrites m0 and says so.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"   // m0 is a reserved register; naming it as clobbered is the point
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_dst), "v"(voff), "s"(sbase) : "memory", "m0");
}
#pragma clang diagnostic pop
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N == 0 || N == 4 || N == 8, "");
  if (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  if (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
}
__device__ __forceinline__ void meet() {  // workgroup barrier that nothing is scheduled across
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// Softmax state of one query (replicated in lanes l and l^32).  Scores leave the MFMA already in the
// exponent domain: t = log2(e) * scale * <q, k> - M, because Q is pre-multiplied by log2(e) * scale and
// the accumulator of the first MFMA of each chain starts at -M (M = the reference the exponentials are
// taken against).  M is an online-softmax running maximum that is refreshed lazily: as long as no
// exponential of a stage exceeds 2^16 the reference stays, so the common path needs no row maximum, no
// subtraction and no rescaling of the output accumulators; the result is the same softmax, since any
// common reference cancels in sum(p v) / sum(p).
// Score and probability arrays have this fixed extent for either head_dim (NB <= kMaxSB blocks are used):
// their types then do not depend on a template parameter, which the register-pinning asm statements need.
constexpr int kMaxSB = 4;

struct Softmax {
  float M;   // reference, log2 domain
  float l;   // this lane's share of sum(p)
};

// Scores of keys at or beyond n_keys become -inf.  Branch- and compare-free (sign mask + bit select), so the
// 16 NB decisions do not each occupy a pair of scalar registers.
template <int NB>
__device__ __forceinline__ void mask_tail(f32x16 (&t)[kMaxSB], const int key0, const int n_keys) {
  const int half = (threadIdx.x & 63) >> 5;
  const int limit = n_keys - key0 - 4 * half;   // register (kb, r) holds key offset 32 kb + 8 (r >> 2) + (r & 3)
#pragma unroll
  for (int kb = 0; kb < NB; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int c = 32 * kb + 8 * (r >> 2) + (r & 3);
      const uint32_t beyond = (uint32_t)((limit - 1 - c) >> 31);   // all ones if c >= limit
      t[kb][r] = __uint_as_float((__float_as_uint(t[kb][r]) & ~beyond) | (0xff800000u & beyond));
    }
}

// p[2 kb + h] = bf16(exp2(t[kb][8h..8h+7])) in B-operand order; returns this lane's sum of the exponentials
template <int NB>
__device__ __forceinline__ float exp_block(const f32x16 (&t)[kMaxSB], bf16x8 (&p)[2 * kMaxSB]) {
  float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
  for (int kb = 0; kb < NB; ++kb)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float e[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) e[r] = __builtin_amdgcn_exp2f(t[kb][8 * h + r]);
#pragma unroll
      for (int r = 0; r < 8; ++r) p[2 * kb + h][r] = (__bf16)e[r];
#pragma unroll
      for (int r = 0; r < 8; r += 2) { sum0 += e[r]; sum1 += e[r + 1]; }
    }
  return sum0 + sum1;
}
// row maximum of the stage for this lane's query, combined over both halves of the wavefront
template <int NB>
__device__ __forceinline__ float block_max(const f32x16 (&t)[kMaxSB]) {
  float mx0 = t[0][0], mx1 = t[1][0];
#pragma unroll
  for (int r = 1; r < 15; r += 2) {
    mx0 = fmaxf(fmaxf(mx0, t[0][r]), t[0][r + 1]);
    mx1 = fmaxf(fmaxf(mx1, t[1][r]), t[1][r + 1]);
  }
  mx0 = fmaxf(mx0, t[0][15]);
  mx1 = fmaxf(mx1, t[1][15]);
#pragma unroll
  for (int kb = 2; kb < NB; ++kb) {
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      if (kb & 1) mx1 = fmaxf(fmaxf(mx1, t[kb][r]), t[kb][r + 1]);
      else mx0 = fmaxf(fmaxf(mx0, t[kb][r]), t[kb][r + 1]);
    }
  }
  const float mx = fmaxf(mx0, mx1);
  const uint32_t mu = __float_as_uint(mx);
  const auto sw = __builtin_amdgcn_permlane32_swap(mu, mu, false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
constexpr float kOverflowGuard = 65536.0f;   // a stage's exponentials may grow to 2^16 before the reference moves

enum { kPerLane = 0, kLinear = 1, kScalarWalk = 2, kWrapped = 3 };   // how the loader walks the tile (see the DMA loader)

template <int D, int MODE>
__global__ __launch_bounds__(kThreads) void attention_bf16_kernel(const View16 vw, const float c_log2, const int heads,
                                                                  const int n_qblocks, const int n_tiles, const AttnTable tab,
                                                                  const uint8_t* __restrict__ run_flags, const int first_copy_block,
                                                                  const int64_t copy_vecs, uint8_t* __restrict__ has_cache) {
  static_assert(D == 128 || D == 64, "head_dim 64 or 128");
  static_assert(D == 128 || MODE == kLinear, "head_dim 64 streams packed tiles only");
  // LDS rows ("slots") are always 256 bytes.  With head_dim 128 a slot is one key and a stage 64 keys; with
  // head_dim 64 a stage is 128 keys and slot 32 g + r holds key 64 g + r in its first half and key
  // 64 g + 32 + r in its second, so the fragment reads and the MFMA count per stage are the same and only
  // the pairing of fragments with accumulators differs (see qk and pv).
  constexpr int kSB = (D == 128) ? 2 : 4;   // 32-key score blocks per stage
  constexpr int kKeys = 32 * kSB;           // keys per stage
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  SG_LDS uint8_t* const lds = (SG_LDS uint8_t*)smem;
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

  // Work = (active tile, head, query block) triples, query block fastest.  Workgroups are dealt round-robin
  // to the 8 XCDs; renumber so that each XCD walks a contiguous range of the work and its CUs stream the same
  // head's K/V through one L2.  Only the tiles whose run flag is set are numbered, so the work is spread
  // evenly over the XCDs whichever tiles the gate reuses; the rest of the grid exits here.
  const uint32_t active = attn_active_mask(run_flags, n_tiles);
  const int per_tile = heads * n_qblocks;
  const int total = __builtin_popcount(active) * per_tile;
  const int per_xcd = (total + kXcd - 1) / kXcd;
  const int xcd = blockIdx.x % kXcd, slot = blockIdx.x / kXcd;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) {
    // The workgroups behind the attention grid carry the step's cache refresh (cache_x <- x for the tiles that run):
    // they are dispatched last, onto the compute units the attention's final, partial round leaves idle, and
    // stream through HBM, which the attention hardly uses.  Chunks of one vector per thread are dealt round-robin,
    // so the copy walks both buffers as one contiguous window.
    if ((int)blockIdx.x < first_copy_block) return;
    const int c = blockIdx.x - first_copy_block, n_copy = gridDim.x - first_copy_block;
    for (uint32_t m = active; m; m &= m - 1) {
      const int t = __builtin_ctz(m);
      const u32x4* __restrict__ src = (const u32x4*)tab.q[t];
      u32x4* __restrict__ dst = (u32x4*)tab.refresh[t];
      int64_t i = (int64_t)c * kThreads + threadIdx.x;
      const int64_t step = (int64_t)n_copy * kThreads;
      for (; i + 7 * step < copy_vecs; i += 8 * step) {   // eight 16-byte loads in flight per thread
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * step);
#pragma unroll
        for (int u = 0; u < 8; ++u) __builtin_nontemporal_store(v[u], dst + i + u * step);
      }
      for (; i < copy_vecs; i += step) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
      if (c == 0 && threadIdx.x == 0) has_cache[t] = 1;
    }
    return;
  }
  const int nth = logical / per_tile, in_tile = logical - nth * per_tile;
  const int tile = __builtin_amdgcn_readfirstlane(attn_nth_tile(active, nth));
  const int head = in_tile / n_qblocks, qblk = in_tile - head * n_qblocks;
  const u32x4* const qg = (const u32x4*)tab.q[tile];
  const u32x4* const kg = (const u32x4*)tab.k[tile];
  const u32x4* const vg = (const u32x4*)tab.v[tile];
  uint16_t* const out = (uint16_t*)tab.out[tile];
  const int wy0 = (MODE == kWrapped) ? tab.y0[tile] : 0, wx0 = (MODE == kWrapped) ? tab.x0[tile] : 0;
  // offset of tile token n from the tile's pointers, in 16-byte units
  auto token_off16 = [&](int n) SG_INLINE -> uint32_t {
    if (MODE == kWrapped) return wrap_offset16(vw, wrap_cursor_at(vw, n), wy0, wx0);
    return cursor_at(vw, n).off16;
  };

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, half = lane >> 5;
  const int N = vw.N;
  const uint32_t head_off16 = (uint32_t)head * vw.head16;
  const u32x4* const kh = kg + head_off16;   // wave-uniform bases of this head
  const u32x4* const vh = vg + head_off16;

  // ---- Q fragments (B operand of S^T = K Q^T): query q0 + lq, d = 16 kk + 8 half + 0..7
  const int q0 = qblk * kBR + wave * 32;
  bf16x8 qf[D / 16];
  {
    int n = q0 + lq;
    if (n > N - 1) n = N - 1;
    const u32x4* src = qg + head_off16 + token_off16(n);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      const u32x4 raw = src[2 * kk + half];
      u32x4 scaled;   // q * log2(e) * scale, rounded to bf16 once
#pragma unroll
      for (int e = 0; e < 4; ++e)
        scaled[e] = pack_bf16x2(bf16_bits_to_f32(raw[e] & 0xffffu) * c_log2, __uint_as_float(raw[e] & 0xffff0000u) * c_log2);
      qf[kk] = __builtin_bit_cast(bf16x8, scaled);
    }
  }

  // ---- LDS layout: K stages [4][64 rows][256 B] at 0, V stages at 64 KiB.  16-byte chunk c of K row r
  // sits at chunk c ^ (r & 15); chunk c of V row r at c ^ ((r & 3) << 2): both fragment reads below are
  // then bank-conflict free.  All per-lane addresses are fixed; stage and sub-block enter as immediates.
  uint32_t kaddr[8];   // A operand of QK: slot lq (+32), chunk 2 kk + half
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) kaddr[kk] = lds0 + lq * kRowBytes + (((2 * kk + half) ^ (lq & 15)) << 4);
  // V^T fragments through the transposing read: within a 16-lane group lane s reads 4 consecutive d of key
  // row (s >> 2); the hardware hands lane i the 4 keys of d column i.
  const int grp = lane >> 4, gi = lane & 15;
  const int vt_row = 4 * (grp >> 1) + (gi >> 2);
  const int vt_dbyte = (16 * (grp & 1) + 4 * (gi & 3)) * 2;
  uint32_t vaddr[4];   // + 4096 ks (+ 2048 for slots +8), 64-byte block db of the slot
#pragma unroll
  for (int db = 0; db < 4; ++db)
    vaddr[db] = lds0 + kVRegion + vt_row * kRowBytes + (((4 * db + (vt_dbyte >> 4)) ^ ((vt_row & 3) << 2)) << 4) + (vt_dbyte & 15);

  // ---- DMA loader: wavefront w moves rows 8w..8w+7 of every stage, 4 rows (1 KiB) per instruction; lane l
  // fills chunk slot (l & 15) of row 8w + 4u + (l >> 4) and therefore fetches the chunk that belongs there.
  //
  // kScalarWalk / kLinear: the 8 rows of a wavefront are always consecutive tokens of one tile row (tile
  // width a multiple of 8, or a packed tile whose rows are adjacent anyway).  The address then splits into
  // a wave-uniform 64-bit pointer that walks the tile (scalar registers, scalar ALU) and a per-lane byte
  // offset that never changes, so the steady loop spends no vector instructions on addressing.
  // kPerLane: every lane walks its own row with a cursor and 32-bit offsets from the head's base.
  // kWrapped: the same for the wrapped window of a shifted partition; the offset is formed from the token's
  // coordinates each time, since a tile row may cross the canvas edge.
  constexpr bool kLaneWalk = (MODE == kPerLane || MODE == kWrapped);
  const int ld_sub = lane >> 4, ld_slot = lane & 15;
  uint32_t kchunk[2], vchunk[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int row = 8 * wave + 4 * u + ld_sub;
    kchunk[u] = ld_slot ^ (row & 15);
    vchunk[u] = ld_slot ^ ((row & 3) << 2);
  }
  const uint32_t last16 = token_off16(N - 1);   // the last valid row: stands in for rows >= N
  const uint32_t dma_dst = lds0 + wave * (8 * kRowBytes);
  // scalar walk: pointers to row 8w of the stage to issue (K and V), its tile row / column, lane offsets
  const char* kcur = (const char*)kh;
  const char* vcur = (const char*)vh;
  int32_t row_i = 0, col_j = 0;
  uint32_t klane[2], vlane[2];
  // per-lane walk
  RowCursor cur[2];
  WrapCursor wcur[2];
  uint32_t koff[2], voff[2];              // byte offsets from kh / vh of the next stage to issue
  // head_dim 64: key (within a stage) whose chunk this lane moves, for K and for V
  int ktok[2], vtok[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int slot_u = 8 * wave + 4 * u + ld_sub;
    ktok[u] = 64 * (slot_u >> 5) + 32 * (int)(kchunk[u] >> 3) + (slot_u & 31);
    vtok[u] = 64 * (slot_u >> 5) + 32 * (int)(vchunk[u] >> 3) + (slot_u & 31);
  }
  if (!kLaneWalk) {
    const int n0 = (D == 128) ? 8 * wave : 0;
    const RowCursor c = cursor_at(vw, n0 < N ? n0 : 0);
    row_i = __builtin_amdgcn_readfirstlane(c.i);
    col_j = __builtin_amdgcn_readfirstlane(c.j);
    const uint64_t first = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)c.off16) << 4;
    kcur += first;
    vcur += first;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (D == 128) {
        klane[u] = ((uint32_t)(4 * u + ld_sub) * vw.st16 + kchunk[u]) << 4;
        vlane[u] = ((uint32_t)(4 * u + ld_sub) * vw.st16 + vchunk[u]) << 4;
      } else {   // offsets from the stage's first key; the pointers below start at key 0, not at the wavefront's rows
        klane[u] = ((uint32_t)ktok[u] * vw.st16 + (kchunk[u] & 7)) << 4;
        vlane[u] = ((uint32_t)vtok[u] * vw.st16 + (vchunk[u] & 7)) << 4;
      }
    }
  } else {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = 8 * wave + 4 * u + ld_sub;
      uint32_t off16;
      if (MODE == kWrapped) {
        wcur[u] = wrap_cursor_at(vw, row < N ? row : N - 1);
        off16 = wrap_offset16(vw, wcur[u], wy0, wx0);
      } else {
        cur[u] = cursor_at(vw, row < N ? row : N - 1);
        off16 = cur[u].off16;
      }
      koff[u] = (off16 + kchunk[u]) << 4;
      voff[u] = (off16 + vchunk[u]) << 4;
    }
  }
  // per-lane walk: row u of this lane moves one stage on (only while the new row exists)
  auto lane_advance = [&](int u, int n) SG_INLINE {
    uint32_t off16;
    if (MODE == kWrapped) {
      if (n + kKeys < N) wrap_cursor_advance(vw, wcur[u], kKeys);
      off16 = wrap_offset16(vw, wcur[u], wy0, wx0);
    } else {
      if (n + kKeys < N) cursor_advance(vw, cur[u], kKeys);
      off16 = cur[u].off16;
    }
    koff[u] = (off16 + kchunk[u]) << 4;
    voff[u] = (off16 + vchunk[u]) << 4;
  };
  const uint64_t stage_bytes = (uint64_t)(kKeys * 16) * vw.st16;
  const uint64_t row_skip_bytes = (uint64_t)vw.row_skip16 << 4, frame_skip_bytes = (uint64_t)vw.frame_skip16 << 4;
  auto scalar_advance = [&]() SG_INLINE {   // the wavefront's rows move one stage on
    uint64_t delta = stage_bytes;
    if (MODE == kScalarWalk) {
      col_j += kKeys;
      if (vw.tw >= kKeys) {         // at most one tile-row wrap: branch-free
        const bool wrap = col_j >= vw.tw;
        col_j -= wrap ? vw.tw : 0;
        row_i += wrap ? 1 : 0;
        const bool fwrap = row_i == vw.th;
        row_i = fwrap ? 0 : row_i;
        delta += (wrap ? row_skip_bytes : 0) + (fwrap ? frame_skip_bytes : 0);
      } else {
        while (col_j >= vw.tw) {
          col_j -= vw.tw;
          delta += row_skip_bytes;
          if (++row_i == vw.th) { row_i = 0; delta += frame_skip_bytes; }
        }
      }
    }
    kcur += delta;
    vcur += delta;
  };
  // issue stage `blk` (all of its rows below N) into ring slot `st`; advance to the next stage
  auto issue_full = [&](int blk, int st) SG_INLINE {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (!kLaneWalk) {
        dma16(kcur, klane[u], dma_dst + st * kTileBytes + u * (4 * kRowBytes));
        dma16(vcur, vlane[u], dma_dst + kVRegion + st * kTileBytes + u * (4 * kRowBytes));
      } else {
        dma16(kh, koff[u], dma_dst + st * kTileBytes + u * (4 * kRowBytes));
        dma16(vh, voff[u], dma_dst + kVRegion + st * kTileBytes + u * (4 * kRowBytes));
        lane_advance(u, blk * kKeys + 8 * wave + 4 * u + ld_sub);
      }
    }
    if (!kLaneWalk) scalar_advance();
  };
  // same for a stage that may hold rows >= N: those lanes fetch the last valid row (masked later)
  auto issue_any = [&](int blk, int st) SG_INLINE {
    const int n0 = blk * kKeys + ((D == 128) ? 8 * wave : 0);   // wave-uniform
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int n = n0 + 4 * u + ld_sub;
      if (D == 64) {               // the stage's first key is valid; keys >= N take the last row, at or after it
        const uint32_t back = (uint32_t)(((const char*)kh + ((uint64_t)last16 << 4)) - kcur);
        const uint32_t ko = (n0 + ktok[u] < N) ? klane[u] : back + ((kchunk[u] & 7) << 4);
        const uint32_t vo = (n0 + vtok[u] < N) ? vlane[u] : back + ((vchunk[u] & 7) << 4);
        dma16(kcur, ko, dma_dst + st * kTileBytes + u * (4 * kRowBytes));
        dma16(vcur, vo, dma_dst + kVRegion + st * kTileBytes + u * (4 * kRowBytes));
      } else if (!kLaneWalk) {
        if (n0 + 7 < N) {          // all 8 rows valid
          dma16(kcur, klane[u], dma_dst + st * kTileBytes + u * (4 * kRowBytes));
          dma16(vcur, vlane[u], dma_dst + kVRegion + st * kTileBytes + u * (4 * kRowBytes));
        } else if (n0 < N) {       // partly valid: rows >= N take the last row, which lies at or after row n0
          const uint32_t back = (uint32_t)(((const char*)kh + ((uint64_t)last16 << 4)) - kcur);
          const uint32_t ko = (n < N) ? klane[u] : back + (kchunk[u] << 4);
          const uint32_t vo = (n < N) ? vlane[u] : back + (vchunk[u] << 4);
          dma16(kcur, ko, dma_dst + st * kTileBytes + u * (4 * kRowBytes));
          dma16(vcur, vo, dma_dst + kVRegion + st * kTileBytes + u * (4 * kRowBytes));
        } else {                   // no valid row: every lane takes the last row
          const uint64_t lastb = (uint64_t)last16 << 4;
          dma16((const char*)kh + lastb, kchunk[u] << 4, dma_dst + st * kTileBytes + u * (4 * kRowBytes));
          dma16((const char*)vh + lastb, vchunk[u] << 4, dma_dst + kVRegion + st * kTileBytes + u * (4 * kRowBytes));
        }
      } else {
        const uint32_t ko = (n < N) ? koff[u] : ((last16 + kchunk[u]) << 4);
        const uint32_t vo = (n < N) ? voff[u] : ((last16 + vchunk[u]) << 4);
        dma16(kh, ko, dma_dst + st * kTileBytes + u * (4 * kRowBytes));
        dma16(vh, vo, dma_dst + kVRegion + st * kTileBytes + u * (4 * kRowBytes));
        lane_advance(u, n);
      }
    }
    if (!kLaneWalk && n0 + kKeys < N) scalar_advance();
  };

  f32x16 oacc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  Softmax sm;
  sm.M = 0.f;
  sm.l = 0.f;
  f32x16 cinit;   // accumulator start of every score chain: -M in all registers
#pragma unroll
  for (int r = 0; r < 16; ++r) cinit[r] = 0.f;

  auto kfrag = [&](int kk, int kb, int off) SG_INLINE -> bf16x8 {
    return __builtin_bit_cast(bf16x8, *(const SG_LDS u32x4*)(uintptr_t)(kaddr[kk] + off + kb * (32 * kRowBytes)));
  };
  auto vfrag = [&](int ks, int db, int off) SG_INLINE -> bf16x8 {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SG_LDS s16x4*)(uintptr_t)(vaddr[db] + off + ks * (16 * kRowBytes)));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SG_LDS s16x4*)(uintptr_t)(vaddr[db] + off + ks * (16 * kRowBytes) + 8 * kRowBytes));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
  };
  // Fragment reads run kPF MFMA steps ahead of their use; the K fragments of the first step of a QK product
  // are read during the last step of the PV product before it, so the matrix pipe does not drain between
  // the two.  (Two steps ahead is no faster and spills registers; reading the first V^T fragments ahead,
  // during the softmax, was measured 7 % slower.)
  constexpr int kPF = 2;
  constexpr int kKPre = 1;
  bf16x8 kpre[kKPre][2];  // K fragments of the first kKPre QK steps, read during the PV tail
  // S^T = K Q^T of the stage at LDS byte offset `off`: two independent accumulator chains
  // head_dim 64: the second half of a slot is another key, so steps kk >= 4 feed the next score block
  // (block 2 kb + (kk >> 2), Q fragment kk & 3) and there are four chains, two of them in flight at a time
  auto qk = [&](int off, f32x16 (&s)[kMaxSB], bool prefetched) SG_INLINE {
    bf16x8 a[8][2];
#pragma unroll
    for (int kk = 0; kk < kPF; ++kk) {
      if (prefetched && kk < kKPre) { a[kk][0] = kpre[kk][0]; a[kk][1] = kpre[kk][1]; }
      else { a[kk][0] = kfrag(kk, 0, off); a[kk][1] = kfrag(kk, 1, off); }
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      if (kk + kPF < 8) { a[kk + kPF][0] = kfrag(kk + kPF, 0, off); a[kk + kPF][1] = kfrag(kk + kPF, 1, off); }
      __builtin_amdgcn_sched_barrier(0);
      constexpr int kPerChain = D / 16;            // MFMA steps per score block
      const int b0 = (D == 128) ? 0 : (kk >> 2);   // score blocks fed by this step: b0 and b0 + kSB / 2
      const int b1 = b0 + kSB / 2;
      const int qi = kk % kPerChain;
      if (qi == 0) {
        s[b0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk][0], qf[qi], cinit, 0, 0, 0);
        s[b1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk][1], qf[qi], cinit, 0, 0, 0);
      } else {
        s[b0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk][0], qf[qi], s[b0], 0, 0, 0);
        s[b1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk][1], qf[qi], s[b1], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // O^T += V^T P^T: four independent accumulator chains (one per 32 rows of d); if a QK product follows
  // (K stage at `k_off`), its first fragments are read in the last step
  // (head_dim 64: fragment (ks, db) is d block db & 1 of the 16 keys 4 (ks >> 1) + 2 (db >> 1) + (ks & 1), two chains)
  auto pv = [&](int off, const bf16x8 (&pp)[2 * kMaxSB], int k_off, bool k_follows) SG_INLINE {
    auto acc_of = [](int i) SG_INLINE { return (D == 128) ? (i & 3) : (i & 1); };
    auto p_of = [](int i) SG_INLINE { return (D == 128) ? (i >> 2) : 4 * (i >> 3) + 2 * ((i & 3) >> 1) + ((i >> 2) & 1); };
    bf16x8 a[16];
#pragma unroll
    for (int i = 0; i < 2 * kPF; ++i) a[i] = vfrag(i >> 2, i & 3, off);
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      if (i + 2 * kPF < 16) {
        a[i + 2 * kPF] = vfrag((i + 2 * kPF) >> 2, (i + 2 * kPF) & 3, off);
        a[i + 2 * kPF + 1] = vfrag((i + 2 * kPF + 1) >> 2, (i + 2 * kPF + 1) & 3, off);
      } else if (k_follows && (i + 2 * kPF - 16) / 2 >= kPF - kKPre) {
        const int kk = (i + 2 * kPF - 16) / 2 - (kPF - kKPre);
        kpre[kk][0] = kfrag(kk, 0, k_off);
        kpre[kk][1] = kfrag(kk, 1, k_off);
      }
      __builtin_amdgcn_sched_barrier(0);
      oacc[acc_of(i)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], pp[p_of(i)], oacc[acc_of(i)], 0, 0, 0);
      oacc[acc_of(i + 1)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i + 1], pp[p_of(i + 1)], oacc[acc_of(i + 1)], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  f32x16 s[kMaxSB];   // scores of the stage in flight (the first kSB entries) between an MFMA phase and the next softmax phase
  // softmax phase of one stage: scores t (exponent domain) -> p, l.  The exponentials are taken against the
  // current reference; if one of them outgrew the guard (or on the first stage, which sets the reference) the
  // reference moves by delta per query: scores, running sum and output accumulators are brought to the new
  // reference and the exponentials are retaken.  One copy of the code, looped at most twice.
  auto softmax_phase = [&](int key0, bool masked, bool first, bf16x8 (&p)[2 * kMaxSB]) SG_INLINE {
    if (masked) mask_tail<kSB>(s, key0, N);
    bool move = first;
    float sum;
#pragma nounroll
    for (;;) {
      if (move) {
        const float mx = block_max<kSB>(s);
        const float delta = first ? mx : fmaxf(mx, 0.f);
        const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(-delta);
#pragma unroll
        for (int kb = 0; kb < kSB; ++kb) s[kb] -= delta;
        sm.M += delta;
#pragma unroll
        for (int r = 0; r < 16; ++r) cinit[r] = -sm.M;
        sm.l *= alpha;
#pragma unroll
        for (int db = 0; db < D / 32; ++db) oacc[db] *= alpha;
      }
      sum = exp_block<kSB>(s, p);
      if (move || !__any(!(sum < kOverflowGuard))) break;
      move = true;
    }
    sm.l += sum;
  };

  // ---- Schedule.  Wavefronts 0-3 (group 0) and 4-7 (group 1) share the four SIMDs pairwise and run half an
  // iteration apart, so that while one wavefront of a SIMD feeds the matrix pipe (MFMA phase: PV(k), QK(k+1))
  // the other works the vector ALU (softmax phase).  One workgroup barrier B_k per iteration re-establishes
  // the offset: after it group 0 starts MFMA phase k (its softmax k ran before the barrier) while group 1
  // starts softmax k followed by MFMA phase k.
  // Ring of 4 stages: between B_k and B_k+1 both groups read V of stage k and K of stage k+1; stage k+3 is
  // issued right after B_k into the slot of stage k-1 (last read before B_k) and must have landed by B_k+2.
  const int n_blocks = (N + kKeys - 1) / kKeys;
  const bool tail = (N % kKeys) != 0;
  // Which wavefront of a SIMD takes which role matters: the SIMD serves its older wavefront (0-3) first.  With
  // head_dim 128 (MFMA phase longer than the softmax phase) the older one leads with the MFMA phase; with head_dim 64
  // (softmax phase longer) it has to lead with the softmax, or the younger one's softmax starves behind both phases of
  // the older one and its MFMA phase then runs with nothing beside it (measured: 1.08 -> 1.22 PFLOP/s; the opposite
  // choice costs head_dim 128 a quarter of its rate).
  const int grp1 = __builtin_amdgcn_readfirstlane((wave >> 2) ^ (D == 64 ? 1 : 0));
  auto wait_stage = [&](int younger_stages) SG_INLINE {   // own transfers: all but the youngest `younger_stages` stages landed
    __builtin_amdgcn_sched_barrier(0);
    if (younger_stages >= 2) wait_vmcnt<8>();
    else if (younger_stages == 1) wait_vmcnt<4>();
    else wait_vmcnt<0>();
  };
  bf16x8 p[2 * kMaxSB];   // the first 2 kSB entries
  // keeps the score registers live across the phase boundary (a macro: the statement has to sit in the
  // lambdas that are its call sites)
#define SG_PIN_SCORES()                                                                \
  do {                                                                                 \
    asm volatile("" : : "v"(s[0]), "v"(s[1]));                                         \
    if constexpr (kSB == 4) asm volatile("" : : "v"(s[kSB - 2]), "v"(s[kSB - 1]));      \
  } while (0)
  auto mfma_phase_static = [&](auto st_tag) SG_INLINE {
    constexpr int ST = decltype(st_tag)::value;
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
    pv(ST * kTileBytes, p, ((ST + 1) % kStages) * kTileBytes, true);
    qk(((ST + 1) % kStages) * kTileBytes, s, true);
    SG_PIN_SCORES();
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto mfma_phase_any = [&](int k) SG_INLINE {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
    pv((k % kStages) * kTileBytes, p, ((k + 1) % kStages) * kTileBytes, k + 1 < n_blocks);
    if (k + 1 < n_blocks) qk(((k + 1) % kStages) * kTileBytes, s, true);
    SG_PIN_SCORES();
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto softmax_pinned = [&](int j, bool masked, bool first) SG_INLINE {
    softmax_phase(j * kKeys, masked, first, p);
    asm volatile("" : : "v"(p[0]), "v"(p[1]), "v"(p[2]), "v"(p[3]), "v"(sm.l), "v"(cinit));
    if constexpr (kSB == 4) asm volatile("" : : "v"(p[kSB]), "v"(p[kSB + 1]), "v"(p[kSB + 2]), "v"(p[kSB + 3]));
    __builtin_amdgcn_sched_barrier(0);
  };

  for (int b = 0; b < 3; ++b)
    if (b < n_blocks) issue_any(b, b);
  wait_stage(n_blocks >= 3 ? 2 : (n_blocks == 2 ? 1 : 0));
  meet();
  qk(0, s, false);
  SG_PIN_SCORES();
  const int n_steady = (n_blocks >= 2 * kStages) ? kStages + ((n_blocks - 2 * kStages) / kStages) * kStages : 0;

  if (!grp1) {
    softmax_pinned(0, tail && n_blocks == 1, true);
    wait_stage(n_blocks >= 3 ? 1 : 0);
    meet();   // B_0
    auto general = [&](int k) SG_INLINE {
      if (k + 3 < n_blocks) issue_any(k + 3, (k + 3) % kStages);
      mfma_phase_any(k);
      if (k + 1 < n_blocks) softmax_pinned(k + 1, tail && k + 1 == n_blocks - 1, false);
      wait_stage(k + 3 <= n_blocks - 1 ? 1 : 0);
      meet();
    };
    auto steady = [&](int k, auto st_tag) SG_INLINE {
      constexpr int ST = decltype(st_tag)::value;
      issue_full(k + 3, (ST + 3) % kStages);
      mfma_phase_static(st_tag);
      softmax_pinned(k + 1, false, false);
      wait_stage(1);
      meet();
    };
    int k = 0;
    for (; k < kStages && k < n_blocks; ++k) general(k);
    for (; k < n_steady; k += kStages) {
      steady(k, std::integral_constant<int, 0>{});
      steady(k + 1, std::integral_constant<int, 1>{});
      steady(k + 2, std::integral_constant<int, 2>{});
      steady(k + 3, std::integral_constant<int, 3>{});
    }
    for (; k < n_blocks; ++k) general(k);
  } else {
    wait_stage(n_blocks >= 3 ? 1 : 0);
    meet();   // B_0
    auto general = [&](int k) SG_INLINE {
      if (k + 3 < n_blocks) issue_any(k + 3, (k + 3) % kStages);
      softmax_pinned(k, tail && k == n_blocks - 1, k == 0);
      mfma_phase_any(k);
      wait_stage(k + 3 <= n_blocks - 1 ? 1 : 0);
      meet();
    };
    auto steady = [&](int k, auto st_tag) SG_INLINE {
      constexpr int ST = decltype(st_tag)::value;
      issue_full(k + 3, (ST + 3) % kStages);
      softmax_pinned(k, false, false);
      mfma_phase_static(st_tag);
      wait_stage(1);
      meet();
    };
    int k = 0;
    for (; k < kStages && k < n_blocks; ++k) general(k);
    for (; k < n_steady; k += kStages) {
      steady(k, std::integral_constant<int, 0>{});
      steady(k + 1, std::integral_constant<int, 1>{});
      steady(k + 2, std::integral_constant<int, 2>{});
      steady(k + 3, std::integral_constant<int, 3>{});
    }
    for (; k < n_blocks; ++k) general(k);
  }

  // ---- epilogue: O^T accumulators -> packed tile [head][n][d]; register r of block db is
  // d = 32 db + 8 (r>>2) + 4 half + (r&3): 4 consecutive d = one 8-byte store
  {
    const int n = q0 + lq;
    const uint32_t lu = __float_as_uint(sm.l);
    const auto sw = __builtin_amdgcn_permlane32_swap(lu, lu, false, false);
    const float inv = 1.0f / (__uint_as_float(sw[0]) + __uint_as_float(sw[1]));
    if (n < N) {
      uint16_t* dst = out + ((size_t)head * N + n) * D;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w;
          w[0] = pack_bf16x2(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv);
          w[1] = pack_bf16x2(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
          *(u32x2*)(dst + 32 * db + 8 * g + 4 * half) = w;
        }
    }
  }
}

}  // namespace

int launch_attention_bf16(const TileView& tv, int heads, int head_dim, float scale, const AttnBatch& b, hipStream_t s) {
  if (head_dim != 128 && head_dim != 64) return SG_ERR_UNSUPPORTED;
  if (b.n_tiles <= 0) return SG_OK;
  const bool linear = (tv.W == tv.tw && tv.H == tv.th) && !tv.wrapped;
  // head_dim 64 streams packed tiles only (two keys share an LDS slot, 32 keys apart: not one tile row);
  // tiles read in place from a canvas take the register-staged kernel
  if (head_dim == 64 && !linear) return launch_attention_bf16_generic(tv, heads, head_dim, scale, b, s);
  const View16 vw = make_view16(tv);
  // a wavefront moves 8 consecutive tile tokens per stage: contiguous in memory whenever they cannot
  // straddle a tile row (tile width a multiple of 8) or the tile rows are themselves adjacent (packed tile)
  const int mode = tv.wrapped ? kWrapped : (linear ? kLinear : (tv.tw % 8 == 0 ? kScalarWalk : kPerLane));
  // The per-lane cursors address a head's K/V with 32-bit byte offsets from a wave-uniform base; canvases
  // whose per-head extent does not fit take the kernel with 64-bit addressing.
  const int64_t head_extent = ((int64_t)tv.T * tv.H * tv.W) * tv.stride_token;
  if ((mode == kPerLane || mode == kWrapped) && head_extent * 2 >= (1ll << 32))
    return launch_attention_bf16_generic(tv, heads, head_dim, scale, b, s);
  const int n_qblocks = (tv.N + kBR - 1) / kBR;
  const float c_log2 = scale * 1.4426950408889634f;
  // the kernels need more dynamic LDS than the default limit; the attribute is set once per device and kernel
  constexpr int kMaxDevices = 64;
  static std::atomic<bool> attr_set[kMaxDevices][5];   // zero-initialised; set twice by racing threads is harmless
  int dev = 0, n_cu = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
  SG_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  if (n_cu < 4) n_cu = 4;
  // the cache refresh rides on this launch for packed tiles (their inputs are one contiguous run each)
  const bool fuse_refresh = b.refresh_dst && b.has_cache && b.refresh_bytes > 0 && (b.refresh_bytes & 15) == 0 && linear;
  bool tab_refresh_ok = false;
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
    }
    const int64_t total = (int64_t)n * heads * n_qblocks;   // the grid covers every tile; skipped tiles' share exits at once
    const int64_t attn_blocks = ((total + kXcd - 1) / kXcd) * kXcd;
    // fused cache refresh: as many copy workgroups as the attention's last round leaves compute units idle (at least
    // a quarter of the device), appended to the grid
    int64_t copy_blocks = 0;
    if (fuse_refresh) {
      copy_blocks = n_cu - attn_blocks % n_cu;
      if (copy_blocks < n_cu / 4) copy_blocks += n_cu;
      tab_refresh_ok = true;
    }
    if (attn_blocks + copy_blocks > (1ll << 31) - 1) return SG_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)(attn_blocks + copy_blocks));
    const uint8_t* flags = b.run_flags ? b.run_flags + t0 : nullptr;
    for (int i = 0; i < kAttnTilesPerLaunch; ++i) tab.refresh[i] = (fuse_refresh && i < n) ? b.refresh_dst[t0 + i] : nullptr;
    auto launch = [&](auto kern, int slot) -> int {
      if (dev < 0 || dev >= kMaxDevices || !attr_set[dev][slot].load(std::memory_order_acquire)) {
        SG_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
        if (dev >= 0 && dev < kMaxDevices) attr_set[dev][slot].store(true, std::memory_order_release);
      }
      kern<<<grid, kThreads, kLdsBytes, s>>>(vw, c_log2, heads, n_qblocks, n, tab, flags, (int)attn_blocks,
                                             fuse_refresh ? b.refresh_bytes / 16 : 0,
                                             fuse_refresh ? b.has_cache + t0 : nullptr);
      return SG_OK;
    };
    int st = SG_OK;
    if (head_dim == 64) st = launch(attention_bf16_kernel<64, kLinear>, 4);
    else if (mode == kLinear) st = launch(attention_bf16_kernel<128, kLinear>, kLinear);
    else if (mode == kScalarWalk) st = launch(attention_bf16_kernel<128, kScalarWalk>, kScalarWalk);
    else if (mode == kWrapped) st = launch(attention_bf16_kernel<128, kWrapped>, kWrapped);
    else st = launch(attention_bf16_kernel<128, kPerLane>, kPerLane);
    if (st != SG_OK) return st;
    SG_HIP_TRY(hipGetLastError());
  }
  if (b.refreshed) *b.refreshed = tab_refresh_ok;
  return SG_OK;
}

}  // namespace sg
