// sg_cache_gate_static: the cache gate for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels and same results
// as sg_cache_gate; the partial sums of the two-stage reduction live in a fixed device array owned by
// the library instead of a caller workspace.
#include <atomic>
#include <cmath>
#include "sg_common.h"

// One (num, den) fp64 pair per wavefront of the partial-sum kernel and tile: 16 KiB per tile, 1 MiB in
// all.  Every device the library runs on holds its own copy until the process ends.
static __device__ __align__(256) unsigned char scratch[(size_t)SG_STATIC_GATE_MAX_TILES * sg::kGateSlots * 2 * sizeof(double)];

namespace sg {
namespace {

// In host code `scratch` is only a handle for the symbol, not a device address: the address of each
// device's copy is looked up once, with that device current, and only that pointer goes to kernels.
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];   // zero-initialised

int static_scratch(void** out) {
  int dev = 0;
  SG_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SG_ERR_UNSUPPORTED;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {   // two threads racing here look up the same address twice: harmless
    SG_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SG_ERR_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return SG_OK;
}

}  // namespace
}  // namespace sg

using namespace sg;

extern "C" int sg_cache_gate_static(const void* const* x_cur, const void* const* x_cached, const uint8_t* has_cache,
                                    int32_t n_tiles, int64_t elems_per_tile, int32_t dtype, float threshold,
                                    float* scores, uint8_t* recompute, void* stream) {
  if (n_tiles < 0 || elems_per_tile < 0) return SG_ERR_INVALID_ARG;
  if (dtype != SG_F32 && dtype != SG_BF16) return SG_ERR_INVALID_ARG;
  if (std::isnan(threshold)) return SG_ERR_INVALID_ARG;
  if (n_tiles > SG_STATIC_GATE_MAX_TILES) return SG_ERR_WORKSPACE;   // more tiles than the fixed scratch holds
  if (n_tiles == 0) return SG_OK;
  if (!x_cur || !x_cached || !has_cache || !scores || !recompute) return SG_ERR_INVALID_ARG;
  for (int i = 0; i < n_tiles; ++i) {
    if (!x_cur[i] || (((uintptr_t)x_cur[i]) & 15u)) return SG_ERR_INVALID_ARG;
    if (!x_cached[i] || (((uintptr_t)x_cached[i]) & 15u)) return SG_ERR_INVALID_ARG;
  }
  void* ws = nullptr;
  const int st = static_scratch(&ws);
  if (st != SG_OK) return st;
  // The partial-sum kernel writes every slot the finalize kernel reads (zero pairs for tiles without a
  // cache), so nothing of the previous call's contents has to be cleared.
  return launch_gate(x_cur, x_cached, has_cache, n_tiles, elems_per_tile, dtype, threshold, scores, recompute, ws,
                     (hipStream_t)stream);
}
