// Internal declarations shared by the translation units of liblpp (not installed).
#ifndef LPP_INTERNAL_H_
#define LPP_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <vector>

#include "lpp.h"

// Host-side image of a static draft tree plus its device copy.
struct lpp_tree {
  int32_t M = 0;             // rows (root + drafted nodes)
  int32_t depth = 0;         // levels below the root
  int32_t n_parents = 0;     // rows with at least one child
  int32_t max_children = 0;
  bool consecutive_children = true;  // the children of every row are consecutive rows
  int32_t words = 0;         // 64-bit words per ancestor bitmask
  std::vector<int32_t> parent, row_depth, child_ptr, child_idx;
  std::vector<int32_t> heavy_first;  // rows by descending number of children (ties: ascending row)
  std::vector<uint64_t> anc; // [M * words]
  // device copies (null for a host-only handle)
  int device = -1;
  int32_t n_cu = 256;        // compute units of that device (launch heuristics)
  int32_t clock_khz = 2400000;  // its shader clock
  int32_t walk_patience = 1 << 19;   // rounds the resident-grid walk waits for the other rows (lpp_tree_set_walk_patience)
  int32_t* d_child_ptr = nullptr;  // [M + 1]
  int32_t* d_child_idx = nullptr;  // [max(N, 1)]
  uint64_t* d_anc = nullptr;       // [M * words]
  // "last block done" tickets of the fused kernels: zero between calls.  Calls that
  // share one handle must therefore be ordered on a stream.
  int32_t* d_counters = nullptr;   // [2 * LPP_COUNTER_SLOTS]: verify, then attention
  // verify with the whole grid resident: words the rows leave for the block that walks
  // ([LPP_MAX_ROWS] decisions, [LPP_MAX_ROWS] draws, each tagged with its call; then the number
  // of walks that gave up)
  int32_t* d_mail = nullptr;       // [kMailWords], zero when the handle is made
};
constexpr int kMailGaveUp = 2 * LPP_MAX_ROWS;
constexpr int kMailWords = 2 * LPP_MAX_ROWS + 1;

#define LPP_COUNTER_SLOTS 4096

#define LPP_HIP_TRY(expr)                      \
  do {                                         \
    hipError_t e_ = (expr);                    \
    if (e_ != hipSuccess) {                    \
      (void)hipGetLastError();                 \
      return LPP_EHIP;                         \
    }                                          \
  } while (0)

// The largest dynamic LDS size a kernel has been enabled for so far, per device: the attribute
// (hipFuncAttributeMaxDynamicSharedMemorySize) belongs to one device's copy of the kernel.  One
// such cache per kernel, zero-initialised; `floor` is what a kernel may use without asking.
constexpr int kLppMaxDevices = 64;
struct LppLdsLimit {
  std::atomic<size_t> raised[kLppMaxDevices];
};
inline int32_t lpp_ensure_lds(const void* kern, LppLdsLimit& lim, size_t lds, size_t floor = 0) {
  if (lds <= floor) return LPP_OK;
  int dev = -1;
  LPP_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kLppMaxDevices) return LPP_EUNSUPPORTED;
  if (lds > lim.raised[dev].load(std::memory_order_relaxed)) {
    LPP_HIP_TRY(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    lim.raised[dev].store(lds, std::memory_order_relaxed);
  }
  return LPP_OK;
}

#ifdef __HIPCC__
// Orders the LDS traffic of one wave (no other wave is waited for).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}
#endif

static inline size_t lpp_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#endif  // LPP_INTERNAL_H_
