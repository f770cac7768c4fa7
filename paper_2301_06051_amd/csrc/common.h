// Host-side helpers shared by the entry points of libdsvt.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <atomic>

#include "dsvt.h"

#define DSVT_HIP_TRY(expr)                    \
  do {                                        \
    if ((expr) != hipSuccess) {               \
      (void)hipGetLastError();                \
      return DSVT_EHIP;                       \
    }                                         \
  } while (0)

// Lets `kernel` ask for `bytes` of dynamic LDS (more than the 64 KB default), once per device: `done` holds one
// bit per device id.  Called on every launch path; after the first time it is one atomic load.
inline int dsvt_allow_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  DSVT_HIP_TRY(hipGetDevice(&dev));
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return DSVT_OK;
  DSVT_HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  done.fetch_or(bit, std::memory_order_release);
  return DSVT_OK;
}

static inline size_t dsvt_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int64_t dsvt_ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Per-kernel timing hooks (see prof.hip): record an event pair around a launch when enabled.
void dsvt_prof_mark_begin(int kernel_id, hipStream_t stream);
void dsvt_prof_mark_end(int kernel_id, hipStream_t stream);
enum {
  DSVT_K_PART_MARK = 0, DSVT_K_PART_COUNT, DSVT_K_PART_SCAN, DSVT_K_PART_EMIT, DSVT_K_PART_CLEAR,
  DSVT_K_PART_TILES, DSVT_K_LAYER, DSVT_K_POOL_GROUP, DSVT_K_POOL_ATTN, DSVT_K_BEV_CLEAR, DSVT_K_BEV_SCATTER,
  DSVT_K_VFE_GROUP, DSVT_K_VFE_REDUCE, DSVT_K_COUNT
};
struct dsvt_prof_scope {
  int id; hipStream_t s;
  dsvt_prof_scope(int id_, hipStream_t s_) : id(id_), s(s_) { dsvt_prof_mark_begin(id, s); }
  ~dsvt_prof_scope() { dsvt_prof_mark_end(id, s); }
};
