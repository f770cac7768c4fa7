// One-workgroup exclusive scan over an int32 array in memory, shared by the pooling and the
// voxel-encoding entry points.  POPC: the scanned value of an element is its number of set bits
// (a bitmap's running voxel count), else the element itself.  A thread takes 16 consecutive
// elements per round (four 16-byte loads), so a round covers 16,384 of them with one block scan of
// the threads' totals.  `in` and `out` must be 16-byte aligned (they may be the same array);
// n_dev, if given, holds the element count on the device and is clamped to n_max; *total gets the
// sum, and out[n] too when TAIL is set (an offsets array of n + 1 entries).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kScanItems = 16;
template <bool POPC, bool TAIL = false>
__global__ void __launch_bounds__(1024) k_block_scan(const uint32_t* in, int32_t* out, int64_t n_max,
                                                     const int32_t* __restrict__ n_dev, int32_t* __restrict__ total) {
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry_s;
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int64_t n = n_max;
  if (n_dev) { const int64_t m = *n_dev; n = m < 0 ? 0 : (m < n_max ? m : n_max); }
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int64_t base = 0; base < n; base += 1024 * kScanItems) {
    const int64_t w0 = base + (int64_t)tid * kScanItems;
    uint32_t v[kScanItems];
    if (w0 + kScanItems <= n) {
#pragma unroll
      for (int32_t q = 0; q < kScanItems / 4; ++q) {
        const uint4 t = reinterpret_cast<const uint4*>(in + w0)[q];
        v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
      }
    } else {
#pragma unroll
      for (int32_t j = 0; j < kScanItems; ++j) v[j] = w0 + j < n ? in[w0 + j] : 0u;
    }
    int32_t pre[kScanItems], mine = 0;
#pragma unroll
    for (int32_t j = 0; j < kScanItems; ++j) { pre[j] = mine; mine += POPC ? __popc(v[j]) : (int32_t)v[j]; }
    int32_t incl = mine;
    for (int32_t d = 1; d < 64; d <<= 1) {
      const int32_t up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    int32_t before = carry_s;
    for (int32_t k = 0; k < wv; ++k) before += wave_tot[k];
    const int32_t first = before + incl - mine;
    if (w0 + kScanItems <= n) {
#pragma unroll
      for (int32_t q = 0; q < kScanItems / 4; ++q)
        reinterpret_cast<int4*>(out + w0)[q] =
            make_int4(first + pre[4 * q], first + pre[4 * q + 1], first + pre[4 * q + 2], first + pre[4 * q + 3]);
    } else {
#pragma unroll
      for (int32_t j = 0; j < kScanItems; ++j)
        if (w0 + j < n) out[w0 + j] = first + pre[j];
    }
    __syncthreads();
    if (tid == 1023) carry_s = before + incl;
    __syncthreads();
  }
  if (tid == 0) {
    if (total) *total = carry_s;
    if (TAIL) out[n] = carry_s;
  }
}

}  // namespace
