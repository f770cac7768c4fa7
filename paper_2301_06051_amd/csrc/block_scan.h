// Exclusive scan over an int32 array in memory, shared by the pooling and the voxel-encoding entry
// points.  POPC: the scanned value of an element is its number of set bits (a bitmap's running voxel
// count), else the element itself.  A workgroup of 1,024 threads scans one chunk of 16,384 elements
// (a thread takes 16 consecutive ones: four 16-byte loads, then one block scan of the threads'
// totals); what comes before its chunk it adds up by itself, so the workgroups of a launch do not
// wait for one another (chunk b re-reads b chunks: a few microseconds where one workgroup walking
// over all chunks in turn took three per chunk).  `in` and `out` must be 16-byte aligned and must
// not overlap; n_dev, if given, holds the element count on the device and is clamped to n_max;
// *total gets the sum, and out[n] too when TAIL is set (an offsets array of n + 1 entries).
// Launch with block_scan_grid(n_max) workgroups of 1,024 threads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kScanItems = 16;
constexpr int kScanChunk = 1024 * kScanItems;

inline unsigned block_scan_grid(int64_t n_max) { return n_max <= kScanChunk ? 1u : (unsigned)((n_max + kScanChunk - 1) / kScanChunk); }

template <bool POPC, bool TAIL = false>
__global__ void __launch_bounds__(1024) k_block_scan(const uint32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n_max,
                                                     const int32_t* __restrict__ n_dev, int32_t* __restrict__ total) {
  __shared__ int32_t wave_tot[16], wave_pre[16];
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int64_t n = n_max;
  if (n_dev) { const int64_t m = *n_dev; n = m < 0 ? 0 : (m < n_max ? m : n_max); }
  const int64_t base = (int64_t)blockIdx.x * kScanChunk;
  if (base >= n && blockIdx.x != 0) return;              // (an empty array: the first workgroup writes the zero totals)
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
  // everything before the chunk (whole 16-byte pieces: base is a multiple of the chunk), four pieces in flight per thread
  int32_t before = 0;
  for (int64_t i = (int64_t)tid * 4; i < base; i += 4 * 4096) {
    uint4 t[4];
#pragma unroll
    for (int32_t u = 0; u < 4; ++u) t[u] = i + u * 4096 < base ? *reinterpret_cast<const uint4*>(in + i + u * 4096) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int32_t u = 0; u < 4; ++u)
      before += POPC ? __popc(t[u].x) + __popc(t[u].y) + __popc(t[u].z) + __popc(t[u].w) : (int32_t)(t[u].x + t[u].y + t[u].z + t[u].w);
  }
  int32_t pre[kScanItems], mine = 0;
#pragma unroll
  for (int32_t j = 0; j < kScanItems; ++j) { pre[j] = mine; mine += POPC ? __popc(v[j]) : (int32_t)v[j]; }
  int32_t incl = mine;
  for (int32_t d = 1; d < 64; d <<= 1) {
    const int32_t up = __shfl_up(incl, d, 64);
    if (lane >= d) incl += up;
    before += __shfl_xor(before, d, 64);                 // (all lanes end with the wavefront's sum)
  }
  if (lane == 63) { wave_tot[wv] = incl; wave_pre[wv] = before; }
  __syncthreads();
  int32_t first = incl - mine, all = 0;
  for (int32_t k = 0; k < 16; ++k) {
    first += wave_pre[k] + (k < wv ? wave_tot[k] : 0);
    all += wave_pre[k] + wave_tot[k];
  }
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
  if (tid == 0 && base + kScanChunk >= n) {             // the workgroup of the last element
    if (total) *total = all;
    if (TAIL) out[n] = all;
  }
}

}  // namespace
