// dsvt_vfe: the step before the first DSVT block (Sec. 3.1 overview: the point cloud becomes sparse voxels
// through a voxel feature encoding module; the paper cites earlier pillar encoders for it).  Built here: an
// optional per-point linear map followed by the channel-wise maximum over each voxel's points.
//
// Voxels are found without a sort: an occupancy bitmap over the grid's cells, in key order, and a pop-count
// scan number the non-empty cells in ascending key; a counting sort by voxel (one returning atomic per point)
// then lists each voxel's points, and one thread per (voxel, channel) takes the maximum.  The order of a voxel's
// points in that list varies from run to run, the maximum does not.  Pure bandwidth: points are read three
// times (20 bytes each), the feature rows written once.
#include "common.h"
#include "block_scan.h"

#include <hip/hip_bf16.h>

namespace {

constexpr int kMaxFin = 16;
constexpr uint32_t kOutside = 0xFFFFFFFFu;

struct VfeGeom {
  int32_t grid[3], batch, f_in;
  float lo[3], sz[3];
};

// Cell key ((b*X + x)*Y + y)*Z + z of a point, or kOutside.  The cell is decided in float32, one rounded
// operation at a time (no fused multiply-add, no reciprocal): t = (p - lo) / size, inside iff 0 <= t < cells.
__device__ __forceinline__ uint32_t point_key(const VfeGeom& g, const float* __restrict__ p, int32_t b, int4* cell) {
  if (b < 0 || b >= g.batch) return kOutside;
  int32_t c[3];
#pragma unroll
  for (int a = 0; a < 3; ++a) {
    const float t = __fdiv_rn(__fsub_rn(p[a], g.lo[a]), g.sz[a]);
    if (!(t >= 0.f && t < (float)g.grid[a])) return kOutside;     // NaN fails both
    c[a] = (int32_t)t;
  }
  if (cell) *cell = make_int4(b, c[0], c[1], c[2]);
  return (uint32_t)(((b * g.grid[0] + c[0]) * g.grid[1] + c[1]) * g.grid[2] + c[2]);
}

__global__ void kv_clear(uint32_t* __restrict__ bitmap, int64_t n_words, int32_t* __restrict__ count, int64_t n_count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) bitmap[i] = 0u;
  if (i < n_count) count[i] = 0;
}

__global__ void kv_mark(VfeGeom g, const float* __restrict__ points, const int32_t* __restrict__ point_batch, int32_t n,
                        uint32_t* __restrict__ bitmap, uint32_t* __restrict__ keys) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint32_t key = point_key(g, points + (int64_t)i * g.f_in, point_batch ? point_batch[i] : 0, nullptr);
  keys[i] = key;
  if (key != kOutside) atomicOr(&bitmap[key >> 5], 1u << (key & 31u));
}

// Voxel index of every point (rank of its cell among the occupied ones) and its place among the voxel's points.
__global__ void kv_count(const uint32_t* __restrict__ keys, int32_t n, const uint32_t* __restrict__ bitmap,
                         const int32_t* __restrict__ word_prefix, int32_t max_voxels, int32_t* __restrict__ count,
                         int32_t* __restrict__ point_vox, int32_t* __restrict__ point_pos, int32_t* __restrict__ status) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint32_t key = keys[i];
  int32_t v = -1, pos = 0;
  if (key != kOutside) {
    const uint32_t word = key >> 5, bit = key & 31u;
    v = word_prefix[word] + __popc(bitmap[word] & ((1u << bit) - 1u));
    if (v >= max_voxels) { atomicOr(status, DSVT_ST_VOXEL_OVERFLOW); v = -1; }
    else pos = atomicAdd(&count[v], 1);
  }
  point_vox[i] = v;
  point_pos[i] = pos;
}

__global__ void kv_place(const int32_t* __restrict__ point_vox, const int32_t* __restrict__ point_pos,
                         const int32_t* __restrict__ offs, int32_t n, int32_t* __restrict__ order) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t v = point_vox[i];
  if (v >= 0) order[offs[v] + point_pos[i]] = i;       // offs[v] + pos < offs[v + 1] <= n
}

template <typename T> __device__ __forceinline__ T to_out(float v);
template <> __device__ __forceinline__ float to_out<float>(float v) { return v; }
template <> __device__ __forceinline__ __hip_bfloat16 to_out<__hip_bfloat16>(float v) { return __float2bfloat16(v); }

// One thread per (voxel, channel): h = b[c] + sum_k w[c,k] f[k] over the voxel's points, running maximum.  The C
// threads of a voxel read the same point row (one broadcast load per value) and write consecutive outputs.
template <typename T>
__global__ void __launch_bounds__(256) kv_reduce(VfeGeom g, const float* __restrict__ points,
                                                 const int32_t* __restrict__ point_batch, const int32_t* __restrict__ order,
                                                 const int32_t* __restrict__ offs, const int32_t* __restrict__ n_voxels,
                                                 int32_t max_voxels, const float* __restrict__ w, const float* __restrict__ bias,
                                                 int32_t relu, int32_t C, int32_t* __restrict__ coords, T* __restrict__ x) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int32_t nv = min(*n_voxels, max_voxels);
  const int32_t v = (int32_t)(t / C);
  if (v >= nv) return;
  const int32_t c = (int32_t)(t - (int64_t)v * C);
  float wr[kMaxFin];
#pragma unroll
  for (int k = 0; k < kMaxFin; ++k) wr[k] = (w && k < g.f_in) ? w[c * g.f_in + k] : 0.f;
  const float b0 = bias ? bias[c] : 0.f;
  const int32_t p0 = offs[v], p1 = offs[v + 1];
  float best = -INFINITY;
  for (int32_t q = p0; q < p1; ++q) {
    const float* f = points + (int64_t)order[q] * g.f_in;
    float h;
    if (w) {
      h = b0;
#pragma unroll
      for (int k = 0; k < kMaxFin; ++k)
        if (k < g.f_in) h = fmaf(wr[k], f[k], h);
    } else {
      h = f[c] + b0;
    }
    best = fmaxf(best, h);
  }
  if (relu) best = fmaxf(best, 0.f);
  x[(int64_t)v * C + c] = to_out<T>(best);
  if (c == 0) {
    const int32_t i = order[p0];                      // every voxel has at least one point
    int4 cell = make_int4(0, 0, 0, 0);
    point_key(g, points + (int64_t)i * g.f_in, point_batch ? point_batch[i] : 0, &cell);
    reinterpret_cast<int4*>(coords)[v] = cell;
  }
}

struct VfePlan {
  VfeGeom g;
  int64_t n_words;
  size_t off_bitmap, off_prefix, off_count, off_offs, off_keys, off_vox, off_pos, off_order, total;
};

int make_plan(const dsvt_vfe_cfg* cfg, int32_t n_points, int32_t max_voxels, VfePlan* pl) {
  if (!cfg || n_points <= 0 || max_voxels <= 0 || cfg->batch <= 0) return DSVT_EINVAL;
  if (cfg->f_in < 3 || cfg->f_in > kMaxFin || cfg->C <= 0) return DSVT_EINVAL;
  if (cfg->dtype != DSVT_F32 && cfg->dtype != DSVT_BF16) return DSVT_EINVAL;
  if (!cfg->w && cfg->C != cfg->f_in) return DSVT_EINVAL;
  int64_t cells = cfg->batch;
  for (int a = 0; a < 3; ++a) {
    if (cfg->grid[a] <= 0 || !(cfg->voxel_size[a] > 0.f) || !(cfg->range_min[a] == cfg->range_min[a])) return DSVT_EINVAL;
    cells *= cfg->grid[a];
    pl->g.grid[a] = cfg->grid[a];
    pl->g.lo[a] = cfg->range_min[a];
    pl->g.sz[a] = cfg->voxel_size[a];
  }
  if (cells >= (1ll << 31)) return DSVT_EUNSUPPORTED;
  if ((int64_t)max_voxels * cfg->C >= (1ll << 39)) return DSVT_EINVAL;
  pl->g.batch = cfg->batch;
  pl->g.f_in = cfg->f_in;
  pl->n_words = (int64_t)dsvt_align_up((size_t)dsvt_ceil_div(cells, 32), 64);
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off = dsvt_align_up(off + bytes, 256); return o; };
  pl->off_bitmap = take((size_t)pl->n_words * 4);
  pl->off_prefix = take((size_t)pl->n_words * 4);
  pl->off_count = take(((size_t)max_voxels + 1) * 4);
  pl->off_offs = take(((size_t)max_voxels + 1) * 4);
  pl->off_keys = take((size_t)n_points * 4);
  pl->off_vox = take((size_t)n_points * 4);
  pl->off_pos = take((size_t)n_points * 4);
  pl->off_order = take((size_t)n_points * 4);
  pl->total = off;
  return DSVT_OK;
}

}  // namespace

extern "C" int dsvt_vfe_workspace_size(const dsvt_vfe_cfg* cfg, int32_t n_points, int32_t max_voxels, size_t* bytes) {
  if (!bytes) return DSVT_EINVAL;
  VfePlan pl;
  const int rc = make_plan(cfg, n_points, max_voxels, &pl);
  if (rc != DSVT_OK) return rc;
  *bytes = pl.total;
  return DSVT_OK;
}

extern "C" int dsvt_vfe(const dsvt_vfe_cfg* cfg, const float* points, const int32_t* point_batch, int32_t n_points,
                        int32_t* coords, void* x, int32_t* n_voxels, int32_t max_voxels, void* ws, size_t ws_bytes,
                        int32_t* status, void* stream) {
  VfePlan pl;
  const int rc = make_plan(cfg, n_points, max_voxels, &pl);
  if (rc != DSVT_OK) return rc;
  if (!points || !coords || !x || !n_voxels || !ws || !status) return DSVT_EINVAL;
  if (cfg->batch > 1 && !point_batch) return DSVT_EINVAL;
  if (((uintptr_t)coords | (uintptr_t)ws) & 15u) return DSVT_EINVAL;
  if (ws_bytes < pl.total) return DSVT_ENOSPC;
  hipStream_t st = (hipStream_t)stream;
  char* base = reinterpret_cast<char*>(ws);
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(base + pl.off_bitmap);
  int32_t* prefix = reinterpret_cast<int32_t*>(base + pl.off_prefix);
  int32_t* count = reinterpret_cast<int32_t*>(base + pl.off_count);
  int32_t* offs = reinterpret_cast<int32_t*>(base + pl.off_offs);
  uint32_t* keys = reinterpret_cast<uint32_t*>(base + pl.off_keys);
  int32_t* vox = reinterpret_cast<int32_t*>(base + pl.off_vox);
  int32_t* pos = reinterpret_cast<int32_t*>(base + pl.off_pos);
  int32_t* order = reinterpret_cast<int32_t*>(base + pl.off_order);
  const int tb = 256;
  const unsigned pb = (unsigned)dsvt_ceil_div(n_points, tb);
  {
    dsvt_prof_scope ps(DSVT_K_VFE_GROUP, st);
    const int64_t n_count = (int64_t)max_voxels + 1;
    const int64_t n_clear = pl.n_words > n_count ? pl.n_words : n_count;
    kv_clear<<<(unsigned)dsvt_ceil_div(n_clear, tb), tb, 0, st>>>(bitmap, pl.n_words, count, n_count);
    kv_mark<<<pb, tb, 0, st>>>(pl.g, points, point_batch, n_points, bitmap, keys);
    k_block_scan<true><<<1, 1024, 0, st>>>(bitmap, prefix, pl.n_words, nullptr, n_voxels);
    kv_count<<<pb, tb, 0, st>>>(keys, n_points, bitmap, prefix, max_voxels, count, vox, pos, status);
    k_block_scan<false, true><<<1, 1024, 0, st>>>(reinterpret_cast<const uint32_t*>(count), offs, max_voxels, n_voxels, nullptr);
    kv_place<<<pb, tb, 0, st>>>(vox, pos, offs, n_points, order);
  }
  {
    dsvt_prof_scope ps(DSVT_K_VFE_REDUCE, st);
    const unsigned rb = (unsigned)dsvt_ceil_div((int64_t)max_voxels * cfg->C, tb);
    if (cfg->dtype == DSVT_BF16)
      kv_reduce<__hip_bfloat16><<<rb, tb, 0, st>>>(pl.g, points, point_batch, order, offs, n_voxels, max_voxels, cfg->w, cfg->b,
                                                   cfg->relu, cfg->C, coords, reinterpret_cast<__hip_bfloat16*>(x));
    else
      kv_reduce<float><<<rb, tb, 0, st>>>(pl.g, points, point_batch, order, offs, n_voxels, max_voxels, cfg->w, cfg->b,
                                          cfg->relu, cfg->C, coords, reinterpret_cast<float*>(x));
  }
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}
