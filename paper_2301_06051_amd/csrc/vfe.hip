// dsvt_vfe: the step before the first DSVT block (Sec. 3.1 overview: the point cloud becomes sparse voxels
// through a voxel feature encoding module; the paper cites earlier pillar encoders for it).  Built here: an
// optional per-point linear map followed by the channel-wise maximum over each voxel's points.
//
// Voxels are found without a sort: an occupancy map over the grid's cells, in key order (a byte per cell while
// the points mark it, then packed to bits), and a pop-count scan number the non-empty cells in ascending key; a
// counting sort by voxel (one returning atomic per point) then copies each voxel's points into one run of rows,
// and wavefronts with equal shares of those rows take the maxima from LDS.  The order of a voxel's points in its
// run varies from call to call, the maximum does not.  Pure bandwidth: points are read twice and copied once,
// the feature rows written once.
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

// 16 bytes of the cell map per thread, and the per-voxel point counts.
__global__ void kv_clear(uint4* __restrict__ cell_map, int64_t n16, int32_t* __restrict__ count, int64_t n_count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) cell_map[i] = make_uint4(0u, 0u, 0u, 0u);
  if (i < n_count) count[i] = 0;
}

// Occupancy goes into a byte per cell with a plain store: every writer stores the same 1, so no atomic is needed.
// (Atomic ORs into a bitmap queue up on the few cache lines next to the sensor, where a pillar collects a hundred
// points and a line holds a thousand cells: 28 us for 180,000 points against 8 us this way.)
__global__ void kv_mark(VfeGeom g, const float* __restrict__ points, const int32_t* __restrict__ point_batch, int32_t n,
                        uint8_t* __restrict__ cell_map, uint32_t* __restrict__ keys) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint32_t key = point_key(g, points + (int64_t)i * g.f_in, point_batch ? point_batch[i] : 0, nullptr);
  keys[i] = key;
  if (key != kOutside) cell_map[key] = 1;
}

// 32 cells' bytes (each 0 or 1) -> one bitmap word, bit k = cell 32 w + k.
__global__ void kv_pack(const uint4* __restrict__ cell_map, int64_t n_words, uint32_t* __restrict__ bitmap) {
  const int64_t wd = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (wd >= n_words) return;
  const uint4 a = cell_map[2 * wd], b = cell_map[2 * wd + 1];
  const uint32_t q[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
  uint32_t word = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) word |= ((q[k] * 0x01020408u) >> 24) << (4 * k);     // the four low bits of four bytes
  bitmap[wd] = word;
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

// Counting sort, second half: every point's row copied to its voxel's run, so that the reduction reads
// consecutive (zero-padded) rows; run_info[j] = (voxel of row j, first row of its run, first row of the next run).
// The first point of a voxel also writes the voxel's coordinates.
template <int PITCH4>
__global__ void kv_place(VfeGeom g, const float* __restrict__ points, const int32_t* __restrict__ point_batch,
                         const int32_t* __restrict__ point_vox, const int32_t* __restrict__ point_pos,
                         const int32_t* __restrict__ offs, int32_t n, float4* __restrict__ sorted,
                         int4* __restrict__ run_info, int32_t* __restrict__ coords) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t v = point_vox[i];
  if (v < 0) return;
  const int32_t pos = point_pos[i], f_in = g.f_in;
  const int32_t start = offs[v], end = offs[v + 1];
  const int32_t j = start + pos;                             // j < end <= n
  const float* src = points + (int64_t)i * f_in;
  float f[4 * PITCH4];                                       // rows padded with zeros to whole 16-byte pieces
#pragma unroll
  for (int k = 0; k < 4 * PITCH4; ++k) f[k] = k < f_in ? src[k] : 0.f;
#pragma unroll
  for (int k4 = 0; k4 < PITCH4; ++k4)
    sorted[(int64_t)j * PITCH4 + k4] = make_float4(f[4 * k4], f[4 * k4 + 1], f[4 * k4 + 2], f[4 * k4 + 3]);
  run_info[j] = make_int4(v, start, end, 0);
  if (pos == 0) {
    int4 cell = make_int4(0, 0, 0, 0);
    point_key(g, src, point_batch ? point_batch[i] : 0, &cell);
    reinterpret_cast<int4*>(coords)[v] = cell;
  }
}

// Work is split by points, not by voxels (a pillar next to the sensor holds a hundred points, most hold one): a
// wavefront takes the voxels whose runs start inside its kQuota rows of the sorted array; what it needs to know
// about them comes from run_info at its first row and at the next workgroup's, so that its first loads do not
// wait for one another.  A wavefront works alone; lane l owns channels l, l + 64, ... and keeps their rows of
// w in registers, so a row fetched from LDS serves all of them.
// The rows are staged in LDS (kStage of them; a run that reaches further is read from memory), then every thread
// walks them voxel by voxel -- all lanes read the same row, so an LDS read is one broadcast -- and writes the
// voxel's maximum when its run ends.  h = b[c] + sum_k w[c,k] f[k] in k order; w == NULL: h = f[c].
constexpr int kQuota = 16, kStage = 128, kRedWaves = 4;

template <int FIN, int CPL>
__device__ __forceinline__ void fold_row(const float4* __restrict__ row, const float (&wr)[CPL][FIN], const float (&b0)[CPL],
                                         float (&best)[CPL]) {
  constexpr int P4 = (FIN + 3) / 4;
  float f[4 * P4];
#pragma unroll
  for (int k4 = 0; k4 < P4; ++k4) {
    const float4 t = row[k4];
    f[4 * k4] = t.x; f[4 * k4 + 1] = t.y; f[4 * k4 + 2] = t.z; f[4 * k4 + 3] = t.w;
  }
#pragma unroll
  for (int m = 0; m < CPL; ++m) {
    float h = b0[m];
#pragma unroll
    for (int k = 0; k < FIN; ++k) h = fmaf(wr[m][k], f[k], h);
    best[m] = fmaxf(best[m], h);
  }
}

// FIN: the point row's length rounded up to a supported one (the extra columns of w are zero); the rows' pitch is
// ceil(FIN / 4) 16-byte pieces.  CPL: channels per lane.
template <int FIN, int CPL>
__global__ void __launch_bounds__(64 * kRedWaves) kv_reduce(const float4* __restrict__ sorted, const int4* __restrict__ run_info,
                                                const int32_t* __restrict__ n_rows_dev, const int32_t* __restrict__ n_voxels,
                                                int32_t max_voxels, int32_t n_points, int32_t f_in,
                                                const float* __restrict__ w, const float* __restrict__ bias,
                                                int32_t relu, int32_t C, int32_t bf16_out, void* __restrict__ x) {
  constexpr int PITCH4 = (FIN + 3) / 4, PITCH = 4 * PITCH4;
  // Every wavefront works on a quota of its own and shares nothing with the others: four of them form a
  // workgroup only so that the dispatcher spreads them over a compute unit's four SIMDs (as one-wavefront
  // workgroups they were packed onto a third of the chip).
  __shared__ int32_t range_all[kRedWaves][4];
  __shared__ float4 rows_all[kRedWaves][kStage * PITCH4];
  __shared__ int32_t end_all[kRedWaves][kQuota];        // last row + 1 of each of the wavefront's voxels, relative
  const int32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int32_t* range_s = range_all[wv];
  float4* rows_s = rows_all[wv];
  int32_t* end_s = end_all[wv];
  const int32_t part = blockIdx.x * kRedWaves + wv;
  if (lane < 2) {
    // lane 0: the first voxel whose run starts at or after row j0, and that row; lane 1: the same for j0 + kQuota.
    const int32_t j = (part + lane) * kQuota;
    const int32_t total = *n_rows_dev, nv = min(*n_voxels, max_voxels);
    const int4 info = run_info[min(j, n_points - 1)];   // (meaningless at or beyond row `total`, and then unused)
    int32_t v = nv, p = total;
    if (j < total) {
      const bool starts = info.y == j;
      v = starts ? info.x : info.x + 1;
      p = starts ? j : info.z;
    }
    range_s[lane] = v;
    range_s[2 + lane] = p;
  }
  float wr[CPL][FIN], b0[CPL];
#pragma unroll
  for (int m = 0; m < CPL; ++m) {
    const int32_t c = lane + 64 * m;
#pragma unroll
    for (int k = 0; k < FIN; ++k) wr[m][k] = (w && c < C && k < f_in) ? w[c * f_in + k] : 0.f;
    b0[m] = (bias && c < C) ? bias[c] : 0.f;
  }
  __syncthreads();
  const int32_t va = range_s[0], n_vox = range_s[1] - va;      // n_vox <= kQuota: every run has a row; <= 0: nothing to do
  const int32_t p_begin = range_s[2], p_end = n_vox > 0 ? range_s[3] : p_begin;
  for (int32_t r = lane; r < p_end - p_begin; r += 64) {
    const int4 info = run_info[p_begin + r];
    if (info.y == p_begin + r) end_s[info.x - va] = info.z - p_begin;    // the run's first row announces its end
    if (r < kStage) {
#pragma unroll
      for (int k4 = 0; k4 < PITCH4; ++k4) rows_s[r * PITCH4 + k4] = sorted[(int64_t)(p_begin + r) * PITCH4 + k4];
    }
  }
  __syncthreads();
  const float* rows_f = reinterpret_cast<const float*>(rows_s);
  const float* sorted_f = reinterpret_cast<const float*>(sorted);
  int32_t lo = 0;
  for (int32_t vl = 0; vl < n_vox; ++vl) {
    const int32_t hi = end_s[vl], hi_s = min(hi, (int32_t)kStage);
    float best[CPL];
#pragma unroll
    for (int m = 0; m < CPL; ++m) best[m] = -INFINITY;
    if (w) {
#pragma unroll 2
      for (int32_t q = lo; q < hi_s; ++q) fold_row<FIN, CPL>(rows_s + q * PITCH4, wr, b0, best);
      for (int32_t q = max(lo, (int32_t)kStage); q < hi; ++q)             // the part of a long run that was not staged
        fold_row<FIN, CPL>(sorted + (int64_t)(p_begin + q) * PITCH4, wr, b0, best);
    } else if (lane < C) {                                // no linear map (C = f_in <= 16): channel `lane` of the row
      for (int32_t q = lo; q < hi_s; ++q) best[0] = fmaxf(best[0], rows_f[q * PITCH + lane] + b0[0]);
      for (int32_t q = max(lo, (int32_t)kStage); q < hi; ++q)
        best[0] = fmaxf(best[0], sorted_f[(int64_t)(p_begin + q) * PITCH + lane] + b0[0]);
    }
#pragma unroll
    for (int m = 0; m < CPL; ++m) {
      const int32_t c = lane + 64 * m;
      const float y = relu ? fmaxf(best[m], 0.f) : best[m];
      if (c < C) {
        if (bf16_out) reinterpret_cast<__hip_bfloat16*>(x)[(int64_t)(va + vl) * C + c] = __float2bfloat16(y);
        else reinterpret_cast<float*>(x)[(int64_t)(va + vl) * C + c] = y;
      }
    }
    lo = hi;
  }
}

struct VfePlan {
  VfeGeom g;
  int64_t n_words;
  size_t off_cells, off_bitmap, off_prefix, off_count, off_offs, off_keys, off_vox, off_pos, off_info, off_nrows, off_sorted, total;
};

int make_plan(const dsvt_vfe_cfg* cfg, int32_t n_points, int32_t max_voxels, VfePlan* pl) {
  if (!cfg || n_points <= 0 || max_voxels <= 0 || cfg->batch <= 0) return DSVT_EINVAL;
  if (cfg->f_in < 3 || cfg->f_in > kMaxFin || cfg->C <= 0 || cfg->C > 512) return DSVT_EINVAL;
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
  pl->off_cells = take((size_t)pl->n_words * 32);
  pl->off_bitmap = take((size_t)pl->n_words * 4);
  pl->off_prefix = take((size_t)pl->n_words * 4);
  pl->off_count = take(((size_t)max_voxels + 1) * 4);
  pl->off_offs = take(((size_t)max_voxels + 1) * 4);
  pl->off_keys = take((size_t)n_points * 4);
  pl->off_vox = take((size_t)n_points * 4);
  pl->off_pos = take((size_t)n_points * 4);
  pl->off_info = take((size_t)n_points * 16);
  pl->off_nrows = take(4);
  pl->off_sorted = take((size_t)n_points * ((cfg->f_in + 3) / 4) * 16);
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
  uint8_t* cells = reinterpret_cast<uint8_t*>(base + pl.off_cells);
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(base + pl.off_bitmap);
  int32_t* prefix = reinterpret_cast<int32_t*>(base + pl.off_prefix);
  int32_t* count = reinterpret_cast<int32_t*>(base + pl.off_count);
  int32_t* offs = reinterpret_cast<int32_t*>(base + pl.off_offs);
  uint32_t* keys = reinterpret_cast<uint32_t*>(base + pl.off_keys);
  int32_t* vox = reinterpret_cast<int32_t*>(base + pl.off_vox);
  int32_t* pos = reinterpret_cast<int32_t*>(base + pl.off_pos);
  float* sorted = reinterpret_cast<float*>(base + pl.off_sorted);
  int4* run_info = reinterpret_cast<int4*>(base + pl.off_info);
  int32_t* n_rows = reinterpret_cast<int32_t*>(base + pl.off_nrows);
  const int tb = 256;
  const unsigned pb = (unsigned)dsvt_ceil_div(n_points, tb);
  {
    dsvt_prof_scope ps(DSVT_K_VFE_GROUP, st);
    const int64_t n_count = (int64_t)max_voxels + 1, n16 = pl.n_words * 2;
    const int64_t n_clear = n16 > n_count ? n16 : n_count;
    kv_clear<<<(unsigned)dsvt_ceil_div(n_clear, tb), tb, 0, st>>>(reinterpret_cast<uint4*>(cells), n16, count, n_count);
    kv_mark<<<pb, tb, 0, st>>>(pl.g, points, point_batch, n_points, cells, keys);
    kv_pack<<<(unsigned)dsvt_ceil_div(pl.n_words, tb), tb, 0, st>>>(reinterpret_cast<const uint4*>(cells), pl.n_words, bitmap);
    k_block_scan<true><<<block_scan_grid(pl.n_words), 1024, 0, st>>>(bitmap, prefix, pl.n_words, nullptr, n_voxels);
    kv_count<<<pb, tb, 0, st>>>(keys, n_points, bitmap, prefix, max_voxels, count, vox, pos, status);
    k_block_scan<false, true><<<block_scan_grid(max_voxels), 1024, 0, st>>>(reinterpret_cast<const uint32_t*>(count), offs, max_voxels, n_voxels, n_rows);
    float4* sorted4 = reinterpret_cast<float4*>(sorted);
    switch ((cfg->f_in + 3) / 4) {
      case 1: kv_place<1><<<pb, tb, 0, st>>>(pl.g, points, point_batch, vox, pos, offs, n_points, sorted4, run_info, coords); break;
      case 2: kv_place<2><<<pb, tb, 0, st>>>(pl.g, points, point_batch, vox, pos, offs, n_points, sorted4, run_info, coords); break;
      case 3: kv_place<3><<<pb, tb, 0, st>>>(pl.g, points, point_batch, vox, pos, offs, n_points, sorted4, run_info, coords); break;
      default: kv_place<4><<<pb, tb, 0, st>>>(pl.g, points, point_batch, vox, pos, offs, n_points, sorted4, run_info, coords); break;
    }
  }
  {
    dsvt_prof_scope ps(DSVT_K_VFE_REDUCE, st);
    const unsigned rb = (unsigned)dsvt_ceil_div(n_points, kQuota * kRedWaves);
    const int cpl = (cfg->C + 63) / 64;                                        // channels per lane: 1, 2, 3, 4 or 8
    const int fin = cfg->f_in <= 6 ? (cfg->f_in < 4 ? 4 : cfg->f_in) : cfg->f_in <= 8 ? 8 : cfg->f_in <= 12 ? 12 : 16;
    const float4* sorted4 = reinterpret_cast<const float4*>(sorted);
#define DSVT_VFE_LAUNCH(FIN, CPL)                                                                                  \
    kv_reduce<FIN, CPL><<<rb, 64 * kRedWaves, 0, st>>>(sorted4, run_info, n_rows, n_voxels, max_voxels, n_points, cfg->f_in,    \
                                           cfg->w, cfg->b, cfg->relu, cfg->C, cfg->dtype == DSVT_BF16, x)
#define DSVT_VFE_CPL(FIN)                                                                                          \
    switch (cpl) {                                                                                                 \
      case 1: DSVT_VFE_LAUNCH(FIN, 1); break;                                                                      \
      case 2: DSVT_VFE_LAUNCH(FIN, 2); break;                                                                      \
      case 3: DSVT_VFE_LAUNCH(FIN, 3); break;                                                                      \
      case 4: DSVT_VFE_LAUNCH(FIN, 4); break;                                                                      \
      default: DSVT_VFE_LAUNCH(FIN, 8); break;                                                                     \
    }
    switch (fin) {
      case 4: DSVT_VFE_CPL(4); break;
      case 5: DSVT_VFE_CPL(5); break;
      case 6: DSVT_VFE_CPL(6); break;
      case 8: DSVT_VFE_CPL(8); break;
      case 12: DSVT_VFE_CPL(12); break;
      default: DSVT_VFE_CPL(16); break;
    }
#undef DSVT_VFE_CPL
#undef DSVT_VFE_LAUNCH
  }
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}
