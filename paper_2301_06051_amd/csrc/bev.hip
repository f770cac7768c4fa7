// dsvt_bev_scatter: the step after the last DSVT block (Sec. 3.1, overview): each occupied cell's
// row is placed at its cell of a dense channels-last map, the image a 2D network takes.  Pure
// bandwidth: the dense map is written once (zeros, then the occupied cells' rows), the sparse rows
// are read once.
#include "common.h"

namespace {

// 16 bytes per thread over the whole dense map.
__global__ void k_bev_clear(uint4* __restrict__ out, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) out[i] = make_uint4(0u, 0u, 0u, 0u);
}

// One 16-byte chunk of one voxel's row per thread: consecutive threads write consecutive bytes of
// the cell's C-vector (channels-last), so both the read and the write are fully coalesced.
__global__ void k_bev_scatter(const int4* __restrict__ coords, const uint4* __restrict__ x, int32_t n, int32_t chunks,
                              int32_t batch, int32_t gx, int32_t gy, int32_t gz, uint4* __restrict__ out,
                              int32_t* __restrict__ status) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t i = t / chunks;
  if (i >= n) return;
  const int32_t c = (int32_t)(t - i * chunks);
  const int4 v = coords[i];                       // (b, x, y, z)
  const bool ok = v.x >= 0 && v.x < batch && v.y >= 0 && v.y < gx && v.z >= 0 && v.z < gy && v.w >= 0 && v.w < gz;
  if (!ok) {
    if (c == 0) atomicOr(status, DSVT_ST_COORD_RANGE);
    return;
  }
  const int64_t cell = (((int64_t)v.x * gx + v.y) * gy + v.z) * gz + v.w;
  out[cell * chunks + c] = x[i * chunks + c];
}

}  // namespace

extern "C" int dsvt_bev_scatter(const int32_t* coords, const void* x, int32_t n_voxels, int32_t C, int32_t dtype,
                                int32_t batch, const int32_t grid[3], void* out, int32_t* status, void* stream) {
  if (!coords || !x || !grid || !out || !status || n_voxels <= 0 || batch <= 0 || C <= 0) return DSVT_EINVAL;
  if (dtype != DSVT_F32 && dtype != DSVT_BF16) return DSVT_EINVAL;
  const int64_t row_bytes = (int64_t)C * (dtype == DSVT_BF16 ? 2 : 4);
  if (row_bytes % 16 != 0) return DSVT_EUNSUPPORTED;
  for (int a = 0; a < 3; ++a) if (grid[a] <= 0) return DSVT_EINVAL;
  if (((uintptr_t)coords | (uintptr_t)x | (uintptr_t)out) & 15u) return DSVT_EINVAL;
  const int64_t cells = (int64_t)batch * grid[0] * grid[1] * grid[2];
  const int64_t chunks = row_bytes / 16, n16 = cells * chunks;
  if (cells >= (1ll << 40) || n16 / 256 >= (1ll << 31) || (int64_t)n_voxels * chunks / 256 >= (1ll << 31)) return DSVT_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  {
    dsvt_prof_scope ps(DSVT_K_BEV_CLEAR, st);
    k_bev_clear<<<(unsigned)dsvt_ceil_div(n16, 256), 256, 0, st>>>(reinterpret_cast<uint4*>(out), n16);
  }
  {
    dsvt_prof_scope ps(DSVT_K_BEV_SCATTER, st);
    k_bev_scatter<<<(unsigned)dsvt_ceil_div((int64_t)n_voxels * chunks, 256), 256, 0, st>>>(
        reinterpret_cast<const int4*>(coords), reinterpret_cast<const uint4*>(x), n_voxels, (int32_t)chunks, batch, grid[0],
        grid[1], grid[2], reinterpret_cast<uint4*>(out), status);
  }
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}
