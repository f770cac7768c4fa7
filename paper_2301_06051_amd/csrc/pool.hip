// dsvt_attn_pool: attention-style 3D pooling (Sec. 3.3, Eq. 6-7).  Not built yet.
#include "common.h"

extern "C" int dsvt_attn_pool_workspace_size(const dsvt_pool_cfg* cfg, int32_t n_voxels, size_t* bytes) {
  (void)cfg; (void)n_voxels; (void)bytes;
  return DSVT_EUNSUPPORTED;
}

extern "C" int dsvt_attn_pool(const dsvt_pool_cfg* cfg, const int32_t* coords, const void* x, int32_t n_voxels,
                              int32_t* out_coords, void* out, int32_t* n_out, void* ws, size_t ws_bytes,
                              int32_t* status, void* stream) {
  (void)cfg; (void)coords; (void)x; (void)n_voxels; (void)out_coords; (void)out; (void)n_out; (void)ws;
  (void)ws_bytes; (void)status; (void)stream;
  return DSVT_EUNSUPPORTED;
}
