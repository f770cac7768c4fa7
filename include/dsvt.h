/*
 * dsvt.h -- C ABI of libdsvt: Dynamic Sparse Window Attention (DSVT, arXiv 2301.06051)
 * for AMD MI355X (gfx950).
 *
 * Conventions for every entry point
 *   - Plain C, one shared object.  No entry point allocates, frees or keeps any pointer.
 *     (One buffer carries state from call to call: the partition's `ws`, see dsvt_partition.)
 *   - Pointers marked [device] are device memory owned by the caller; pointers marked
 *     [host] are ordinary host memory.  Structs themselves are read on the host.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream) and the call returns without waiting for it.
 *   - Row-major arrays; matrix weights are [out, in].  Feature arrays and matrix weights
 *     share one element type (`dtype`): DSVT_F32 or DSVT_BF16.  Biases, LayerNorm
 *     parameters and the relative-position table are always float.
 *   - Return value: DSVT_OK, or a negative code for what the host can see (bad argument,
 *     unsupported shape, workspace too small, launch failure).  Nothing is enqueued when a
 *     negative code is returned (one exception: DSVT_EHIP from a launch that fails in the middle
 *     of a partition's chain of kernels, after which that call's `ws` is marked unprepared).  Errors only a kernel can see (a coordinate outside the
 *     grid, a repeated coordinate, more sets than `max_sets`, a partition buffer that was
 *     not prepared, more voxels than `max_voxels`) OR bits into the caller's
 *     [device] `status` word; outputs are then unspecified but no access leaves the
 *     caller's buffers.
 *   - Voxel coordinates are int32 rows (b, x, y, z), 0 <= b < batch, unique per call.
 */
#ifndef DSVT_H
#define DSVT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { DSVT_OK = 0, DSVT_EINVAL = -1, DSVT_ENOSPC = -2, DSVT_EHIP = -3, DSVT_EUNSUPPORTED = -4 };
enum { DSVT_F32 = 0, DSVT_BF16 = 1 };
/* bits of the device status word */
enum { DSVT_ST_COORD_RANGE = 1, DSVT_ST_COORD_REPEAT = 2, DSVT_ST_SET_OVERFLOW = 4, DSVT_ST_WS_STATE = 8,
       DSVT_ST_VOXEL_OVERFLOW = 16, DSVT_ST_TILE_OVERFLOW = 32 };

/* ---------------------------------------------------------------------------------------
 * Set partition (Sec. 3.2 "Dynamic set partition", Eq. 2-4; "Rotated set attention";
 * "Hybrid window partition").
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int32_t grid[3];  /* cells along X, Y, Z                                             */
  int32_t win[3];   /* window size L, W, H in cells                                    */
  int32_t shift[3]; /* cells added to (x,y,z) before the window split; 0 <= shift < win */
  int32_t tau;      /* set size: slots per set                                         */
  int32_t batch;    /* frames in the call; b is the top digit of the window key        */
  int32_t axis;     /* inner-window order: 0 = x,y,z most-to-least significant (X-axis
                       main order), 1 = y,x,z (Y-axis main order).  2..5: the baselines of
                       the set-partition ablation (Sec. 4.4), each of them a different
                       numbering of the voxels inside a window: 2, 3 "Random" = order 0, 1 with the window's V
                       cells shuffled, key -> (key*mul + add) mod V, mul = the smallest integer
                       >= floor(0.618 V) + (axis odd) coprime to V, add = V/3 + (axis odd)
                       (V <= 65536); 4, 5 "Sparse" = order 0, 1 with the ranks re-dealt: the
                       voxel of rank d goes behind all voxels of a smaller d mod S, so every
                       subset spreads over the whole window.  ("Regional" is order 0 in both
                       layers of a block.)  dsvt_partition_xy and _xy_multi take an even
                       value and produce the pair (axis, axis + 1).                       */
} dsvt_part_cfg;

/* Host-only.  Upper bound on the number of sets, floor(N/tau) + min(N, #windows), on the number
 * of workgroup tiles (see dsvt_maps), and the bytes of scratch dsvt_partition or dsvt_partition_xy
 * needs for n_voxels voxels.  Any output may be NULL. */
int dsvt_partition_bound(const dsvt_part_cfg* cfg, int32_t n_voxels, int32_t* max_sets, int32_t* max_tiles,
                         size_t* ws_bytes);

/* Work list for the layer kernels, written by dsvt_partition (all [device], caller-owned).  The sets
 * are cut into tiles: runs of consecutive sets whose distinct voxels (every set padded to a multiple
 * of 4 rows) fit one 96-row workgroup tile.
 *   tile_first [max_tiles+1]     tile t covers sets tile_first[t] .. tile_first[t+1]-1
 *   n_tiles    scalar            number of tiles (<= max_tiles)
 *   tile_order [max_tiles]       tiles in launch order (most rows first)
 *   tile_desc  [max_tiles][256]  (8-byte aligned) per tile in launch order: [0] rows, [1] sets, [2+s] first row and
 *                                [26+s] distinct voxels of its s-th set, [64+2r] voxel of row r (-1 =
 *                                padding), [65+2r] (slots holding that voxel << 24) | position code
 *                                (x*(2W-1) + y)*(2H-1) + z.  The arrays need no clearing: every
 *                                entry of the first n_tiles descriptors that a kernel reads is
 *                                written by the call; the rest keeps what it held.
 * Needs tau <= 96, grid[0]*(2W-1)*(2H-1) < 2^24 and max_tiles of at least the bound dsvt_partition_bound
 * reports (with fewer, the sets past the last tile -- or, in a frame of more than 16,384 sets, all sets -- get
 * none, their voxels are not processed by a layer, and the partition sets DSVT_ST_TILE_OVERFLOW in *status).
 * Tiles hold 100 - 4*ceil(tau/4) rows on average; a frame whose tiles would not occupy the 256 compute
 * units once is cut into more, shorter tiles, and a frame of several rounds over the compute units gets tiles
 * filled as far as their sets go (up to 96 rows) when that saves a round or the frame has many rounds. */
typedef struct {
  int32_t max_tiles;
  int32_t *tile_first, *n_tiles, *tile_order, *tile_desc;
} dsvt_tile_list;

/* Builds the slot maps of one (window configuration, axis).
 *   window key  = ((b*nWx + (x+sx)/L)*nWy + (y+sy)/W)*nWz + (z+sz)/H, nW* = ceil((grid+shift)/win)
 *   per window with N voxels: S = ceil(N/tau) sets (Eq. 2); slot k of its j-th set holds the
 *   voxel of inner-window rank floor((j*tau+k)*N / (S*tau)) (Eq. 3, exact integer floor).
 *   Windows are taken in ascending key, sets of a window in ascending j.
 * coords     [device] int32 [n_voxels,4]
 * set_inds   [device] int32 [max_sets,tau] out: voxel index per slot; rows >= *n_sets untouched
 * voxel_slot [device] int32 [n_voxels]     out: smallest flat slot s*tau+k that holds the voxel
 * n_sets     [device] int32 scalar         out: total number of sets
 * set_win    [device] int32 [max_sets]     out: window key of every set; may be NULL
 * tiles      [host]   work list to fill (see dsvt_tile_list); may be NULL
 * ws         [device] at least the bytes dsvt_partition_bound reports, prepared by dsvt_partition_ws_init.
 *            Not plain scratch: part of it is an occupancy bitmap that every call finds zero and leaves
 *            zero (clearing it per call would put one more launch in front of every frame), so the
 *            buffer must stay untouched between calls; calls that share a ws must not overlap
 *            (n_voxels may change from call to call, up to the count the buffer was sized for).  A
 *            call on a ws that was not prepared for this geometry marks nothing, reports *n_sets = 0
 *            and sets DSVT_ST_WS_STATE in *status.
 * status     [device] int32 word, OR-ed with DSVT_ST_* bits (the caller zeroes it)
 * Errors: DSVT_EINVAL (NULL pointer, non-positive size, shift outside [0,win), axis outside 0..5,
 * key space of 2^31 or more cells), DSVT_ENOSPC (ws_bytes too small), DSVT_EUNSUPPORTED (a work
 * list asked for outside its limits), DSVT_EHIP. */
int dsvt_partition(const dsvt_part_cfg* cfg, const int32_t* coords, int32_t n_voxels,
                   int32_t* set_inds, int32_t* voxel_slot, int32_t* n_sets, int32_t max_sets,
                   int32_t* set_win, const dsvt_tile_list* tiles,
                   void* ws, size_t ws_bytes, int32_t* status, void* stream);

/* Prepares ws for dsvt_partition / dsvt_partition_xy calls with this cfg geometry (grid, window,
 * batch; shift, tau and axis may change freely) and n_voxels: zeroes the occupancy bitmap and writes
 * the header the kernels check.  Once per buffer, again only if the geometry changes or something
 * else wrote to the buffer.  Asynchronous on stream.  Errors: DSVT_EINVAL, DSVT_ENOSPC, DSVT_EHIP. */
int dsvt_partition_ws_init(const dsvt_part_cfg* cfg, int32_t n_voxels, void* ws, size_t ws_bytes, void* stream);

/* Both rotated partitions of one window configuration (Sec. 3.2: a block's first layer takes the sets
 * in X-axis inner order, its second in Y-axis order) in one pass over the voxels.  The windows, the
 * number of sets per window (Eq. 2) and hence n_sets, set_win and the tile boundaries are the same for
 * both; only the order of the voxels inside a window differs.  cfg->axis is the first order of the pair and must be
 * even: 0 for the X-/Y-axis pair, 2 or 4 for the pairs of the ablation's baselines (DSVT_EINVAL otherwise).  Arguments as for
 * dsvt_partition, with one set_inds and voxel_slot per axis; `tiles` receives the common tile_first,
 * n_tiles and tile_order and the X-axis descriptors, tile_desc_y [device, max_tiles*256 int32] the
 * Y-axis descriptors (required when tiles is given).  The maps of the Y-axis layer are then
 * {set_inds_y, voxel_slot_y, n_sets, {max_tiles, tile_first, n_tiles, tile_order, tile_desc_y}}.
 * Results are identical to two dsvt_partition calls with axis cfg->axis and cfg->axis + 1.  Same errors. */
int dsvt_partition_xy(const dsvt_part_cfg* cfg, const int32_t* coords, int32_t n_voxels,
                      int32_t* set_inds_x, int32_t* set_inds_y, int32_t* voxel_slot_x, int32_t* voxel_slot_y,
                      int32_t* n_sets, int32_t max_sets, int32_t* set_win,
                      const dsvt_tile_list* tiles, int32_t* tile_desc_y,
                      void* ws, size_t ws_bytes, int32_t* status, void* stream);

/* The partitions of several window configurations over the same voxels in one pass: a stage computes
 * its unshifted and its shifted windows once per frame and its blocks alternate between them
 * (Sec. 3.2, window shift between consecutive blocks), so every launch handles all configurations
 * side by side and the frame waits for one chain of launches instead of one per configuration.
 * Each job is the argument list of one dsvt_partition_xy call (every job its own ws, status and
 * outputs; tiles [host] may be NULL).  At most 4 jobs.  Results are identical to n_jobs
 * dsvt_partition_xy calls.  Errors as there; DSVT_EINVAL for n_jobs outside 1..4. */
typedef struct {
  dsvt_part_cfg cfg;                        /* axis: even, as for dsvt_partition_xy */
  int32_t *set_inds_x, *set_inds_y, *voxel_slot_x, *voxel_slot_y, *n_sets, *set_win;
  int32_t max_sets;
  const dsvt_tile_list* tiles;
  int32_t* tile_desc_y;
  void* ws;
  size_t ws_bytes;
  int32_t* status;
} dsvt_xy_job;
int dsvt_partition_xy_multi(const dsvt_xy_job* jobs, int32_t n_jobs, const int32_t* coords, int32_t n_voxels,
                            void* stream);

/* The maps one layer consumes (outputs of dsvt_partition, all [device]). */
typedef struct {
  int32_t n_voxels, max_sets, tau;
  const int32_t* set_inds;   /* [max_sets,tau]                                          */
  const int32_t* voxel_slot; /* [n_voxels]; not read by the layer kernels: may be NULL   */
  const int32_t* n_sets;     /* scalar, <= max_sets                                     */
  dsvt_tile_list tiles;      /* the work list of the same dsvt_partition call, or all-NULL: the
                                kernels then take two sets per workgroup and derive the rows
                                from set_inds and coords on chip                         */
} dsvt_maps;

/* ---------------------------------------------------------------------------------------
 * One DSVT layer's parameters (appendix "Network Architecture": MHSA, residual, LN,
 * MLP C -> hidden -> C with GELU, residual, LN; Eq. 5 for PE).
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int32_t C, heads, hidden, dtype;
  const void *w_qkv; /* [3C,C] rows: Q outputs, then K, then V     [device] */
  const void *w_o;   /* [C,C]                                       [device] */
  const void *w_1;   /* [hidden,C]                                  [device] */
  const void *w_2;   /* [C,hidden]                                  [device] */
  const float *b_qkv, *b_o, *b_1, *b_2;            /* [3C] [C] [hidden] [C]  [device] */
  const float *ln1_g, *ln1_b, *ln2_g, *ln2_b;      /* [C] each               [device] */
  float ln_eps;
  const float* rel_bias; /* [device] [heads, (2L-1)(2W-1)(2H-1)] added to the logit of (query a,
                            key b) at index ((xa-xb+L-1)*(2W-1) + ya-yb+W-1)*(2H-1) + za-zb+H-1;
                            NULL = no positional term                                    */
  int32_t win[3];        /* L, W, H of the window the maps were built with               */
  int32_t dup_mode;      /* 0: a slot repeating its predecessor's voxel is masked as a key
                               (sentence after Eq. 3); 1: repeated slots stay as keys    */
  const void* packed;    /* [device] the four matrices re-ordered for the matrix cores by
                            dsvt_layer_pack; the layer kernels read the matrices only from here */
} dsvt_layer_w;

/* Supported shapes: (C,heads,hidden) = (64,4,128) in F32 or BF16, (128,8,256) and (192,8,384) in BF16,
 * tau <= 96 (<= 64 for maps without a tile list); anything else returns DSVT_EUNSUPPORTED. */

/* Weight preparation, once per layer (weights do not change between frames).
 * dsvt_layer_packed_size: host-only, bytes of the packed buffer for this layer's shape.
 * dsvt_layer_pack: enqueue the re-ordering of w_qkv, w_o, w_1, w_2 into `packed` ([device], 16-byte
 * aligned, at least that many bytes; DSVT_ENOSPC otherwise).  Afterwards set layer->packed = packed. */
int dsvt_layer_packed_size(const dsvt_layer_w* layer, size_t* bytes);
int dsvt_layer_pack(const dsvt_layer_w* layer, void* packed, size_t bytes, void* stream);

/* Host-only: scratch bytes the two calls below need (currently 0 for both; callers must still ask). */
int dsvt_set_attention_workspace_size(const dsvt_layer_w* layer, int32_t n_voxels, size_t* bytes);
int dsvt_block_workspace_size(const dsvt_layer_w* layer, int32_t n_voxels, size_t* bytes);

/* y = MHSA over every set (Eq. 5, first two lines: INDEX, then attention with PE), out-projected
 * and returned per voxel; no residual, LN or MLP.
 * coords [device] int32 [N,4]; x [device] [N,C] in; y [device] [N,C] out (must not alias x). */
int dsvt_set_attention(const dsvt_layer_w* layer, const dsvt_maps* maps, const int32_t* coords,
                       const void* x, void* y, void* ws, size_t ws_bytes, void* stream);

/* One DSVT block (Eq. 5, Fig. 3): the full layer with maps[0] (X-axis partition), then the full
 * layer with maps[1] (Y-axis partition).  x_out [device] [N,C] may be x_in itself. */
int dsvt_block(const dsvt_layer_w layer[2], const dsvt_maps maps[2], const int32_t* coords,
               const void* x_in, void* x_out, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Attention-style 3D pooling (Sec. 3.3, Eq. 6-7).
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int32_t grid[3];  /* input cells X, Y, Z                                              */
  int32_t pool[3];  /* region l, w, h in cells; l*w*h <= 8                               */
  int32_t batch, C, heads, dtype;
  const void *w_q, *w_k, *w_v, *w_o;             /* [C,C] each   [device] */
  const float *b_q, *b_k, *b_v, *b_o, *ln_g, *ln_b; /* [C] each  [device] */
  float ln_eps;
  int32_t mask_empty; /* 1: keys/values are the region's occupied voxels; 0: all l*w*h slots,
                         holes carrying zero features (so their key/value are the biases) */
  const void* packed; /* [device] matrices and key/value biases re-ordered by dsvt_pool_pack; the
                         kernels read them only from here */
} dsvt_pool_cfg;

/* Weight preparation, once per pooling module: as dsvt_layer_packed_size / dsvt_layer_pack. */
int dsvt_pool_packed_size(const dsvt_pool_cfg* cfg, size_t* bytes);
int dsvt_pool_pack(const dsvt_pool_cfg* cfg, void* packed, size_t bytes, void* stream);

int dsvt_attn_pool_workspace_size(const dsvt_pool_cfg* cfg, int32_t n_voxels, size_t* bytes);

/* Every non-empty region (b, x/l, y/w, z/h) becomes one output voxel, in ascending key
 * ((b*Xp + x/l)*Yp + y/w)*Zp + z/h.  P = channel-wise max over the region's voxels (Eq. 6) is the
 * query; out = LN(P + Attn(Q = P, KV = region) W_o + b_o) (Eq. 7).
 * out_coords [device] int32 [n_voxels,4] (first *n_out rows written: b, x/l, y/w, z/h)
 * out        [device] [n_voxels,C]       (first *n_out rows written)
 * n_out      [device] int32 scalar
 * Supported: (C,heads) = (64,4) in F32 or BF16, (128,8) and (192,8) in BF16; l*w*h <= 8; out must not alias x.
 * status gets DSVT_ST_COORD_RANGE for a coordinate outside the grid (that voxel is skipped). */
int dsvt_attn_pool(const dsvt_pool_cfg* cfg, const int32_t* coords, const void* x, int32_t n_voxels,
                   int32_t* out_coords, void* out, int32_t* n_out,
                   void* ws, size_t ws_bytes, int32_t* status, void* stream);

/* dsvt_attn_pool for callers that cannot allocate device memory or carry a workspace around: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as dsvt_attn_pool, without `ws`: the scratch (occupancy bitmap, its prefix, the
 * dense slot table) is an array of DSVT_POOL_STATIC_SCRATCH_BYTES built into the library, one copy per
 * GPU, held from the moment the library is loaded until the process ends.  The call allocates and
 * frees nothing.  DSVT_ENOSPC when dsvt_attn_pool_workspace_size(cfg, n_voxels) exceeds that size
 * (8 MiB: e.g. 300,000 voxels in regions of 4 cells on a 468 x 468 x 32 grid).  Every call on a GPU uses
 * that GPU's one array: calls on different streams of one GPU must not overlap (they would race on
 * it); what the array held before does not matter (each call clears what it reads).  The first call
 * on a device looks the array's address up (no allocation; make it outside graph capture). */
#define DSVT_POOL_STATIC_SCRATCH_BYTES (8u << 20)
int dsvt_attn_pool_static(const dsvt_pool_cfg* cfg, const int32_t* coords, const void* x, int32_t n_voxels,
                          int32_t* out_coords, void* out, int32_t* n_out, int32_t* status, void* stream);

/* ---------------------------------------------------------------------------------------
 * Bird's-eye-view map (Sec. 3.1, overview: the step after the last block, which lays the sparse voxel
 * rows out as the dense map the 2D backbone works on).
 * out [device] [batch, X, Y, Z, C] of dtype, channels last (Z = 1 for pillars and for the voxel
 * variant after its last pooling: a [batch, X, Y, C] image); the whole of it is written: the
 * voxel's row at its cell, zeros elsewhere.  coords [device] int32 [n_voxels,4] = (b, x, y, z),
 * unique; x [device] [n_voxels, C].  C * sizeof(dtype) must be a multiple of 16, all three
 * pointers 16-byte aligned, out must not alias x.  A coordinate outside the grid sets
 * DSVT_ST_COORD_RANGE in *status [device] and that voxel is skipped.  Asynchronous on stream.
 * ------------------------------------------------------------------------------------ */
int dsvt_bev_scatter(const int32_t* coords, const void* x, int32_t n_voxels, int32_t C, int32_t dtype,
                     int32_t batch, const int32_t grid[3], void* out, int32_t* status, void* stream);

/* ---------------------------------------------------------------------------------------
 * Voxel feature encoding (Sec. 3.1, overview): points are binned into the occupied cells of the grid
 * and reduced per cell to one feature row, the token the first block takes.  The paper names
 * the step and cites earlier pillar encoders; built here is the plain member of that family:
 *   x[v] = max over the points p of voxel v of (w f_p + b), channel by channel, then max(., 0)
 *   if relu; w == NULL: x[v] = max over p of f_p (C == f_in).
 * A point's cell along an axis is t = (p - range_min) / voxel_size evaluated in float32, one
 * rounded operation each; the point lies in the grid iff 0 <= t < grid (a NaN does not), its cell
 * is t truncated.  Points outside the grid, or with a batch index outside [0, batch), are ignored.
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int32_t grid[3];      /* cells along X, Y, Z                                             */
  int32_t batch;        /* frames in the call                                              */
  float range_min[3];   /* position of the corner of cell (0,0,0)                          */
  float voxel_size[3];  /* cell edge lengths, > 0                                          */
  int32_t f_in;         /* floats per point, 3 <= f_in <= 16; the first three are x, y, z   */
  int32_t C;            /* output channels, <= 512                                         */
  int32_t dtype;        /* element type of the output rows x                               */
  const float* w;       /* [C, f_in] [device] or NULL                                      */
  const float* b;       /* [C] [device] or NULL                                            */
  int32_t relu;
} dsvt_vfe_cfg;

int dsvt_vfe_workspace_size(const dsvt_vfe_cfg* cfg, int32_t n_points, int32_t max_voxels, size_t* bytes);

/* points      [device] float [n_points, f_in]
 * point_batch [device] int32 [n_points] frame of each point; may be NULL when batch == 1
 * coords      [device] int32 [max_voxels,4], 16-byte aligned: (b, x, y, z) of the non-empty voxels in
 *             ascending key ((b*X + x)*Y + y)*Z + z -- the rows dsvt_partition and dsvt_block take
 * x           [device] [max_voxels, C] of dtype: their features
 * n_voxels    [device] int32 scalar: the number of non-empty voxels (may exceed max_voxels, see below)
 * ws          [device] scratch of dsvt_vfe_workspace_size bytes, 16-byte aligned; no state is kept in it
 * status gets DSVT_ST_VOXEL_OVERFLOW when there are more than max_voxels non-empty voxels: the first
 * max_voxels rows are then complete and the rest is dropped.  batch*X*Y*Z must be below 2^31.
 * Asynchronous on stream.  The result does not depend on the order of the points. */
int dsvt_vfe(const dsvt_vfe_cfg* cfg, const float* points, const int32_t* point_batch, int32_t n_points,
             int32_t* coords, void* x, int32_t* n_voxels, int32_t max_voxels, void* ws, size_t ws_bytes,
             int32_t* status, void* stream);

/* ---------------------------------------------------------------------------------------
 * Instrumentation for benchmarks (not part of the method): per-kernel time from hipEvent pairs
 * recorded around every launch while enabled (launches of one kernel that follow one another on a
 * stream share a pair: begin before the first, end after the last).  Host-only; not thread-safe.
 * dsvt_prof_enable creates events for up to max_launches launches (later ones go unrecorded);
 * dsvt_prof_collect waits for them, fills total_ms[k] / launches[k] for the
 * dsvt_prof_kernel_count() kernel ids (names from dsvt_prof_kernel_name), destroys the events
 * and switches recording off.
 * ------------------------------------------------------------------------------------ */
int dsvt_prof_enable(int32_t max_launches);
int dsvt_prof_collect(float* total_ms /*[host]*/, int32_t* launches /*[host]*/, int32_t n_kernels);
int32_t dsvt_prof_kernel_count(void);
const char* dsvt_prof_kernel_name(int32_t id);

#ifdef __cplusplus
}
#endif
#endif /* DSVT_H */
