// dsvt_partition: rotated dynamic set partition (Sec. 3.2, Eq. 2-4) on gfx950.
//
// Voxel cells are unique, so the sort by (window key, inner-window key) is done without
// comparing anything: every voxel sets one bit in an occupancy bitmap laid out as
// [window][inner key], and a voxel's inner-window rank is the number of set bits before its
// own inside its window's bit range.  Per window a wavefront (or a slice of one) pop-counts
// the words and leaves a running prefix per word; one scan over the windows turns voxel and
// set counts into offsets; then every voxel writes the slots that Eq. (3) assigns to its rank:
//   floor(t*N/(S*tau)) == d   <=>   ceil(d*S*tau/N) <= t < ceil((d+1)*S*tau/N).
#include "common.h"

namespace {

constexpr uint32_t kBadKey = 0xFFFFFFFFu;
constexpr int64_t kFusedThreads = 32 * 1024;     // window-count work (windows x lanes per window) one workgroup takes on itself

struct PartGeom {
  int32_t grid[3], win[3], shift[3], nw[3];
  int32_t batch, tau, axis;
  int32_t words_per_win;   // 32-bit bitmap words per window (window volume rounded up to 32)
  int32_t n_windows;       // batch * nw[0] * nw[1] * nw[2]
};

__global__ void k_clear(uint32_t* __restrict__ words, int64_t n, int32_t* __restrict__ desc, int64_t n_desc) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) words[i] = 0u;
  if (i < n_desc) desc[i] = -1;
}

// One thread per voxel: composite key = window key * (32*words_per_win) + inner key; set its bit.
__global__ void k_mark(PartGeom g, const int4* __restrict__ coords, int32_t n, uint32_t* __restrict__ bitmap,
                       uint32_t* __restrict__ keys, int32_t* __restrict__ status) {
  int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int4 c = coords[i];                       // (b, x, y, z)
  bool ok = c.x >= 0 && c.x < g.batch && c.y >= 0 && c.y < g.grid[0] && c.z >= 0 && c.z < g.grid[1] &&
            c.w >= 0 && c.w < g.grid[2];
  if (!ok) {
    keys[i] = kBadKey;
    atomicOr(status, DSVT_ST_COORD_RANGE);
    return;
  }
  int32_t x = c.y + g.shift[0], y = c.z + g.shift[1], z = c.w + g.shift[2];
  int32_t wx = x / g.win[0], wy = y / g.win[1], wz = z / g.win[2];
  int32_t xi = x - wx * g.win[0], yi = y - wy * g.win[1], zi = z - wz * g.win[2];
  uint32_t wkey = (uint32_t)(((c.x * g.nw[0] + wx) * g.nw[1] + wy) * g.nw[2] + wz);
  uint32_t inner = g.axis == 0 ? (uint32_t)((xi * g.win[1] + yi) * g.win[2] + zi)
                               : (uint32_t)((yi * g.win[0] + xi) * g.win[2] + zi);
  uint32_t key = wkey * (uint32_t)(g.words_per_win * 32) + inner;
  uint32_t bit = 1u << (key & 31u);
  uint32_t old = atomicOr(&bitmap[key >> 5], bit);
  if (old & bit) atomicOr(status, DSVT_ST_COORD_REPEAT);
  keys[i] = key;
}

// `group` lanes (a power of two <= 64) per window: pop-count the window's words, leave in
// word_prefix[] the number of set bits in the window's earlier words, and the window total.
__device__ __forceinline__ void window_count(int32_t tid, const uint32_t* __restrict__ bitmap,
                                             uint32_t* __restrict__ word_prefix, int32_t* __restrict__ win_count,
                                             int32_t n_windows, int32_t words_per_win, int32_t group) {
  int32_t w = tid / group, lane = tid & (group - 1);
  if (w >= n_windows) return;               // whole groups leave together
  const int64_t base = (int64_t)w * words_per_win;
  uint32_t running = 0;
  for (int32_t w0 = 0; w0 < words_per_win; w0 += group) {
    int32_t j = w0 + lane;
    uint32_t v = j < words_per_win ? (uint32_t)__popc(bitmap[base + j]) : 0u;
    uint32_t incl = v;
    for (int32_t d = 1; d < group; d <<= 1) {
      uint32_t up = __shfl_up(incl, d, group);
      if (lane >= d) incl += up;
    }
    if (j < words_per_win) word_prefix[base + j] = running + incl - v;
    running += __shfl(incl, group - 1, group);
  }
  if (lane == 0) win_count[w] = (int32_t)running;
}

__global__ void k_window_count(const uint32_t* __restrict__ bitmap, uint32_t* __restrict__ word_prefix,
                               int32_t* __restrict__ win_count, int32_t n_windows, int32_t words_per_win,
                               int32_t group) {
  window_count(blockIdx.x * blockDim.x + threadIdx.x, bitmap, word_prefix, win_count, n_windows, words_per_win, group);
}

// One workgroup: exclusive scans of voxels-per-window and sets-per-window (Eq. 2).
__device__ __forceinline__ void scan_windows(const int32_t* __restrict__ win_count, int32_t* __restrict__ win_soff,
                                             int32_t n_windows, int32_t tau, int32_t max_sets,
                                             int32_t* __restrict__ n_sets, int32_t* __restrict__ status,
                                             int32_t* __restrict__ set_w, int32_t set_cap) {
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry_s;
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int32_t base = 0; base < n_windows; base += 1024) {
    int32_t w = base + tid;
    int32_t nvox = w < n_windows ? win_count[w] : 0;
    int32_t s = (nvox + tau - 1) / tau;
    int32_t incl = s;
    for (int32_t d = 1; d < 64; d <<= 1) {
      int32_t up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    int32_t before = carry_s;
    for (int32_t k = 0; k < wv; ++k) before += wave_tot[k];
    if (w < n_windows) {
      win_soff[w] = before + incl - s;
      for (int32_t j = 0; j < s; ++j)                       // window of each of its sets, for k_tiles
        if (before + incl - s + j < set_cap) set_w[before + incl - s + j] = w;
    }
    __syncthreads();
    if (tid == 1023) carry_s = before + incl;
    __syncthreads();
  }
  if (tid == 0) {
    *n_sets = carry_s;
    if (carry_s > max_sets) atomicOr(status, DSVT_ST_SET_OVERFLOW);
  }
}

__global__ void __launch_bounds__(1024) k_scan_windows(const int32_t* __restrict__ win_count,
                                                       int32_t* __restrict__ win_soff, int32_t n_windows,
                                                       int32_t tau, int32_t max_sets, int32_t* __restrict__ n_sets,
                                                       int32_t* __restrict__ status, int32_t* __restrict__ set_w,
                                                       int32_t set_cap) {
  scan_windows(win_count, win_soff, n_windows, tau, max_sets, n_sets, status, set_w, set_cap);
}

// Tile descriptor, one per workgroup tile of the layer kernels, in launch order (256 ints):
//   [0] rows R (sets padded to multiples of 4)   [1] sets ns
//   [2 + s] first row of set s                    [2 + 24 + s] distinct voxels of set s   (s < ns <= 24)
//   [64 + r] voxel of row r, -1 for padding rows  [160 + r] (multiplicity << 24) | position code of row r
constexpr int kDescInts = 256, kDescSets = 24, kDescR0 = 2, kDescNu = 2 + kDescSets, kDescVox = 64, kDescLin = 160;
constexpr int kTileRows = 96;

// Distinct voxels of the j-th set of a window with N voxels in S sets (closed form from Eq. 3).
__device__ __forceinline__ int32_t set_distinct(int64_t N, int64_t S, int64_t j, int64_t tau) {
  if (N < 32768 && S * tau < 65536) {                       // the usual case: everything fits 32-bit division
    const uint32_t n = (uint32_t)N, T = (uint32_t)(S * tau), a = (uint32_t)(j * tau);
    return (int32_t)(((a + (uint32_t)tau - 1u) * n) / T - (a * n) / T + 1u);
  }
  const int64_t lo = (j * tau * N) / (S * tau), hi = ((j * tau + tau - 1) * N) / (S * tau);
  return (int32_t)(hi - lo + 1);
}

struct TileOut {                       // all null when the caller wants no work list
  int32_t *tile_first, *n_tiles, *tile_order, *tile_desc;
  int32_t max_tiles;
};

// One workgroup: cut the set sequence into tiles for the layer kernels, order the tiles for launch
// and write the descriptor headers.  With P(s) the running sum of padded rows before set s, set s
// starts a tile when P crosses a multiple of rows_per_cut; a tile then holds at most
// rows_per_cut - 4 + pad4(tau) rows.  set_loc[s] = (descriptor slot << 7) | first row, for k_emit.
__device__ __forceinline__ void build_tiles(const int32_t* set_w, const int32_t* win_count, const int32_t* win_soff,
                                            const int32_t* n_sets_ptr, int32_t set_cap, int32_t tau, int32_t n_windows,
                                            int32_t rows_per_cut, TileOut out, int32_t* tile_rows, int32_t* tile_pos,
                                            int32_t* set_p, int32_t* set_loc) {
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry_s;
  __shared__ int32_t hist[32], running[32], wave_cnt[16][32];
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int32_t n_sets = *n_sets_ptr;
  n_sets = n_sets < set_cap ? n_sets : set_cap;
  if (n_sets <= 0) {
    if (tid == 0) { *out.n_tiles = 0; out.tile_first[0] = 0; }
    return;
  }
  if (tid == 0) carry_s = 0;
  __syncthreads();
  // pass 1: padded rows per set, their running sum, the tile of every set
  for (int32_t base = 0; base < n_sets; base += 1024) {
    const int32_t s = base + tid;
    int32_t rows = 0;
    if (s < n_sets) {
      int32_t w = set_w[s];
      w = w < 0 ? 0 : (w >= n_windows ? n_windows - 1 : w);
      const int64_t N = win_count[w] > 0 ? win_count[w] : 1, S = (N + tau - 1) / tau;
      rows = (set_distinct(N, S, s - win_soff[w], tau) + 3) & ~3;
      rows = rows > kTileRows ? kTileRows : (rows < 4 ? 4 : rows);
    }
    int32_t incl = rows;
    for (int32_t d = 1; d < 64; d <<= 1) {
      int32_t up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    int32_t before = carry_s;
    for (int32_t k = 0; k < wv; ++k) before += wave_tot[k];
    const int32_t P = before + incl - rows;                 // rows before set s
    if (s < n_sets) {
      set_p[s] = P;
      set_loc[s] = -1;                                      // set in pass 4
      if (s == n_sets - 1) set_p[n_sets] = P + rows;
    }
    __syncthreads();
    if (tid == 1023) carry_s = before + incl;
    __syncthreads();
  }
  // pass 2: tile boundaries.  A set starts a tile when the running row count crosses a multiple of
  // rows_per_cut between its predecessor's start and its own; tiles are numbered by counting these
  // starts (a scan), so none is empty even when one set is longer than rows_per_cut.  A tile then
  // holds at most rows_per_cut - 4 + pad4(tau) <= 96 rows.
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int32_t base = 0; base < n_sets; base += 1024) {
    const int32_t s = base + tid;
    const bool first = s < n_sets && (s == 0 || set_p[s - 1] / rows_per_cut != set_p[s] / rows_per_cut);
    int32_t incl = first ? 1 : 0;
    for (int32_t d = 1; d < 64; d <<= 1) {
      int32_t up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    int32_t before = carry_s;
    for (int32_t k = 0; k < wv; ++k) before += wave_tot[k];
    const int32_t tile = before + incl - 1;                   // tile of set s
    if (s < n_sets) {
      set_loc[s] = tile;                                      // until pass 4 replaces it
      if (first && tile < out.max_tiles) { out.tile_first[tile] = s; tile_rows[tile] = set_p[s]; }
      if (s == n_sets - 1) {
        const int32_t nt = tile + 1 < out.max_tiles ? tile + 1 : out.max_tiles;
        *out.n_tiles = nt;
        out.tile_first[nt] = n_sets;
        tile_rows[nt] = set_p[n_sets];
      }
    }
    __syncthreads();
    if (tid == 1023) carry_s = before + incl;
    __syncthreads();
  }
  __threadfence_block();
  __syncthreads();
  // pass 3: launch order = tiles with more rows first (a stable counting sort on rows / 4), so
  // that the short tiles fill the tail of the launch
  const int32_t nt = *out.n_tiles;
  if (tid < 32) hist[tid] = 0;
  __syncthreads();
  for (int32_t base = 0; base < nt; base += 1024) {
    const int32_t t = base + tid;
    if (t < nt) {
      int32_t b = 24 - (tile_rows[t + 1] - tile_rows[t]) / 4;
      b = b < 0 ? 0 : (b > 31 ? 31 : b);
      atomicAdd(&hist[b], 1);
    }
  }
  __syncthreads();
  if (tid == 0) { int32_t acc = 0; for (int32_t b = 0; b < 32; ++b) { running[b] = acc; acc += hist[b]; } }
  __syncthreads();
  for (int32_t base = 0; base < nt; base += 1024) {
    const int32_t t = base + tid;
    int32_t b = -1;
    if (t < nt) {
      b = 24 - (tile_rows[t + 1] - tile_rows[t]) / 4;
      b = b < 0 ? 0 : (b > 31 ? 31 : b);
    }
    for (int32_t k = lane; k < 32; k += 64) wave_cnt[wv][k] = 0;
    int32_t rank = 0;                                       // among this wavefront's lanes of the same bucket
    unsigned long long todo = __ballot(b >= 0);
    while (todo) {
      const int32_t leader = __ffsll((long long)todo) - 1;
      const int32_t lb = __shfl(b, leader, 64);
      const unsigned long long same = __ballot(b == lb);
      if (b == lb) rank = __popcll(same & ((1ull << lane) - 1ull));
      if (lane == leader) wave_cnt[wv][lb] = __popcll(same);
      todo &= ~same;
    }
    __syncthreads();
    if (b >= 0) {
      int32_t pos = running[b] + rank;
      for (int32_t k = 0; k < wv; ++k) pos += wave_cnt[k][b];
      out.tile_order[pos] = t;
      tile_pos[t] = pos;
      int32_t* d = out.tile_desc + (int64_t)pos * kDescInts;    // descriptor header of launch slot pos
      d[0] = tile_rows[t + 1] - tile_rows[t];
      d[1] = out.tile_first[t + 1] - out.tile_first[t];
    }
    __syncthreads();
    if (tid < 32) { int32_t add = 0; for (int32_t k = 0; k < 16; ++k) add += wave_cnt[k][tid]; running[tid] += add; }
    __syncthreads();
  }
  // pass 4: per set, its descriptor slot, first row and distinct count
  for (int32_t base = 0; base < n_sets; base += 1024) {
    const int32_t s = base + tid;
    if (s < n_sets) {
      const int32_t t = set_loc[s];
      int32_t loc = -1;
      if (t >= 0 && t < nt) {
        const int32_t pos = tile_pos[t], ls = s - out.tile_first[t], r0 = set_p[s] - tile_rows[t];
        int32_t w = set_w[s];
        w = w < 0 ? 0 : (w >= n_windows ? n_windows - 1 : w);
        const int64_t N = win_count[w] > 0 ? win_count[w] : 1, S = (N + tau - 1) / tau;
        if (ls >= 0 && ls < kDescSets && r0 >= 0 && r0 <= kTileRows - 4) {
          int32_t* d = out.tile_desc + (int64_t)pos * kDescInts;
          d[kDescR0 + ls] = r0;
          d[kDescNu + ls] = set_distinct(N, S, s - win_soff[w], tau);
          loc = (pos << 7) | r0;
        }
      }
      set_loc[s] = loc;
    }
  }
}

__global__ void __launch_bounds__(1024) k_tiles(const int32_t* set_w, const int32_t* win_count, const int32_t* win_soff,
                                                const int32_t* n_sets_ptr, int32_t set_cap, int32_t tau, int32_t n_windows,
                                                int32_t rows_per_cut, TileOut out, int32_t* tile_rows, int32_t* tile_pos,
                                                int32_t* set_p, int32_t* set_loc) {
  build_tiles(set_w, win_count, win_soff, n_sets_ptr, set_cap, tau, n_windows, rows_per_cut, out, tile_rows, tile_pos, set_p,
              set_loc);
}

// Small frames: the three steps between k_mark and k_emit in one workgroup and one launch (each is a
// few microseconds of work; as separate launches their start-up and the gaps between them are most
// of a partition's latency, which the first layer of a frame has to wait for).
__global__ void __launch_bounds__(1024) k_count_scan_tiles(const uint32_t* bitmap, uint32_t* word_prefix, int32_t* win_count,
                                                           int32_t* win_soff, int32_t n_windows, int32_t words_per_win,
                                                           int32_t group, int32_t tau, int32_t max_sets, int32_t* n_sets,
                                                           int32_t* status, int32_t* set_w, int32_t set_bound,
                                                           int32_t set_cap, int32_t rows_per_cut, TileOut out,
                                                           int32_t* tile_rows, int32_t* tile_pos, int32_t* set_p,
                                                           int32_t* set_loc) {
  if (words_per_win <= 8) {
    // a thread per window: its few words are independent loads, the prefix a short serial sum
    for (int32_t w = threadIdx.x; w < n_windows; w += 1024) {
      const int64_t base = (int64_t)w * words_per_win;
      uint32_t v[8];
#pragma unroll
      for (int32_t j = 0; j < 8; ++j) v[j] = j < words_per_win ? bitmap[base + j] : 0u;
      uint32_t running = 0;
#pragma unroll
      for (int32_t j = 0; j < 8; ++j) {
        if (j < words_per_win) word_prefix[base + j] = running;
        running += (uint32_t)__popc(v[j]);
      }
      win_count[w] = (int32_t)running;
    }
  } else {
    const int64_t n_threads = (int64_t)n_windows * group;
    for (int64_t base = 0; base < n_threads; base += 1024)      // 1024 is a multiple of every group size
      window_count((int32_t)(base + threadIdx.x), bitmap, word_prefix, win_count, n_windows, words_per_win, group);
  }
  __threadfence_block();
  __syncthreads();
  scan_windows(win_count, win_soff, n_windows, tau, max_sets, n_sets, status, set_w, set_bound);
  __threadfence_block();
  __syncthreads();
  if (out.tile_desc != nullptr)
    build_tiles(set_w, win_count, win_soff, n_sets, set_cap, tau, n_windows, rows_per_cut, out, tile_rows, tile_pos, set_p,
                set_loc);
}

// One thread per voxel: rank d inside its window, then the slots t with floor(t*N/(S*tau)) == d;
// with a work list also the voxel's row of its tile descriptor.
__global__ void k_emit(PartGeom g, const int4* __restrict__ coords, const uint32_t* __restrict__ keys, int32_t n,
                       const uint32_t* __restrict__ bitmap, const uint32_t* __restrict__ word_prefix,
                       const int32_t* __restrict__ win_count, const int32_t* __restrict__ win_soff, int32_t max_sets,
                       int32_t* __restrict__ set_inds, int32_t* __restrict__ voxel_slot, int32_t* __restrict__ set_win,
                       const int32_t* __restrict__ set_loc, int32_t* __restrict__ tile_desc, int32_t n_desc_slots) {
  int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint32_t key = keys[i];
  if (key == kBadKey) { voxel_slot[i] = -1; return; }
  const int32_t tau = g.tau;
  uint32_t word = key >> 5, bit = key & 31u;
  int32_t w = (int32_t)(word / (uint32_t)g.words_per_win);
  int64_t d = word_prefix[word] + (uint32_t)__popc(bitmap[word] & ((1u << bit) - 1u));
  int64_t N = win_count[w];
  int64_t S = (N + tau - 1) / tau, T = S * tau;
  int64_t t_lo, t_hi, first_d;                               // first_d: rank of the first voxel of this voxel's first set
  if (N > 0 && N < 32768 && T < 65536) {                     // the usual case: 32-bit division
    const uint32_t n = (uint32_t)N, tt = (uint32_t)T, dd = (uint32_t)d;
    const uint32_t lo = (dd * tt + n - 1u) / n, hi = ((dd + 1u) * tt + n - 1u) / n;
    t_lo = lo; t_hi = hi;
    first_d = ((lo / (uint32_t)tau) * (uint32_t)tau * n) / tt;
  } else {
    t_lo = (d * T + N - 1) / N; t_hi = ((d + 1) * T + N - 1) / N;
    first_d = ((t_lo / tau) * tau * N) / T;
  }
  int64_t base = (int64_t)win_soff[w] * tau, cap = (int64_t)max_sets * tau;
  voxel_slot[i] = (int32_t)(base + t_lo);
  const int32_t j_first = (int32_t)t_lo / tau;               // (t < S * tau and slots < max_sets * tau fit 32 bits)
  int32_t next_set_start = (int32_t)t_lo == j_first * tau ? (int32_t)t_lo : (j_first + 1) * tau;
  for (int32_t t = (int32_t)t_lo; t < (int32_t)t_hi; ++t) {
    const int64_t slot = base + t;
    if (slot >= cap) break;
    set_inds[slot] = i;
    if (t == next_set_start) { set_win[win_soff[w] + t / tau] = w; next_set_start += tau; }
  }
  if (tile_desc != nullptr) {
    const int64_t j = j_first, s = win_soff[w] + j;
    if (s < max_sets) {
      const int32_t loc = set_loc[s];
      const int32_t slot = loc >> 7, row = (loc & 127) + (int32_t)(d - first_d);
      if (slot >= 0 && slot < n_desc_slots && row < kTileRows) {
        const int4 c = coords[i];
        const int32_t lin = (c.y * (2 * g.win[1] - 1) + c.z) * (2 * g.win[2] - 1) + c.w;
        int32_t* dd = tile_desc + (int64_t)slot * kDescInts;
        dd[kDescVox + row] = i;
        dd[kDescLin + row] = (int32_t)((uint32_t)lin | ((uint32_t)(t_hi - t_lo) << 24));
      }
    }
  }
}

struct PartPlan {
  PartGeom g;
  size_t off_bitmap, off_prefix, off_count, off_soff, off_keys, off_setwin, off_tilerows, off_tilepos, off_setp, off_setloc, total;
  bool desc_ok;
  int64_t n_words;
  int32_t set_bound, tile_bound, rows_per_cut;
};

int make_plan(const dsvt_part_cfg* cfg, int32_t n_voxels, PartPlan* p) {
  if (cfg == nullptr || n_voxels <= 0 || cfg->tau <= 0 || cfg->batch <= 0 || (cfg->axis != 0 && cfg->axis != 1))
    return DSVT_EINVAL;
  PartGeom& g = p->g;
  int64_t vol = 1, nwin = cfg->batch;
  for (int a = 0; a < 3; ++a) {
    if (cfg->grid[a] <= 0 || cfg->win[a] <= 0 || cfg->shift[a] < 0 || cfg->shift[a] >= cfg->win[a]) return DSVT_EINVAL;
    g.grid[a] = cfg->grid[a]; g.win[a] = cfg->win[a]; g.shift[a] = cfg->shift[a];
    g.nw[a] = (int32_t)dsvt_ceil_div((int64_t)cfg->grid[a] + cfg->shift[a], cfg->win[a]);
    vol *= cfg->win[a];
    nwin *= g.nw[a];
    if (vol >= (1ll << 31) || nwin >= (1ll << 31)) return DSVT_EINVAL;
  }
  g.batch = cfg->batch; g.tau = cfg->tau; g.axis = cfg->axis;
  int64_t wpw = dsvt_ceil_div(vol, 32);
  if (nwin * wpw * 32 >= (1ll << 31)) return DSVT_EINVAL;   // composite keys are 32-bit
  g.words_per_win = (int32_t)wpw;
  g.n_windows = (int32_t)nwin;
  p->n_words = nwin * wpw;
  size_t o = 0;
  p->off_bitmap = o; o = dsvt_align_up(o + (size_t)p->n_words * 4, 256);
  p->off_prefix = o; o = dsvt_align_up(o + (size_t)p->n_words * 4, 256);
  p->off_count = o;  o = dsvt_align_up(o + (size_t)nwin * 4, 256);
  p->off_soff = o;   o = dsvt_align_up(o + (size_t)nwin * 4, 256);
  p->off_keys = o;   o = dsvt_align_up(o + (size_t)n_voxels * 4, 256);
  const int64_t bound = n_voxels / cfg->tau + (n_voxels < nwin ? n_voxels : nwin);
  if (bound * cfg->tau >= (1ll << 31)) return DSVT_EINVAL;
  p->set_bound = (int32_t)bound;
  p->off_setwin = o; o = dsvt_align_up(o + (size_t)bound * 4, 256);
  // tiles of the layer kernels: 96 rows, every set padded to a multiple of 4 rows
  const int64_t pad_tau = (cfg->tau + 3) & ~3;
  p->rows_per_cut = (int32_t)(100 - pad_tau);
  p->tile_bound = p->rows_per_cut > 0 ? (int32_t)((n_voxels + 3 * bound) / p->rows_per_cut + 1) : 0;
  p->off_tilerows = o; o = dsvt_align_up(o + (size_t)(p->tile_bound + 1) * 4, 256);
  p->off_tilepos = o;  o = dsvt_align_up(o + (size_t)(p->tile_bound + 1) * 4, 256);
  p->off_setp = o;     o = dsvt_align_up(o + (size_t)(bound + 1) * 4, 256);
  p->off_setloc = o;   o = dsvt_align_up(o + (size_t)(bound + 1) * 4, 256);
  // a descriptor packs (slot << 7 | row) and (multiplicity << 24 | position code) into 32 bits
  p->desc_ok = p->rows_per_cut >= 4 && p->tile_bound < (1 << 23) &&
               (int64_t)cfg->grid[0] * (2 * cfg->win[1] - 1) * (2 * cfg->win[2] - 1) < (1 << 24) && cfg->tau < 128;
  p->total = o;
  return DSVT_OK;
}

}  // namespace

extern "C" int dsvt_partition_bound(const dsvt_part_cfg* cfg, int32_t n_voxels, int32_t* max_sets, int32_t* max_tiles,
                                    size_t* ws_bytes) {
  PartPlan p;
  int rc = make_plan(cfg, n_voxels, &p);
  if (rc != DSVT_OK) return rc;
  if (max_sets) *max_sets = p.set_bound;
  if (max_tiles) *max_tiles = p.tile_bound;
  if (ws_bytes) *ws_bytes = p.total;
  return DSVT_OK;
}

extern "C" int dsvt_partition(const dsvt_part_cfg* cfg, const int32_t* coords, int32_t n_voxels, int32_t* set_inds,
                              int32_t* voxel_slot, int32_t* n_sets, int32_t max_sets, int32_t* set_win,
                              const dsvt_tile_list* tiles, void* ws, size_t ws_bytes, int32_t* status, void* stream) {
  PartPlan p;
  int rc = make_plan(cfg, n_voxels, &p);
  if (rc != DSVT_OK) return rc;
  if (!coords || !set_inds || !voxel_slot || !n_sets || !ws || !status || max_sets <= 0) return DSVT_EINVAL;
  if ((int64_t)max_sets * cfg->tau >= (1ll << 31)) return DSVT_EINVAL;
  if (ws_bytes < p.total) return DSVT_ENOSPC;
  TileOut tout = {nullptr, nullptr, nullptr, nullptr, 0};
  if (tiles != nullptr) {
    if (!tiles->tile_first || !tiles->n_tiles || !tiles->tile_order || !tiles->tile_desc || tiles->max_tiles <= 0) return DSVT_EINVAL;
    if (!p.desc_ok) return DSVT_EUNSUPPORTED;
    tout.tile_first = tiles->tile_first; tout.n_tiles = tiles->n_tiles; tout.tile_order = tiles->tile_order;
    tout.tile_desc = tiles->tile_desc;
    tout.max_tiles = tiles->max_tiles < p.tile_bound ? tiles->max_tiles : p.tile_bound;   // scratch is sized for the bound
  }
  // window key of every set: the caller's array, or scratch when it is not wanted
  int32_t set_cap = max_sets < p.set_bound ? max_sets : p.set_bound;
  if (set_win == nullptr) set_win = (int32_t*)((char*)ws + p.off_setwin);   // k_emit rewrites the same values there
  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)ws;
  uint32_t* bitmap = (uint32_t*)(base + p.off_bitmap);
  uint32_t* prefix = (uint32_t*)(base + p.off_prefix);
  int32_t* count = (int32_t*)(base + p.off_count);
  int32_t* soff = (int32_t*)(base + p.off_soff);
  uint32_t* keys = (uint32_t*)(base + p.off_keys);
  int32_t* set_loc = (int32_t*)(base + p.off_setloc);
  const int tb = 256;
  {
    dsvt_prof_scope ps(DSVT_K_PART_CLEAR, st);
    const int64_t n_desc = (int64_t)tout.max_tiles * kDescInts;
    const int64_t n_clear = p.n_words > n_desc ? p.n_words : n_desc;
    k_clear<<<(unsigned)dsvt_ceil_div(n_clear, tb), tb, 0, st>>>(bitmap, p.n_words, tout.tile_desc, n_desc);
  }
  {
    dsvt_prof_scope ps(DSVT_K_PART_MARK, st);
    k_mark<<<(unsigned)dsvt_ceil_div(n_voxels, tb), tb, 0, st>>>(p.g, (const int4*)coords, n_voxels, bitmap, keys, status);
  }
  int32_t group = 1;
  while (group < 64 && group < p.g.words_per_win) group <<= 1;
  if ((int64_t)p.g.n_windows * group <= kFusedThreads) {
    dsvt_prof_scope ps(DSVT_K_PART_TILES, st);
    k_count_scan_tiles<<<1, 1024, 0, st>>>(bitmap, prefix, count, soff, p.g.n_windows, p.g.words_per_win, group, cfg->tau,
                                           max_sets, n_sets, status, (int32_t*)(base + p.off_setwin), p.set_bound, set_cap,
                                           p.rows_per_cut, tout, (int32_t*)(base + p.off_tilerows),
                                           (int32_t*)(base + p.off_tilepos), (int32_t*)(base + p.off_setp), set_loc);
  } else {
    {
      dsvt_prof_scope ps(DSVT_K_PART_COUNT, st);
      int64_t threads = (int64_t)p.g.n_windows * group;
      k_window_count<<<(unsigned)dsvt_ceil_div(threads, tb), tb, 0, st>>>(bitmap, prefix, count, p.g.n_windows,
                                                                          p.g.words_per_win, group);
    }
    {
      dsvt_prof_scope ps(DSVT_K_PART_SCAN, st);
      k_scan_windows<<<1, 1024, 0, st>>>(count, soff, p.g.n_windows, cfg->tau, max_sets, n_sets, status,
                                         (int32_t*)(base + p.off_setwin), p.set_bound);
    }
    if (tiles != nullptr) {
      dsvt_prof_scope ps(DSVT_K_PART_TILES, st);
      k_tiles<<<1, 1024, 0, st>>>((const int32_t*)(base + p.off_setwin), count, soff, n_sets, set_cap, cfg->tau,
                                  p.g.n_windows, p.rows_per_cut, tout, (int32_t*)(base + p.off_tilerows),
                                  (int32_t*)(base + p.off_tilepos), (int32_t*)(base + p.off_setp), set_loc);
    }
  }
  {
    dsvt_prof_scope ps(DSVT_K_PART_EMIT, st);
    k_emit<<<(unsigned)dsvt_ceil_div(n_voxels, tb), tb, 0, st>>>(p.g, (const int4*)coords, keys, n_voxels, bitmap, prefix,
                                                                 count, soff, set_cap, set_inds, voxel_slot, set_win, set_loc,
                                                                 tout.tile_desc, tout.max_tiles);
  }
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}
