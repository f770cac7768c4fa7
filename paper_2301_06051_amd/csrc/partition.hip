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

constexpr size_t kFrontLds = 152 * 1024;         // LDS k_front may ask for
constexpr uint64_t kWsMagic = 0x44535654504152ull;   // scratch header: "the mark bitmap of n_words words is all zero"
constexpr size_t kWsHeader = 256;
constexpr int32_t kRankWords = 8;                 // windows of up to this many bitmap words need no prefix array

struct PartGeom {
  int32_t grid[3], win[3], shift[3], nw[3];
  int32_t batch, tau;
  uint32_t magic[3];       // ceil(2^32 / win[a]) when that divides every x + shift exactly (see div_win), else 0
  uint32_t magic_tau;      // the same for tau (dividends up to a window's volume + tau), 0 when not exact; used by k_front
  int32_t words_per_win;   // 32-bit bitmap words per window (window volume rounded up to 32)
  int32_t n_windows;       // batch * nw[0] * nw[1] * nw[2]
  uint32_t vol;            // cells of a window
  uint32_t shuf_mul[2], shuf_add[2];   // the cell shuffle of inner orders 2 and 3 (see voxel_key)
};

// What differs between the two rotated partitions of one window configuration (Sec. 3.2): the order
// of the voxels inside a window, hence the occupancy bitmap, its prefix and the slot maps.  Windows,
// set counts and tile boundaries are common.  a[k] belongs to inner order axis0 + k.
struct AxisBufs {
  uint32_t* mark;                            // [n_words] bits set by k_mark; zero before and after every call
  uint32_t *bitmap, *prefix;                 // [n_words] each: the call's own copy of the bits, and their running count
  int32_t *set_inds, *voxel_slot, *tile_desc;
};
struct AxisSet {
  AxisBufs a[2];
  int32_t n, axis0;
  const uint64_t* ws_token;                  // scratch header, equal to `token` when the mark bitmaps are known to be zero
  uint64_t token;
};

__device__ __forceinline__ bool ws_ready(const AxisSet& ax) { return *ax.ws_token == ax.token; }

__global__ void k_ws_init(uint32_t* __restrict__ words, int64_t n, uint64_t* __restrict__ ws_token, uint64_t token) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) words[i] = 0u;
  if (i == 0) *ws_token = token;     // (kernels of later calls start after this one has ended)
}

__global__ void k_ws_revoke(uint64_t* __restrict__ ws_token) {
  if (threadIdx.x == 0) *ws_token = 0ull;
}

// x / win[a] for 0 <= x < grid + shift.  With m = ceil(2^32 / d) the high word of x * m is floor(x / d)
// whenever x * (m * d - 2^32) < 2^32, which x < 2^16 and d < 2^15 guarantee (the host sets magic only then).
__device__ __forceinline__ int32_t div_win(const PartGeom& g, int32_t a, int32_t x) {
  if (g.win[a] == 1) return x;
  if (g.magic[a] != 0u) return (int32_t)__umulhi((uint32_t)x, g.magic[a]);
  return x / g.win[a];
}

// x / d by the high word of x * magic (magic = ceil(2^32 / d), exact for the dividends the host checked).
__device__ __forceinline__ uint32_t div_magic(uint32_t x, uint32_t magic) { return __umulhi(x, magic); }

// Window key and in-window cell of a voxel (b, x, y, z); false when it lies outside the grid.
__device__ __forceinline__ bool voxel_cell(const PartGeom& g, int4 c, uint32_t& wkey, int32_t& xi, int32_t& yi, int32_t& zi) {
  const bool ok = (uint32_t)c.x < (uint32_t)g.batch && (uint32_t)c.y < (uint32_t)g.grid[0] &&
                  (uint32_t)c.z < (uint32_t)g.grid[1] && (uint32_t)c.w < (uint32_t)g.grid[2];
  if (!ok) return false;
  const int32_t x = c.y + g.shift[0], y = c.z + g.shift[1], z = c.w + g.shift[2];
  const int32_t wx = div_win(g, 0, x), wy = div_win(g, 1, y), wz = div_win(g, 2, z);
  xi = x - wx * g.win[0]; yi = y - wy * g.win[1]; zi = z - wz * g.win[2];
  wkey = (uint32_t)(((c.x * g.nw[0] + wx) * g.nw[1] + wy) * g.nw[2] + wz);
  return true;
}

// Composite key = window key * (32*words_per_win) + inner key; the inner key runs x-major for the
// X-axis partition (even inner orders) and y-major for the Y-axis one (odd).  Inner orders 2 and 3 are the
// "Random" baseline of the paper's set-partition ablation (Sec. 4.4), which the paper builds by renumbering the
// voxels inside a window: the window's cells in a fixed shuffle, key -> (key * mul + add) mod volume with mul
// coprime to the volume.  (4 and 5, "Sparse", re-deal the ranks instead: see k_emit.)
__device__ __forceinline__ uint32_t voxel_key(const PartGeom& g, int32_t axis, uint32_t wkey, int32_t xi, int32_t yi, int32_t zi) {
  uint32_t inner = (axis & 1) == 0 ? (uint32_t)((xi * g.win[1] + yi) * g.win[2] + zi)
                                   : (uint32_t)((yi * g.win[0] + xi) * g.win[2] + zi);
  if ((axis >> 1) == 1) inner = (inner * g.shuf_mul[axis & 1] + g.shuf_add[axis & 1]) % g.vol;   // (volume <= 2^16)
  return wkey * (uint32_t)(g.words_per_win * 32) + inner;
}

// `group` lanes (a power of two <= 64) per window: pop-count the window's words, leave in
// word_prefix[] the number of set bits in the window's earlier words, and the window total.
// y_words != nullptr: the group also sets, in its LDS words y_words[0 .. words_per_win) (zero on entry), the bits of
// the window's voxels in the other inner order (x and y exchanged), for a second call with lds_src = those words.
__device__ __forceinline__ void window_count(int32_t tid, uint32_t* __restrict__ mark, uint32_t* __restrict__ bitmap,
                                             uint32_t* __restrict__ word_prefix, int32_t* __restrict__ win_count,
                                             int32_t n_windows, int32_t words_per_win, int32_t group,
                                             const uint32_t* lds_src = nullptr, uint32_t* y_words = nullptr,
                                             int32_t win_l = 1, int32_t win_w = 1, int32_t win_h = 1) {
  int32_t w = tid / group, lane = tid & (group - 1);
  if (w >= n_windows) return;               // whole groups leave together
  const int64_t base = (int64_t)w * words_per_win;
  const float rcp_h = __frcp_rn((float)win_h), rcp_w = __frcp_rn((float)win_w);
  uint32_t running = 0;
  for (int32_t w0 = 0; w0 < words_per_win; w0 += group) {
    int32_t j = w0 + lane;
    uint32_t v = 0u;
    if (j < words_per_win) {                 // the word moves from the mark bitmap (left zero) to this call's copy
      uint32_t bits;
      if (lds_src != nullptr) bits = lds_src[j];
      else { bits = mark[base + j]; mark[base + j] = 0u; }
      bitmap[base + j] = bits;
      v = (uint32_t)__popc(bits);
      if (y_words != nullptr) {
        // inner key (x W + y) H + z -> (y L + x) H + z; keys are below 2^16, where (k + 0.5) / d in float truncates to floor(k / d)
        for (uint32_t rest = bits; rest; rest &= rest - 1u) {
          const int32_t key = j * 32 + (__ffs((int)rest) - 1);
          const int32_t t = (int32_t)(((float)key + 0.5f) * rcp_h), z = key - t * win_h;
          const int32_t x = (int32_t)(((float)t + 0.5f) * rcp_w), y = t - x * win_w;
          const int32_t yk = (y * win_l + x) * win_h + z;
          atomicOr(&y_words[yk >> 5], 1u << (yk & 31));
        }
      }
    }
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

// Tile descriptor, one per workgroup tile of the layer kernels, in launch order (256 ints):
//   [0] rows R (sets padded to multiples of 4)   [1] sets ns
//   [2 + s] first row of set s                    [2 + 24 + s] distinct voxels of set s   (s < ns <= 24)
//   [64 + 2 r] voxel of row r, -1 for padding rows  [65 + 2 r] (multiplicity << 24) | position code of row r
// (the two words of a row side by side: k_emit writes them with one 8-byte store)
constexpr int kDescInts = 256, kDescSets = 24, kDescR0 = 2, kDescNu = 2 + kDescSets, kDescRow = 64;
constexpr int kTileRows = 96;
constexpr int32_t kComputeUnits = 256;            // MI355X

// Workgroup barrier that waits for this wavefront's LDS traffic only.  __syncthreads() also waits for its
// outstanding stores to memory (a microsecond each time); the kernels that use it never read back what they wrote there.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Filled tiles: a set starts a tile when it no longer fits the `cap` (at most 96) rows of the tile before.  These boundaries
// depend on each other, so: jump[s] = the set that starts the next tile if s starts one (a binary search over P, the rows
// before every set, for all sets side by side), and the row sequence is taken in pieces of kFillPieceRows rows: the first
// set that begins in a piece starts a tile whatever came before (one short tile per piece: 0.5 % more tiles at 96 rows),
// and a thread per piece follows the jumps from there, all pieces at once.  (Following the jumps from set 0 through the
// whole frame by pointer doubling, the exact fill, took 31 k cycles for 6,500 sets.)
// All in LDS, 1,024 threads; P[0 .. n_sets] is ready on entry, mark[s] = 1 for the tile starts on return; jump2: scratch
// for the list of pieces.
constexpr int32_t kFillPieceShift = 12, kFillPieceRows = 1 << kFillPieceShift;
__device__ __forceinline__ void fill_tile_starts(const int32_t* P, uint16_t* jump, uint16_t* jump2, uint8_t* mark,
                                                 int32_t n_sets, int32_t cap) {
  __shared__ int32_t n_pieces;
  const int32_t tid = threadIdx.x;
  // (a piece holds at least kFillPieceRows / 96 sets, so the list fits the 2 (n_sets + 1) bytes of jump2)
  int32_t* piece_first = reinterpret_cast<int32_t*>((reinterpret_cast<uintptr_t>(jump2) + 3) & ~(uintptr_t)3);
  if (tid == 0) n_pieces = 0;
  lds_barrier();
  constexpr int32_t kB = 8;                                  // sets a thread works on side by side: their LDS reads overlap
  for (int32_t base = 0; base <= n_sets; base += 1024 * kB) {
    // smallest t in (s, n_sets] with P[t + 1] - P[s] > cap (n_sets = none).  A set has at least 4 rows, so t is at most
    // s + cap / 4 + 1: five or six halvings, taken in step for the kB sets.  (A set longer than cap gets a tile of its own.)
    int32_t lo[kB], hi[kB], lim[kB];
#pragma unroll
    for (int32_t k = 0; k < kB; ++k) {
      const int32_t s = base + tid + k * 1024;
      lo[k] = s + 1;
      hi[k] = min(n_sets, s + cap / 4 + 2);
      lim[k] = s < n_sets ? P[s] + cap : 0;
      if (s >= n_sets) { lo[k] = n_sets; hi[k] = n_sets; }
      if (s < n_sets && (s == 0 || (P[s] >> kFillPieceShift) != (P[s - 1] >> kFillPieceShift)))
        piece_first[atomicAdd(&n_pieces, 1)] = s;
    }
    for (int32_t step = 0; step < 7; ++step) {               // 2^7 > 96 / 4 + 2
      int32_t mid[kB], pv[kB];                               // (no branches: the kB reads of a step go out together)
#pragma unroll
      for (int32_t k = 0; k < kB; ++k) { mid[k] = (lo[k] + hi[k]) >> 1; pv[k] = P[min(mid[k] + 1, n_sets)]; }
#pragma unroll
      for (int32_t k = 0; k < kB; ++k) {
        const bool open = lo[k] < hi[k], over = pv[k] > lim[k];
        hi[k] = (open && over) ? mid[k] : hi[k];
        lo[k] = (open && !over) ? mid[k] + 1 : lo[k];
      }
    }
    // the walk below stays inside a piece: a jump that leaves the piece of its set ends it (n_sets)
    int32_t here[kB], there[kB];
#pragma unroll
    for (int32_t k = 0; k < kB; ++k) {
      const int32_t s = base + tid + k * 1024;
      here[k] = P[min(s, n_sets)];
      there[k] = P[lo[k]];                                   // (lo <= n_sets)
    }
#pragma unroll
    for (int32_t k = 0; k < kB; ++k) {
      const int32_t s = base + tid + k * 1024;
      if (s <= n_sets) {                                     // (mark[n_sets] is a dummy)
        jump[s] = (uint16_t)((here[k] >> kFillPieceShift) == (there[k] >> kFillPieceShift) ? lo[k] : n_sets);
        mark[s] = 0;
      }
    }
  }
  lds_barrier();
  const int32_t np = n_pieces;
  for (int32_t i = tid; i < np; i += 1024) {
    int32_t s = piece_first[i];
    // at most kFillPieceRows / 4 + 1 sets begin in a piece; the bound also ends the walk on tables that are not sorted
    for (int32_t step = 0; step <= kFillPieceRows / 4 && s < n_sets; ++step) {
      mark[s] = 1;
      s = jump[s];
    }
  }
  lds_barrier();
}

// Whether a frame's tiles are filled rather than cut every rpc_max rows, and if so their starts (mark[], as
// fill_tile_starts leaves them).  A tile filled up to `cap` rows holds about cap - (mean set rows) / 2.  Filling pays
// when it saves a whole round over the compute units, or when the frame takes more than two rounds anyway.  A frame
// of a few rounds gets the capacity that puts its tile count just under a whole number of rounds (a last round of a
// few full-size tiles costs as much as a full round); should the count still come out above it, the next number of
// rounds is tried.  Frames of more than four rounds get the whole 96 rows (measured at seven rounds: fewer, fuller
// tiles beat a full last round, 167 against 185 us per layer).  Same arguments as fill_tile_starts; every thread returns
// the same answer.
constexpr int32_t kTunedRounds = 4;
__device__ __forceinline__ bool fill_wanted(int32_t total_rows, int32_t n_sets, int32_t rpc_max) {   // fill_tiles' first test
  if (n_sets <= 0 || rpc_max < 4) return false;
  const int32_t rounds_cut = (total_rows + kComputeUnits * rpc_max - 1) / (kComputeUnits * rpc_max);
  const int32_t rounds = (int32_t)ceilf((float)total_rows / (256.f * ((float)kTileRows - 0.5f * (float)total_rows / (float)n_sets)));
  return rounds_cut > 1 && (rounds < rounds_cut || rounds_cut > 2);
}
__device__ __forceinline__ bool fill_tiles(const int32_t* P, uint16_t* jump, uint16_t* jump2, uint8_t* mark, int32_t n_sets,
                                           int32_t rpc_max) {
  __shared__ int32_t n_starts;
  if (n_sets <= 0 || rpc_max < 4) return false;
  const int32_t total_rows = P[n_sets];
  const float half_set = 0.5f * (float)total_rows / (float)n_sets;
  const float best_fill = (float)kTileRows - half_set;
  const int32_t rounds_cut = (total_rows + kComputeUnits * rpc_max - 1) / (kComputeUnits * rpc_max);
  int32_t rounds = (int32_t)ceilf((float)total_rows / (256.f * best_fill));
  if (rounds_cut <= 1) return false;                         // (tile_cut spreads frames of less than a round)
  for (int32_t attempt = 0; attempt < 2; ++attempt, ++rounds) {
    if (!(rounds < rounds_cut || rounds_cut > 2)) return false;
    int32_t cap = kTileRows;
    if (rounds <= kTunedRounds) {
      const float fill = (float)total_rows / (0.97f * 256.f * (float)rounds);
      const int32_t c = ((int32_t)ceilf(fill + half_set) + 3) & ~3;
      cap = c > kTileRows ? kTileRows : c;
    }
    if (threadIdx.x == 0) n_starts = 0;
    fill_tile_starts(P, jump, jump2, mark, n_sets, cap);      // (barriers inside: n_starts is zero for everybody after)
    if (rounds > kTunedRounds) return true;
    int32_t mine = 0;
    for (int32_t s = threadIdx.x; s < n_sets; s += 1024) mine += mark[s];
    if (mine) atomicAdd(&n_starts, mine);
    lds_barrier();
    const int32_t tiles = n_starts;
    lds_barrier();
    if (tiles <= rounds * kComputeUnits) return true;
  }
  return false;
}

// Distinct voxels of the j-th set of a window with N voxels in S sets (closed form from Eq. 3).
__device__ __forceinline__ int32_t set_distinct(int64_t N, int64_t S, int64_t j, int64_t tau) {
  if (N < 32768 && S * tau < 65536) {                       // the usual case: everything fits 32-bit division
    const uint32_t n = (uint32_t)N, T = (uint32_t)(S * tau), a = (uint32_t)(j * tau);
    return (int32_t)(((a + (uint32_t)tau - 1u) * n) / T - (a * n) / T + 1u);
  }
  const int64_t lo = (j * tau * N) / (S * tau), hi = ((j * tau + tau - 1) * N) / (S * tau);
  return (int32_t)(hi - lo + 1);
}

// The same counts for j = 0, 1, 2, ... in turn, with one division per window: floor(j*tau*N / (S*tau)) =
// floor(j*N/S) =: q_j with remainder r_j, both stepped by N/S and N mod S; and the last voxel of set j,
// floor(((j+1)*N - N/tau) / S), is q_{j+1} less one exactly when r_{j+1} * tau < N.
struct SetWalk {
  uint32_t N, S, tau, dq, dr, q, r;
  bool small;                                                // N < 2^16: float division and 24-bit products are exact
  // N < 2^16: the quotient of (N + 0.5) / S in float arithmetic (errors of a few 2^-24 of a quotient below
  // 2^16 / S, against a distance of at least 0.5 / S to the next integer) truncates to floor(N / S)
  __device__ __forceinline__ SetWalk(int32_t n, int32_t s, int32_t t) : N((uint32_t)n), S((uint32_t)s), tau((uint32_t)t), q(0u), r(0u) {
    small = N < 65536u;
    dq = s > 0 ? (small ? (uint32_t)(((float)N + 0.5f) * __frcp_rn((float)S)) : N / S) : 0u;
    dr = small ? N - __umul24(dq, S) : N - dq * S;
  }
  __device__ __forceinline__ void restart() { q = 0u; r = 0u; }
  __device__ __forceinline__ int32_t next() {               // distinct voxels of the next set
    uint32_t q2 = q + dq, r2 = r + dr;
    if (r2 >= S) { r2 -= S; ++q2; }
    const uint32_t nu = q2 - (small ? ((uint32_t)__umul24(r2, tau) < N ? 1u : 0u) : (r2 * tau < N ? 1u : 0u)) - q + 1u;
    q = q2; r = r2;
    return (int32_t)nu;
  }
};

struct TileOut {                       // all null when the caller wants no work list
  int32_t *tile_first, *n_tiles, *tile_order;
  int32_t* tile_desc[2];               // one descriptor array per axis (second null for a single partition)
  int32_t max_tiles;
};

// Everything the kernels need for one window configuration.  Several configurations over the same voxels
// (a stage's unshifted and shifted windows) go through the same launches, one grid slice each.
struct Job {
  PartGeom g;
  AxisSet ax;
  TileOut out;
  int32_t *win_count, *win_soff, *n_sets, *status, *set_win, *set_loc;
  int32_t n_words, max_sets, set_cap, rows_per_cut, tile_cap;
  int32_t fill_sets;                         // k_front: sets its LDS has tables for (filled tiles), 0 = none
  int32_t derive_y;                          // general front end: k_mark sets the X-order bits only, k_window_count transposes them
};
constexpr int32_t kMaxJobs = 4;
struct Jobs { Job j[kMaxJobs]; };

// One thread per voxel and job (blockIdx.y): set its bit in the mark bitmap of every axis.
__global__ void k_mark(Jobs jobs, const int4* __restrict__ coords, int32_t n) {
  const Job& J = jobs.j[blockIdx.y];
  int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  if (!ws_ready(J.ax)) {                     // scratch not prepared: mark nothing, the later kernels report no sets
    if (i == 0) atomicOr(J.status, DSVT_ST_WS_STATE);
    return;
  }
  uint32_t wkey; int32_t xi, yi, zi;
  if (!voxel_cell(J.g, coords[i], wkey, xi, yi, zi)) {
    atomicOr(J.status, DSVT_ST_COORD_RANGE);
    return;
  }
  const int32_t n_mark = J.derive_y ? 1 : J.ax.n;
  for (int32_t k = 0; k < n_mark; ++k) {
    const uint32_t key = voxel_key(J.g, J.ax.axis0 + k, wkey, xi, yi, zi), bit = 1u << (key & 31u);
    const uint32_t old = atomicOr(&J.ax.a[k].mark[key >> 5], bit);
    if (old & bit) atomicOr(J.status, DSVT_ST_COORD_REPEAT);
  }
}

// Padded rows of a set with nu distinct voxels.
__device__ __forceinline__ int32_t set_rows(int32_t nu) {
  const int32_t rows = (nu + 3) & ~3;
  return rows > kTileRows ? kTileRows : (rows < 4 ? 4 : rows);
}

// Rows between two tile cuts: at most rpc_max = 100 - pad4(tau), so that a tile never exceeds 96 rows.  A frame
// whose tiles would not fill the GPU's compute units once gets a smaller cut, i.e. more and shorter tiles on
// more units (measured: a 3,000-voxel frame 28 -> 22 us per layer, 8,000 voxels 29 -> 26 us).  Larger frames keep
// rpc_max: a tile's cost is mostly fixed (weights, barriers), so more tiles per unit buy nothing there.
__device__ __forceinline__ int32_t tile_cut(int32_t total_rows, int32_t rpc_max) {
  if (rpc_max < 16 || total_rows <= 0 || total_rows > rpc_max * kComputeUnits) return rpc_max;
  int32_t rpc = ((total_rows + kComputeUnits - 1) / kComputeUnits + 3) & ~3;     // at most 256 tiles
  rpc = rpc < 16 ? 16 : rpc;
  return rpc < rpc_max ? rpc : rpc_max;
}

// Header of launch slot pos, in every axis's descriptor array.
__device__ __forceinline__ void desc_header(const TileOut& out, int32_t pos, int32_t rows, int32_t sets) {
#pragma unroll
  for (int32_t k = 0; k < 2; ++k)
    if (out.tile_desc[k] != nullptr) {
      int32_t* d = out.tile_desc[k] + (int64_t)pos * kDescInts;
      d[0] = rows;
      d[1] = sets;
    }
}

// Set ls of the descriptor d: first row, distinct voxels, and -1 in the rows that pad it to a multiple of 4.
__device__ __forceinline__ void desc_set(int32_t* d, int32_t ls, int32_t r0, int32_t nu) {
  const int32_t r1 = r0 + set_rows(nu) < kTileRows ? r0 + set_rows(nu) : kTileRows;
  d[kDescR0 + ls] = r0;
  d[kDescNu + ls] = nu;
  for (int32_t r = r0 + nu; r < r1; ++r) *reinterpret_cast<int2*>(d + kDescRow + 2 * r) = make_int2(-1, -1);
}

// What k_emit needs to know about a set with a tile: descriptor slot, place among the tile's sets, first row.
__device__ __forceinline__ int32_t set_loc_code(int32_t pos, int32_t ls, int32_t r0) { return (pos << 12) | (ls << 7) | r0; }

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int32_t dpp_or(int32_t identity, int32_t v) {       // v of the lane CTRL names, identity where there is none
  return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xF, false);
}
// Inclusive scans over a wavefront by data-parallel-primitive moves: shifts by 1, 2, 4, 8 inside rows of
// 16 lanes, then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ int32_t wave_scan_add(int32_t v) {
  v += dpp_or<0x111, 0xF>(0, v);
  v += dpp_or<0x112, 0xF>(0, v);
  v += dpp_or<0x114, 0xF>(0, v);
  v += dpp_or<0x118, 0xF>(0, v);
  v += dpp_or<0x142, 0xA>(0, v);
  v += dpp_or<0x143, 0xC>(0, v);
  return v;
}
__device__ __forceinline__ int32_t wave_scan_max(int32_t v, int32_t lowest) {
  int32_t t;
  t = dpp_or<0x111, 0xF>(lowest, v); v = t > v ? t : v;
  t = dpp_or<0x112, 0xF>(lowest, v); v = t > v ? t : v;
  t = dpp_or<0x114, 0xF>(lowest, v); v = t > v ? t : v;
  t = dpp_or<0x118, 0xF>(lowest, v); v = t > v ? t : v;
  t = dpp_or<0x142, 0xA>(lowest, v); v = t > v ? t : v;
  t = dpp_or<0x143, 0xC>(lowest, v); v = t > v ? t : v;
  return v;
}


// A frame with more sets than the tables hold is taken in pieces of kTilePiece sets, a workgroup per piece, every piece
// starting a tile of its own; what a piece has to know of the others are their tile counts per launch-order bucket.
constexpr int32_t kTilePiece = 4096;
struct TilePiece {
  int32_t mode;                   // 0: the whole frame; 1: a piece, counting its tiles per bucket; 2: a piece, writing
  int32_t s_base;                 // first set of the piece
  int32_t tile_base;              // mode 2: tiles of the pieces before this one
  int32_t* hist_out;              // mode 1: [32] this piece's tiles per bucket
  const int32_t* bucket_base;     // mode 2: [32] in LDS, launch slots before this piece's tiles of a bucket
};

// The work list of a frame, or of a piece of one, whose sets fit the LDS tables (n_sets <= fill_sets, below 65,535): one
// workgroup cuts the set sequence into tiles for the layer kernels, orders the tiles for launch and writes the
// descriptor headers; set_loc[s] = set_loc_code(descriptor slot, place in the tile, first row), for k_emit.  The rows
// before every set, the tile starts and the tiles' first sets stay in LDS from the first pass to the last, so that the
// passes are separated by workgroup barriers only -- no pass reads memory that an earlier pass wrote.
// P [fill_sets + 1] | first set of every tile, 16 bit [fill_sets + 1] | 16 bit [fill_sets + 1] | tile-start marks
// [fill_sets + 1]; the two 16-bit tables are the fill's scratch first.  Sets are counted from the piece's first.
// set_w == nullptr: P [0 .. n_sets] is in place already (k_scan_windows wrote it while it scanned the windows).
__device__ __forceinline__ void build_tiles_lds(const int32_t* set_w, const int32_t* win_count, const int32_t* win_soff,
                                                int32_t n_sets, int32_t tau, int32_t n_windows, int32_t rows_per_cut,
                                                TileOut out, int32_t* set_loc, int32_t fill_sets, int32_t* status,
                                                const TilePiece pc) {
  extern __shared__ uint32_t fill_lds[];
  __shared__ int32_t wave_tot[16];
  __shared__ int32_t carry_s, over_s;
  __shared__ int32_t hist[32], running[32], wave_cnt[16][32];
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int32_t* P = reinterpret_cast<int32_t*>(fill_lds);
  uint16_t* t_first = reinterpret_cast<uint16_t*>(P + fill_sets + 1);
  uint16_t* scratch16 = t_first + fill_sets + 1;
  uint8_t* mark = reinterpret_cast<uint8_t*>(scratch16 + fill_sets + 1);
  if (tid == 0) { carry_s = 0; over_s = -1; }
  lds_barrier();
  // pass 1: padded rows per set, their running sum (four consecutive sets per thread and trip: the two dependent
  // loads of a set -- its window, then the window's count and first set -- are in flight for four sets at once)
  constexpr int32_t kPer = 4;
  for (int32_t base = 0; set_w != nullptr && base < n_sets; base += 1024 * kPer) {
    const int32_t s0 = base + tid * kPer;
    int32_t w[kPer], cnt[kPer], soff[kPer], rows[kPer], pre[kPer];
#pragma unroll
    for (int32_t j = 0; j < kPer; ++j) {
      const int32_t wj = s0 + j < n_sets ? set_w[pc.s_base + s0 + j] : 0;
      w[j] = wj < 0 ? 0 : (wj >= n_windows ? n_windows - 1 : wj);
    }
#pragma unroll
    for (int32_t j = 0; j < kPer; ++j) { cnt[j] = win_count[w[j]]; soff[j] = win_soff[w[j]]; }
    int32_t mine = 0;
#pragma unroll
    for (int32_t j = 0; j < kPer; ++j) {
      const int64_t N = cnt[j] > 0 ? cnt[j] : 1, S = (N + tau - 1) / tau;
      rows[j] = s0 + j < n_sets ? set_rows(set_distinct(N, S, pc.s_base + s0 + j - soff[j], tau)) : 0;
      pre[j] = mine;
      mine += rows[j];
    }
    const int32_t incl = wave_scan_add(mine);
    if (lane == 63) wave_tot[wv] = incl;
    lds_barrier();
    int32_t before = carry_s;
    for (int32_t k = 0; k < wv; ++k) before += wave_tot[k];
#pragma unroll
    for (int32_t j = 0; j < kPer; ++j)
      if (s0 + j < n_sets) P[s0 + j] = before + incl - mine + pre[j];
    if (s0 <= n_sets - 1 && n_sets - 1 < s0 + kPer) P[n_sets] = before + incl;
    lds_barrier();
    if (tid == 1023) carry_s = before + incl;
    lds_barrier();
  }
  // tile starts.  The whole frame: filled tiles (see fill_tile_starts) if it takes many rounds over the compute units,
  // else a set starts a tile when the running row count crosses a multiple of rows_per_cut between its predecessor's
  // start and its own (a tile then holds at most rows_per_cut - 4 + pad4(tau) <= 96 rows).  A piece (a frame of very
  // many rounds): tiles filled to the full 96 rows.
  if (pc.mode != 0) {
    fill_tile_starts(P, t_first, scratch16, mark, n_sets, kTileRows);
  } else {
    rows_per_cut = tile_cut(P[n_sets], rows_per_cut);
    if (!fill_tiles(P, t_first, scratch16, mark, n_sets, rows_per_cut)) {
      lds_barrier();
      for (int32_t s = tid; s <= n_sets; s += 1024) mark[s] = s < n_sets && (s == 0 || P[s - 1] / rows_per_cut != P[s] / rows_per_cut);
    }
  }
  if (tid == 0) carry_s = 0;
  lds_barrier();
  // pass 2: the tiles are numbered by counting their starts (a scan), so none is empty.  (A piece never has more
  // tiles than sets, so only the whole-frame list can turn out too short here.)
  const int32_t tile_lim = (pc.mode == 0 && out.max_tiles < fill_sets) ? out.max_tiles : fill_sets;
  for (int32_t base = 0; base < n_sets; base += 1024 * kPer) {
    const int32_t s0 = base + tid * kPer;
    int32_t pre[kPer], mine = 0;
#pragma unroll
    for (int32_t j = 0; j < kPer; ++j) {
      mine += (s0 + j < n_sets && mark[s0 + j]) ? 1 : 0;
      pre[j] = mine;
    }
    const int32_t incl = wave_scan_add(mine);
    if (lane == 63) wave_tot[wv] = incl;
    lds_barrier();
    int32_t before = carry_s;
    for (int32_t k = 0; k < wv; ++k) before += wave_tot[k];
#pragma unroll
    for (int32_t j = 0; j < kPer; ++j) {
      const int32_t s = s0 + j;
      if (s < n_sets && mark[s]) {
        const int32_t tile = before + incl - mine + pre[j] - 1;
        if (tile < tile_lim) {
          t_first[tile] = (uint16_t)s;
          if (pc.mode != 1) out.tile_first[pc.tile_base + tile] = pc.s_base + s;
        } else if (tile == tile_lim) {
          over_s = s;                                        // first set that no tile is left for
        }
      }
    }
    lds_barrier();
    if (tid == 1023) carry_s = before + incl;
    lds_barrier();
  }
  const bool tiles_short = carry_s > tile_lim;               // the caller's list is shorter than the frame needs
  const int32_t nt = tiles_short ? tile_lim : carry_s;
  const int32_t n_eff = tiles_short ? over_s : n_sets;
  if (tid == 0) {
    if (tiles_short) atomicOr(status, DSVT_ST_TILE_OVERFLOW);   // the sets past the last tile get none
    if (pc.mode == 0) { *out.n_tiles = nt; out.tile_first[nt] = n_eff; }
    t_first[nt] = (uint16_t)n_eff;
  }
  if (tid < 32) hist[tid] = 0;
  lds_barrier();
  // pass 3: launch order = tiles with more rows first (a stable counting sort on rows / 4), so that the short tiles
  // fill the tail of the launch
  for (int32_t t = tid; t < nt; t += 1024) {
    int32_t b = 24 - (P[t_first[t + 1]] - P[t_first[t]]) / 4;
    b = b < 0 ? 0 : (b > 31 ? 31 : b);
    atomicAdd(&hist[b], 1);
  }
  lds_barrier();
  if (pc.mode == 1) {
    if (tid < 32) pc.hist_out[tid] = hist[tid];
    return;
  }
  if (wv == 0) {
    const int32_t h = lane < 32 ? hist[lane] : 0, incl = wave_scan_add(h);
    if (lane < 32) running[lane] = pc.mode == 2 ? pc.bucket_base[lane] : incl - h;
  }
  lds_barrier();
  for (int32_t base = 0; base < nt; base += 1024) {
    const int32_t t = base + tid;
    int32_t b = -1, rows = 0;
    if (t < nt) {
      rows = P[t_first[t + 1]] - P[t_first[t]];
      b = 24 - rows / 4;
      b = b < 0 ? 0 : (b > 31 ? 31 : b);
    }
    for (int32_t k = lane; k < 32; k += 64) wave_cnt[wv][k] = 0;
    // lanes of this wavefront with the same bucket: those that agree with this lane in each of its 5 bits
    unsigned long long same = __ballot(b >= 0);
#pragma unroll
    for (int32_t bit = 0; bit < 5; ++bit) {
      const bool one = (b >> bit) & 1;
      const unsigned long long ones = __ballot(one);
      same &= one ? ones : ~ones;
    }
    const unsigned long long below = same & ((1ull << lane) - 1ull);
    const int32_t rank = __popcll(below);                     // among this wavefront's lanes of the same bucket
    if (b >= 0 && below == 0ull) wave_cnt[wv][b] = __popcll(same);
    lds_barrier();
    if (tid < 512) {                                          // a row of 16 lanes per bucket, a lane per wavefront
      const int32_t bb = tid >> 4, k = tid & 15;
      const int32_t cnt = wave_cnt[k][bb];
      int32_t incl = cnt;
      incl += dpp_or<0x111, 0xF>(0, incl);
      incl += dpp_or<0x112, 0xF>(0, incl);
      incl += dpp_or<0x114, 0xF>(0, incl);
      incl += dpp_or<0x118, 0xF>(0, incl);
      const int32_t first = running[bb];
      wave_cnt[k][bb] = first + incl - cnt;
      if (k == 15) running[bb] = first + incl;                // (read by this row only, all of it before this write)
    }
    lds_barrier();
    if (b >= 0) {
      // the tile's launch slot; then, per set of the tile, its descriptor slot, its place among the tile's sets and
      // its first row
      const int32_t pos = wave_cnt[wv][b] + rank;
      const int32_t s_begin = t_first[t], s_end = t_first[t + 1], p0 = P[s_begin];
      out.tile_order[pos] = pc.tile_base + t;
      desc_header(out, pos, rows, s_end - s_begin);
      for (int32_t s = s_begin; s < s_end; ++s) {
        const int32_t ls = s - s_begin, r0 = P[s] - p0;
        set_loc[pc.s_base + s] = (ls < kDescSets && r0 <= kTileRows - 4) ? set_loc_code(pos, ls, r0) : -1;
      }
    }
    lds_barrier();
  }
  for (int32_t s = n_eff + tid; s < n_sets; s += 1024) set_loc[pc.s_base + s] = -1;
}

// k_scan_windows for a job whose sets fit the LDS tables of the work-list builder: the scans of voxels- and
// sets-per-window as in scan_windows(), and with them the rows before every set (a thread per window walks its
// sets), straight into the builder's table -- the builder then starts from there, in the same launch, instead of
// finding every set's window and size again in a launch of its own.
__device__ __forceinline__ void scan_windows_and_tiles(const int32_t* __restrict__ win_count, int32_t* __restrict__ win_soff,
                                                       int32_t n_windows, int32_t tau, int32_t max_sets, int32_t set_cap,
                                                       int32_t* __restrict__ n_sets_out, int32_t* __restrict__ status,
                                                       int32_t rows_per_cut, TileOut out, int32_t* set_loc, int32_t fill_sets) {
  extern __shared__ uint32_t fill_lds[];
  __shared__ int32_t wave_tot[2][16];
  __shared__ int32_t carry_sr[2];
  int32_t* P = reinterpret_cast<int32_t*>(fill_lds);            // [fill_sets + 1], as build_tiles_lds lays it out
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (tid == 0) { carry_sr[0] = 0; carry_sr[1] = 0; }
  lds_barrier();
  int32_t nvox_next = tid < n_windows ? win_count[tid] : 0;  // (a trip's counts are requested during the trip before)
  for (int32_t base = 0; base < n_windows; base += 1024) {
    const int32_t w = base + tid;
    const int32_t nvox = nvox_next;
    nvox_next = w + 1024 < n_windows ? win_count[w + 1024] : 0;
    const int32_t S = (nvox + tau - 1) / tau;
    SetWalk walk(nvox, S, tau);
    int32_t R = 0;
    for (int32_t j = 0; j < S; ++j) R += set_rows(walk.next());
    const int32_t s_incl = wave_scan_add(S), r_incl = wave_scan_add(R);
    if (lane == 63) { wave_tot[0][wv] = s_incl; wave_tot[1][wv] = r_incl; }
    lds_barrier();
    int32_t s_before = carry_sr[0], r_before = carry_sr[1];
    for (int32_t k = 0; k < wv; ++k) { s_before += wave_tot[0][k]; r_before += wave_tot[1][k]; }
    if (w < n_windows) {
      const int32_t soff = s_before + s_incl - S;
      win_soff[w] = soff;
      int32_t p = r_before + r_incl - R;
      walk.restart();
      for (int32_t j = 0; j < S; ++j) {
        if (soff + j <= fill_sets) P[soff + j] = p;
        p += set_rows(walk.next());
      }
    }
    lds_barrier();
    if (tid == 1023) { carry_sr[0] = s_before + s_incl; carry_sr[1] = r_before + r_incl; }
    lds_barrier();
  }
  const int32_t n_all = carry_sr[0];
  if (tid == 0) {
    *n_sets_out = n_all;
    if (n_all > max_sets) atomicOr(status, DSVT_ST_SET_OVERFLOW);
  }
  int32_t n_sets = n_all < set_cap ? n_all : set_cap;
  n_sets = n_sets < fill_sets ? n_sets : fill_sets;
  if (n_sets <= 0) {
    if (tid == 0) { *out.n_tiles = 0; out.tile_first[0] = 0; }
    return;
  }
  if (tid == 0 && n_sets == n_all) P[n_sets] = carry_sr[1];     // (of a clipped list, P[n_sets] is the row count before the first set left out)
  lds_barrier();
  build_tiles_lds(nullptr, nullptr, nullptr, n_sets, tau, n_windows, rows_per_cut, out, set_loc, fill_sets, status,
                  TilePiece{0, 0, 0, nullptr, nullptr});
}

// k_tiles for one window configuration: the whole frame in the first workgroup if its sets fit the tables, else a
// workgroup per piece of kTilePiece sets, in two launches -- phase 0 counts every piece's tiles per launch-order bucket,
// phase 1 places them (a piece's tiles come after those of the pieces before it, bucket by bucket, so the order is the
// one a single stable sort of all tiles would give).
__device__ __forceinline__ void build_tiles(const int32_t* set_w, const int32_t* win_count, const int32_t* win_soff,
                                            const int32_t* n_sets_ptr, int32_t set_cap, int32_t tau, int32_t n_windows,
                                            int32_t rows_per_cut, TileOut out, int32_t* piece_hist, int32_t* set_loc,
                                            int32_t fill_sets, int32_t* status, int32_t phase) {
  __shared__ int32_t bucket_base_s[32];
  __shared__ int32_t tile_base_s, total_s;
  const int32_t tid = threadIdx.x, lane = tid & 63, piece = blockIdx.y;
  int32_t n_sets = *n_sets_ptr;
  n_sets = n_sets < set_cap ? n_sets : set_cap;
  if (n_sets <= 0) {
    if (tid == 0 && piece == 0 && phase == 1) { *out.n_tiles = 0; out.tile_first[0] = 0; }
    return;
  }
  if (n_sets <= fill_sets && n_sets < 65535) {
    if (piece == 0 && phase == 1)
      build_tiles_lds(set_w, win_count, win_soff, n_sets, tau, n_windows, rows_per_cut, out, set_loc, fill_sets, status,
                      TilePiece{0, 0, 0, nullptr, nullptr});
    return;
  }
  const int32_t n_pieces = (n_sets + kTilePiece - 1) / kTilePiece;
  if (piece >= n_pieces) return;
  const int32_t s_base = piece * kTilePiece, n_mine = n_sets - s_base < kTilePiece ? n_sets - s_base : kTilePiece;
  if (phase == 0) {
    build_tiles_lds(set_w, win_count, win_soff, n_mine, tau, n_windows, rows_per_cut, out, set_loc, fill_sets, status,
                    TilePiece{1, s_base, 0, piece_hist + piece * 32, nullptr});
    return;
  }
  if (tid < 64) {
    int32_t all = 0, mine = 0;                               // tiles of bucket `lane`: of every piece, of the pieces before
    if (lane < 32)
      for (int32_t q = 0; q < n_pieces; ++q) {
        const int32_t h = piece_hist[q * 32 + lane];
        all += h;
        mine += q < piece ? h : 0;
      }
    const int32_t all_incl = wave_scan_add(all), mine_incl = wave_scan_add(mine);
    if (lane < 32) bucket_base_s[lane] = all_incl - all + mine;
    if (lane == 63) { total_s = all_incl; tile_base_s = mine_incl; }
  }
  lds_barrier();
  const int32_t total = total_s;
  if (total > out.max_tiles) {                               // the caller's list is shorter than the frame needs:
    for (int32_t s = tid; s < n_mine; s += 1024) set_loc[s_base + s] = -1;     // no set gets a tile
    if (tid == 0 && piece == 0) { atomicOr(status, DSVT_ST_TILE_OVERFLOW); *out.n_tiles = 0; out.tile_first[0] = 0; }
    return;
  }
  build_tiles_lds(set_w, win_count, win_soff, n_mine, tau, n_windows, rows_per_cut, out, set_loc, fill_sets, status,
                  TilePiece{2, s_base, tile_base_s, nullptr, bucket_base_s});
  if (tid == 0 && piece == n_pieces - 1) { *out.n_tiles = total; out.tile_first[total] = n_sets; }
}

// The general front end's own arguments for one window configuration (frames too large for k_front).
struct GenJob {
  int32_t *ws_setwin, *piece_hist;
  int32_t set_bound, want_tiles, fill_sets;
  int32_t merged;                            // k_scan_windows also builds the work list (sets fit the LDS tables)
};
struct GenJobs { GenJob j[kMaxJobs]; };

// A slice of a wavefront per window: zero the mark words, copy them, count them (blockIdx.y = axis, every axis
// leaves the same counts; blockIdx.z = job).
__global__ void k_window_count(Jobs jobs) {
  const Job& J = jobs.j[blockIdx.z];
  const AxisSet& ax = J.ax;
  if ((int32_t)blockIdx.y >= ax.n) return;
  const int32_t n_windows = J.g.n_windows, words_per_win = J.g.words_per_win;
  int32_t group = 1;
  while (group < 64 && group < words_per_win) group <<= 1;
  const int32_t tid = blockIdx.x * blockDim.x + threadIdx.x;
  if (!ws_ready(ax)) {
    const int32_t w = tid / group;
    if (w < n_windows && blockIdx.y == 0 && (tid & (group - 1)) == 0) J.win_count[w] = 0;
    return;
  }
  if (J.derive_y) {
    // only the X-order bits were marked: the group that moves a window's X words also transposes them, bit by bit,
    // into LDS words of its own, and then treats those as the window's Y-order words (a group is part of one
    // wavefront, whose LDS operations execute in order)
    if (blockIdx.y != 0) return;
    extern __shared__ uint32_t y_lds[];
    uint32_t* mine = y_lds + (threadIdx.x / group) * words_per_win;
    for (int32_t j = threadIdx.x & (group - 1); j < words_per_win; j += group) mine[j] = 0u;
    window_count(tid, ax.a[0].mark, ax.a[0].bitmap, ax.a[0].prefix, J.win_count, n_windows, words_per_win, group,
                 nullptr, mine, J.g.win[0], J.g.win[1], J.g.win[2]);
    window_count(tid, nullptr, ax.a[1].bitmap, ax.a[1].prefix, J.win_count, n_windows, words_per_win, group, mine);
    return;
  }
  window_count(tid, ax.a[blockIdx.y].mark, ax.a[blockIdx.y].bitmap, ax.a[blockIdx.y].prefix, J.win_count, n_windows,
               words_per_win, group);
}

// One workgroup per job.
__global__ void __launch_bounds__(1024) k_scan_windows(Jobs jobs, GenJobs gen) {
  const Job& J = jobs.j[blockIdx.x];
  const GenJob& G = gen.j[blockIdx.x];
  if (G.merged)
    scan_windows_and_tiles(J.win_count, J.win_soff, J.g.n_windows, J.g.tau, J.max_sets, J.set_cap, J.n_sets, J.status,
                           J.rows_per_cut, J.out, J.set_loc, G.fill_sets);
  else
    scan_windows(J.win_count, J.win_soff, J.g.n_windows, J.g.tau, J.max_sets, J.n_sets, J.status, G.ws_setwin, G.set_bound);
}

// Jobs that want a work list and did not get it from k_scan_windows: blockIdx.x = job, blockIdx.y = piece.
__global__ void __launch_bounds__(1024) k_tiles(Jobs jobs, GenJobs gen, int32_t phase) {
  const Job& J = jobs.j[blockIdx.x];
  const GenJob& G = gen.j[blockIdx.x];
  if (!G.want_tiles || G.merged) return;
  build_tiles(G.ws_setwin, J.win_count, J.win_soff, J.n_sets, J.set_cap, J.g.tau, J.g.n_windows, J.rows_per_cut, J.out,
              G.piece_hist, J.set_loc, G.fill_sets, J.status, phase);
}

// Scan over the 1024 threads of a workgroup, continued from one call to the next through `carry`:
// inclusive sums of a and b, and in xm the maximum of m over the threads before this one (and over
// earlier calls).  Every thread of the workgroup calls it; two barriers inside.
struct Scan3 { int32_t a, b, m, xm; };
__device__ __forceinline__ Scan3 block_scan3(Scan3 v, int32_t (*wave_tot)[16], int32_t* carry) {
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  v.a = wave_scan_add(v.a);
  v.b = wave_scan_add(v.b);
  v.m = wave_scan_max(v.m, -1);                         // (every m is at least -1)
  const int32_t below = __shfl_up(v.m, 1, 64);
  if (lane == 63) { wave_tot[0][wv] = v.a; wave_tot[1][wv] = v.b; wave_tot[2][wv] = v.m; }
  lds_barrier();
  // totals of the wavefronts before this one: a scan of the 16 totals in the first row of lanes
  const int32_t ta = wave_scan_add(lane < 16 ? wave_tot[0][lane] : 0), tb = wave_scan_add(lane < 16 ? wave_tot[1][lane] : 0),
                tm = wave_scan_max(lane < 16 ? wave_tot[2][lane] : -1, -1);
  int32_t pa = carry[0], pb = carry[1], pm = carry[2];
  if (wv > 0) {
    pa += __builtin_amdgcn_readlane(ta, wv - 1);
    pb += __builtin_amdgcn_readlane(tb, wv - 1);
    const int32_t m = __builtin_amdgcn_readlane(tm, wv - 1);
    pm = m > pm ? m : pm;
  }
  v.a += pa; v.b += pb;
  v.xm = lane == 0 ? pm : (below > pm ? below : pm);
  v.m = pm > v.m ? pm : v.m;
  lds_barrier();
  if (tid == 1023) { carry[0] = v.a; carry[1] = v.b; carry[2] = v.m; }
  return v;                                 // the new carry is visible after the caller's next barrier
}

// The same for one sum.
__device__ __forceinline__ int32_t block_scan1(int32_t v, int32_t* wave_tot, int32_t* carry) {
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  v = wave_scan_add(v);
  if (lane == 63) wave_tot[wv] = v;
  lds_barrier();
  const int32_t t = wave_scan_add(lane < 16 ? wave_tot[lane] : 0);
  v += *carry + (wv > 0 ? __builtin_amdgcn_readlane(t, wv - 1) : 0);
  lds_barrier();
  if (tid == 1023) *carry = v;
  return v;
}

// Small frames: everything between k_mark and k_emit in one workgroup and one launch.  The marked bits
// are staged in LDS (and the mark bitmap left zero for the next call), and the per-window and per-tile
// tables stay in LDS between the steps: the kernel reads the bitmaps and writes its results, with no
// trip through memory in between.  (Each step is a few microseconds of work; as separate launches their
// start-up and the gaps between them are most of a partition's latency, which the first layer of a
// frame has to wait for.)
// Dynamic LDS, in 32-bit words: bitmaps [ax.n * n_words] | per window: voxels, first set, rows before
// it, tiles started before it, last rows before it [5 * n_windows] | per tile: first set, rows before it [2 * (tile_cap + 1)],
// launch slot [tile_cap] | when there is room, 9 bytes per set for the filled tiles.
template <int NAX>
__global__ void __launch_bounds__(1024) k_front(Jobs jobs) {
  const Job& J = jobs.j[blockIdx.x];
  const PartGeom& g = J.g;
  const AxisSet& ax = J.ax;
  const TileOut& out = J.out;
  int32_t* __restrict__ win_count = J.win_count;
  int32_t* __restrict__ win_soff = J.win_soff;
  int32_t* __restrict__ n_sets = J.n_sets;
  int32_t* __restrict__ status = J.status;
  int32_t* __restrict__ set_loc = J.set_loc;
  const int32_t n_words = J.n_words, max_sets = J.max_sets, set_cap = J.set_cap, tile_cap = J.tile_cap;
  extern __shared__ uint32_t smem[];
  __shared__ int32_t wave_tot[3][16], carry1[3], carry2[3];
  __shared__ int32_t p_cap, over_s, over_p;
  __shared__ int32_t hist[32], running[32], wave_cnt[16][32];
  const int32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int32_t nw = g.n_windows, wpw = g.words_per_win, tau = g.tau;
  const bool want_tiles = out.tile_desc[0] != nullptr;
  const int32_t tile_lim = out.max_tiles < tile_cap ? out.max_tiles : tile_cap;
  uint32_t* bm = smem;
  int32_t* wN = (int32_t*)(smem + (size_t)NAX * n_words);
  int32_t *wSoff = wN + nw, *wP0 = wSoff + nw, *wT0 = wP0 + nw, *wPrev = wT0 + nw;
  int32_t *tFirst = wPrev + nw, *tRows = tFirst + tile_cap + 1, *tPos = tRows + tile_cap + 1;
  const int32_t fill_sets = J.fill_sets;                    // tables of the filled tiles (see fill_tile_starts)
  int32_t* setP = tPos + tile_cap;                           // [fill_sets + 1] rows before every set
  uint16_t* jump = reinterpret_cast<uint16_t*>(setP + fill_sets + 1);
  uint16_t* jump2 = jump + fill_sets + 1;
  uint8_t* mark = reinterpret_cast<uint8_t*>(jump2 + fill_sets + 1);

  if (!ws_ready(ax)) {                       // (k_mark has raised DSVT_ST_WS_STATE)
    if (tid == 0) {
      *n_sets = 0;
      if (want_tiles) { *out.n_tiles = 0; out.tile_first[0] = 0; }
    }
    return;
  }
  if (tid == 0) {
    carry1[0] = carry1[1] = 0; carry1[2] = -1;
    carry2[0] = carry2[1] = 0; carry2[2] = -1;
    p_cap = 0; over_s = -1; over_p = 0;
  }
  // ---- the marked bits: into LDS and into this call's copy for k_emit; the mark bitmap is left zero
  constexpr int32_t kStage = 8;                               // loads in flight per thread and axis
  for (int32_t i0 = tid; i0 < n_words; i0 += kStage * 1024) {
    uint32_t v[NAX][kStage];
#pragma unroll
    for (int32_t k = 0; k < NAX; ++k)
#pragma unroll
      for (int32_t u = 0; u < kStage; ++u) v[k][u] = i0 + u * 1024 < n_words ? ax.a[k].mark[i0 + u * 1024] : 0u;
#pragma unroll
    for (int32_t k = 0; k < NAX; ++k)
#pragma unroll
      for (int32_t u = 0; u < kStage; ++u) {
        const int32_t i = i0 + u * 1024;
        if (i < n_words) { bm[k * n_words + i] = v[k][u]; ax.a[k].mark[i] = 0u; ax.a[k].bitmap[i] = v[k][u]; }
      }
  }
  lds_barrier();
  // ---- a thread per window: count, word prefixes, then scans over the windows of (sets, padded rows,
  // last set's rows of the latest non-empty window) and of the tiles its sets start
  for (int32_t base = 0; base < nw; base += 1024) {
    const int32_t w = base + tid;
    int32_t N = 0;
    if (w < nw) {
      const uint32_t w0 = __umul24((uint32_t)w, (uint32_t)wpw);        // (n_words < 2^22)
      if (wpw <= kRankWords) {                                // k_emit ranks a voxel from the bitmap words themselves
        uint32_t v[kRankWords];
#pragma unroll
        for (int32_t j = 0; j < kRankWords; ++j) v[j] = j < wpw ? bm[w0 + j] : 0u;
#pragma unroll
        for (int32_t j = 0; j < kRankWords; ++j) N += __popc(v[j]);
      } else {
#pragma unroll
        for (int32_t k = 0; k < NAX; ++k) {
          uint32_t* dst_p = ax.a[k].prefix + w0;
          uint32_t run = 0;
          for (int32_t j = 0; j < wpw; ++j) {
            dst_p[j] = run;
            run += (uint32_t)__popc(bm[k * n_words + w0 + j]);
          }
          N = (int32_t)run;                                   // the same for every axis
        }
      }
      win_count[w] = N;
    }
    const int32_t S = (int32_t)div_magic((uint32_t)(N + tau - 1), g.magic_tau);
    SetWalk walk(N, S, tau);
    int32_t R = 0, last_rows = 0;
    for (int32_t j = 0; j < S; ++j) { last_rows = set_rows(walk.next()); R += last_rows; }
    Scan3 v = {S, R, S > 0 ? (w << 7) | last_rows : -1, -1};
    v = block_scan3(v, wave_tot, carry1);
    if (w < nw) {
      win_soff[w] = v.a - S;
      wN[w] = N; wSoff[w] = v.a - S; wP0[w] = v.b - R;
      wPrev[w] = v.xm;                          // (window << 7 | rows of its last set) of the latest non-empty window before
    }
  }
  lds_barrier();
  const int32_t rows_per_cut = tile_cut(carry1[1], J.rows_per_cut);
  bool filled = false;
  if (want_tiles && fill_sets > 0 && carry1[0] <= fill_sets && carry1[0] <= set_cap && carry1[0] < 65535 &&
      fill_wanted(carry1[1], carry1[0], J.rows_per_cut)) {
    for (int32_t w = tid; w < nw; w += 1024) {               // rows before every set
      const int32_t N = wN[w], S = (int32_t)div_magic((uint32_t)(N + tau - 1), g.magic_tau), soff = wSoff[w];
      SetWalk walk(N, S, tau);
      int32_t P = wP0[w];
      for (int32_t j = 0; j < S; ++j) {
        setP[soff + j] = P;
        P += set_rows(walk.next());
      }
    }
    if (tid == 0) setP[carry1[0]] = carry1[1];
    lds_barrier();
    filled = fill_tiles(setP, jump, jump2, mark, carry1[0], J.rows_per_cut);
  }

  // ---- the tiles every window's sets start, and a scan of their number
  for (int32_t base = 0; want_tiles && base < nw; base += 1024) {
    const int32_t w = base + tid;
    const int32_t N = w < nw ? wN[w] : 0, soff = w < nw ? wSoff[w] : 0, P0 = w < nw ? wP0[w] : 0, prev = w < nw ? wPrev[w] : -1;
    const int32_t S = (int32_t)div_magic((uint32_t)(N + tau - 1), g.magic_tau);
    SetWalk walk(N, S, tau);
    // Set s starts a tile when a multiple of rows_per_cut lies in (rows before set s - 1, rows before set s],
    // that is when (rows before set s - 1) mod rows_per_cut plus the rows of set s - 1 reach rows_per_cut.
    const int32_t prev_rows0 = prev >= 0 ? (prev & 127) : 0;
    const uint32_t d0 = (uint32_t)(P0 - prev_rows0);          // rows before the previous set
    const int32_t m0 = (int32_t)(d0 % (uint32_t)rows_per_cut);
    auto for_each_set = [&](auto&& fn) {
      int32_t P = P0, pr = prev_rows0, m = m0;
      walk.restart();
      for (int32_t j = 0; j < S; ++j) {
        const int32_t s = soff + j;
        if (s == set_cap) p_cap = P;
        if (s >= set_cap) break;
        const bool first = filled ? mark[s] != 0 : (s == 0 || m + pr >= rows_per_cut);
        m += pr;
        while (m >= rows_per_cut) m -= rows_per_cut;
        fn(s, P, first);
        pr = set_rows(walk.next());
        P += pr;
      }
    };
    int32_t F = 0;
    for_each_set([&](int32_t, int32_t, bool first) { F += first ? 1 : 0; });
    const int32_t f_incl = block_scan1(F, wave_tot[0], carry2);
    if (w < nw) {
      int32_t t = f_incl - F;                                 // tiles started before this window
      wT0[w] = t;
      for_each_set([&](int32_t s, int32_t P, bool first) {
        if (!first) return;
        if (t < tile_lim) { tFirst[t] = s; tRows[t] = P; out.tile_first[t] = s; }
        else if (t == tile_lim) { over_s = s; over_p = P; }        // first set that no tile is left for
        ++t;
      });
    }
  }
  lds_barrier();
  const int32_t n_tot = carry1[0];
  if (tid == 0) {
    *n_sets = n_tot;
    if (n_tot > max_sets) atomicOr(status, DSVT_ST_SET_OVERFLOW);
  }
  if (!want_tiles) return;
  const bool tiles_short = carry2[0] > tile_lim;          // the caller's list is shorter than the frame needs: later sets get no tile
  const int32_t n_eff = tiles_short ? over_s : (n_tot < set_cap ? n_tot : set_cap);
  const int32_t nt = tiles_short ? tile_lim : carry2[0];
  if (tiles_short && tid == 0) atomicOr(status, DSVT_ST_TILE_OVERFLOW);
  if (n_eff <= 0) {
    if (tid == 0) { *out.n_tiles = 0; out.tile_first[0] = 0; }
    return;
  }
  if (tid == 0) {
    *out.n_tiles = nt;
    out.tile_first[nt] = n_eff;
    tFirst[nt] = n_eff;
    tRows[nt] = tiles_short ? over_p : (n_tot <= set_cap ? carry1[1] : p_cap);
  }
  if (tid < 32) hist[tid] = 0;
  lds_barrier();

  // ---- launch order = tiles with more rows first (a stable counting sort on rows / 4), so that the
  // short tiles fill the tail of the launch
  for (int32_t base = 0; base < nt; base += 1024) {
    const int32_t t = base + tid;
    if (t < nt) {
      int32_t b = 24 - (tRows[t + 1] - tRows[t]) / 4;
      b = b < 0 ? 0 : (b > 31 ? 31 : b);
      atomicAdd(&hist[b], 1);
    }
  }
  lds_barrier();
  if (wv == 0) {
    const int32_t h = lane < 32 ? hist[lane] : 0, incl = wave_scan_add(h);
    if (lane < 32) running[lane] = incl - h;
  }
  lds_barrier();
  for (int32_t base = 0; base < nt; base += 1024) {
    const int32_t t = base + tid;
    int32_t b = -1;
    if (t < nt) {
      b = 24 - (tRows[t + 1] - tRows[t]) / 4;
      b = b < 0 ? 0 : (b > 31 ? 31 : b);
    }
    for (int32_t k = lane; k < 32; k += 64) wave_cnt[wv][k] = 0;
    // lanes of this wavefront with the same bucket: those that agree with this lane in each of its 5 bits
    unsigned long long same = __ballot(b >= 0);
#pragma unroll
    for (int32_t bit = 0; bit < 5; ++bit) {
      const bool one = (b >> bit) & 1;
      const unsigned long long ones = __ballot(one);
      same &= one ? ones : ~ones;
    }
    const unsigned long long below = same & ((1ull << lane) - 1ull);
    const int32_t rank = __popcll(below);                     // among this wavefront's lanes of the same bucket
    if (b >= 0 && below == 0ull) wave_cnt[wv][b] = __popcll(same);
    lds_barrier();
    if (tid < 512) {                                          // a row of 16 lanes per bucket, a lane per wavefront:
      const int32_t bb = tid >> 4, k = tid & 15;              // counts of the wavefronts -> first position of each
      const int32_t cnt = wave_cnt[k][bb];
      int32_t incl = cnt;
      incl += dpp_or<0x111, 0xF>(0, incl);
      incl += dpp_or<0x112, 0xF>(0, incl);
      incl += dpp_or<0x114, 0xF>(0, incl);
      incl += dpp_or<0x118, 0xF>(0, incl);
      const int32_t first = running[bb];
      wave_cnt[k][bb] = first + incl - cnt;
      if (k == 15) running[bb] = first + incl;                // (read by this row only, all of it before this write)
    }
    lds_barrier();
    if (b >= 0) {
      const int32_t pos = wave_cnt[wv][b] + rank;
      out.tile_order[pos] = t;
      tPos[t] = pos;
      desc_header(out, pos, tRows[t + 1] - tRows[t], tFirst[t + 1] - tFirst[t]);
    }
    lds_barrier();
  }
  // ---- per set: its descriptor slot, its place among the tile's sets and its first row, for k_emit
  for (int32_t w = tid; w < nw; w += 1024) {
    const int32_t N = wN[w], S = (int32_t)div_magic((uint32_t)(N + tau - 1), g.magic_tau), soff = wSoff[w];
    int32_t P = wP0[w], t = wT0[w] - 1;
    SetWalk walk(N, S, tau);
    for (int32_t j = 0; j < S; ++j) {
      const int32_t s = soff + j;
      if (s >= set_cap) break;
      const int32_t nu = walk.next();
      if (t + 1 < nt && tFirst[t + 1] == s) ++t;
      int32_t loc = -1;
      if (t >= 0 && t < nt && s < n_eff) {
        const int32_t pos = tPos[t], ls = s - tFirst[t], r0 = P - tRows[t];
        if (ls >= 0 && ls < kDescSets && r0 >= 0 && r0 <= kTileRows - 4) loc = set_loc_code(pos, ls, r0);
      }
      set_loc[s] = loc;
      P += set_rows(nu);
    }
  }
}

// One thread per voxel, axis (blockIdx.y) and job (blockIdx.z): rank d inside its window, then the slots t with
// floor(t*N/(S*tau)) == d; with a work list also the voxel's row of its tile descriptor.  The blocks
// after the voxels' (blockIdx.x >= vox_blocks) put -1 into the descriptor rows past each tile's last.
__global__ void k_emit(Jobs jobs, const int4* __restrict__ coords, int32_t n, int32_t vox_blocks) {
  const Job& J = jobs.j[blockIdx.z];
  const PartGeom& g = J.g;
  const AxisSet& ax = J.ax;
  if ((int32_t)blockIdx.y >= ax.n) return;
  const int32_t* __restrict__ win_count = J.win_count;
  const int32_t* __restrict__ win_soff = J.win_soff;
  int32_t* __restrict__ set_win = J.set_win;
  const int32_t* __restrict__ set_loc = J.set_loc;
  const int32_t* __restrict__ n_tiles = J.out.n_tiles;
  const int32_t max_sets = J.set_cap, n_desc_slots = J.out.max_tiles;
  const AxisBufs& me = ax.a[blockIdx.y];
  int32_t* __restrict__ tile_desc = me.tile_desc;
  if ((int32_t)blockIdx.x >= vox_blocks) {
    if (tile_desc == nullptr || !ws_ready(ax)) return;
    // 16 threads per descriptor share the rows past the tile's last
    const int32_t idx = ((int32_t)blockIdx.x - vox_blocks) * blockDim.x + threadIdx.x;
    const int32_t pos = idx >> 4, part = idx & 15;
    int32_t nt = *n_tiles;
    nt = nt < n_desc_slots ? nt : n_desc_slots;
    if (pos >= nt) return;
    int32_t* dd = tile_desc + (int64_t)pos * kDescInts;
    const int32_t rows = dd[0];
    for (int32_t r = rows + part; r < kTileRows; r += 16) *reinterpret_cast<int2*>(dd + kDescRow + 2 * r) = make_int2(-1, -1);
    return;
  }
  int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int4 c = coords[i];
  uint32_t wkey; int32_t xi, yi, zi;
  if (!ws_ready(ax) || !voxel_cell(g, c, wkey, xi, yi, zi)) { me.voxel_slot[i] = -1; return; }
  const uint32_t key = voxel_key(g, ax.axis0 + (int32_t)blockIdx.y, wkey, xi, yi, zi);
  const int32_t tau = g.tau;
  uint32_t word = key >> 5, bit = key & 31u;
  const int32_t w = (int32_t)wkey;
  int64_t d = (uint32_t)__popc(me.bitmap[word] & ((1u << bit) - 1u));          // set bits before its own inside its window
  if (g.words_per_win <= kRankWords) {
    const uint32_t w0 = wkey * (uint32_t)g.words_per_win;
    uint32_t v[kRankWords];
#pragma unroll
    for (int32_t j = 0; j < kRankWords; ++j) v[j] = w0 + j < word ? me.bitmap[w0 + j] : 0u;
#pragma unroll
    for (int32_t j = 0; j < kRankWords; ++j) d += __popc(v[j]);
  } else {
    d += me.prefix[word];
  }
  int64_t N = win_count[w];
  int64_t S = (N + tau - 1) / tau, T = S * tau;
  if (((ax.axis0 + (int32_t)blockIdx.y) >> 1) == 2 && S > 1) {
    // "Sparse" baseline (Sec. 4.4): every subset spread over the whole window.  The voxel of rank d goes behind
    // all voxels of a smaller residue d mod S (residues below N mod S hold one voxel more), then Eq. 3 as usual.
    const int64_t q = N / S, rem = N - q * S, r = d % S;
    d = r * q + (r < rem ? r : rem) + d / S;
  }
  int64_t t_lo, t_hi, first_d;                               // first_d: rank of the first voxel of this voxel's first set
  if (N > 0 && N < 32768 && T < 65536) {                     // the usual case: 32-bit division
    const uint32_t nn = (uint32_t)N, tt = (uint32_t)T, dd = (uint32_t)d;
    const uint32_t lo = (dd * tt + nn - 1u) / nn, hi = ((dd + 1u) * tt + nn - 1u) / nn;
    t_lo = lo; t_hi = hi;
    first_d = ((lo / (uint32_t)tau) * (uint32_t)tau * nn) / tt;
  } else {
    t_lo = (d * T + N - 1) / N; t_hi = ((d + 1) * T + N - 1) / N;
    first_d = ((t_lo / tau) * tau * N) / T;
  }
  int64_t base = (int64_t)win_soff[w] * tau, cap = (int64_t)max_sets * tau;
  me.voxel_slot[i] = (int32_t)(base + t_lo);
  const int32_t j_first = (int32_t)t_lo / tau;               // (t < S * tau and slots < max_sets * tau fit 32 bits)
  int32_t next_set_start = (int32_t)t_lo == j_first * tau ? (int32_t)t_lo : (j_first + 1) * tau;
  const bool names_sets = blockIdx.y == 0;                   // the window of a set is the same for every axis
  for (int32_t t = (int32_t)t_lo; t < (int32_t)t_hi; ++t) {
    const int64_t slot = base + t;
    if (slot >= cap) break;
    me.set_inds[slot] = i;
    if (t == next_set_start) {                               // the first slot of a set: this thread describes the set
      const int32_t j = t / tau, s = win_soff[w] + j;
      if (names_sets) set_win[s] = w;
      if (tile_desc != nullptr) {
        const int32_t loc = set_loc[s];
        if (loc >= 0 && (loc >> 12) < n_desc_slots)
          desc_set(tile_desc + (int64_t)(loc >> 12) * kDescInts, (loc >> 7) & 31, loc & 127, set_distinct(N, S, j, tau));
      }
      next_set_start += tau;
    }
  }
  if (tile_desc != nullptr) {
    const int64_t j = j_first, s = win_soff[w] + j;
    if (s < max_sets) {
      const int32_t loc = set_loc[s];
      const int32_t slot = loc >> 12, row = (loc & 127) + (int32_t)(d - first_d);
      if (slot >= 0 && slot < n_desc_slots && row < kTileRows) {
        const int32_t lin = (c.y * (2 * g.win[1] - 1) + c.z) * (2 * g.win[2] - 1) + c.w;
        int32_t* dd = tile_desc + (int64_t)slot * kDescInts;
        *reinterpret_cast<int2*>(dd + kDescRow + 2 * row) = make_int2(i, (int32_t)((uint32_t)lin | ((uint32_t)(t_hi - t_lo) << 24)));
      }
    }
  }
}

struct PartPlan {
  PartGeom g;
  size_t off_mark, off_bitmap, off_prefix, off_count, off_soff, off_setwin, off_piecehist, off_setloc, total;
  bool desc_ok;
  int64_t n_words;
  int32_t set_bound, tile_bound, rows_per_cut;
};

int make_plan(const dsvt_part_cfg* cfg, int32_t n_voxels, PartPlan* p) {
  if (cfg == nullptr || n_voxels <= 0 || cfg->tau <= 0 || cfg->batch <= 0 || cfg->axis < 0 || cfg->axis > 5)
    return DSVT_EINVAL;
  PartGeom& g = p->g;
  int64_t vol = 1, nwin = cfg->batch;
  for (int a = 0; a < 3; ++a) {
    if (cfg->grid[a] <= 0 || cfg->win[a] <= 0 || cfg->shift[a] < 0 || cfg->shift[a] >= cfg->win[a]) return DSVT_EINVAL;
    g.grid[a] = cfg->grid[a]; g.win[a] = cfg->win[a]; g.shift[a] = cfg->shift[a];
    g.nw[a] = (int32_t)dsvt_ceil_div((int64_t)cfg->grid[a] + cfg->shift[a], cfg->win[a]);
    g.magic[a] = (cfg->win[a] > 1 && cfg->win[a] < (1 << 15) && (int64_t)cfg->grid[a] + cfg->shift[a] < (1 << 16))
                     ? (uint32_t)(((1ull << 32) + (uint64_t)cfg->win[a] - 1) / (uint64_t)cfg->win[a]) : 0u;
    vol *= cfg->win[a];
    nwin *= g.nw[a];
    if (vol >= (1ll << 31) || nwin >= (1ll << 31)) return DSVT_EINVAL;
  }
  g.batch = cfg->batch; g.tau = cfg->tau;
  g.magic_tau = 0u;
  g.vol = (uint32_t)vol;
  if ((cfg->axis >> 1) == 1 && vol > (1 << 16)) return DSVT_EUNSUPPORTED;   // key * mul must fit 32 bits
  for (int odd = 0; odd < 2; ++odd) {
    int64_t mul = (int64_t)(0.618 * (double)vol);
    mul = (mul < 1 ? 1 : mul) + odd;
    auto gcd = [](int64_t a, int64_t b) { while (b) { const int64_t t = a % b; a = b; b = t; } return a; };
    while (gcd(mul, vol) != 1) ++mul;
    g.shuf_mul[odd] = (uint32_t)(mul % vol);
    g.shuf_add[odd] = (uint32_t)((vol / 3 + odd) % vol);
  }
  int64_t wpw = dsvt_ceil_div(vol, 32);
  if (nwin * wpw * 32 >= (1ll << 31)) return DSVT_EINVAL;   // composite keys are 32-bit
  g.words_per_win = (int32_t)wpw;
  g.n_windows = (int32_t)nwin;
  p->n_words = nwin * wpw;
  size_t o = kWsHeader;                                     // bitmaps and prefixes: room for both axes, back to back
  p->off_mark = o;   o = dsvt_align_up(o + (size_t)p->n_words * 8, 256);
  p->off_bitmap = o; o = dsvt_align_up(o + (size_t)p->n_words * 8, 256);
  p->off_prefix = o; o = dsvt_align_up(o + (size_t)p->n_words * 8, 256);
  p->off_count = o;  o = dsvt_align_up(o + (size_t)nwin * 4, 256);
  p->off_soff = o;   o = dsvt_align_up(o + (size_t)nwin * 4, 256);
  const int64_t bound = n_voxels / cfg->tau + (n_voxels < nwin ? n_voxels : nwin);
  if (bound * cfg->tau >= (1ll << 31)) return DSVT_EINVAL;
  p->set_bound = (int32_t)bound;
  p->off_setwin = o; o = dsvt_align_up(o + (size_t)bound * 4, 256);
  // tiles of the layer kernels: 96 rows, every set padded to a multiple of 4 rows.  The sets of a window
  // with N voxels list at most N + S - 1 distinct voxels (neighbours may share one), so all sets
  // together have at most n + 4 * bound rows, and every rows_per_cut of them start at most one tile.
  const int64_t pad_tau = (cfg->tau + 3) & ~3;
  p->rows_per_cut = (int32_t)(100 - pad_tau);
  p->tile_bound = p->rows_per_cut > 0 ? (int32_t)((n_voxels + 4 * bound) / p->rows_per_cut + 1 + kComputeUnits) : 0;   // (see tile_cut)
  p->off_piecehist = o; o = dsvt_align_up(o + (size_t)(bound / kTilePiece + 1) * 32 * 4, 256);   // (see build_tiles)
  p->off_setloc = o;   o = dsvt_align_up(o + (size_t)(bound + 1) * 4, 256);
  // set_loc packs (slot << 12 | place << 7 | row), a descriptor (multiplicity << 24 | position code) into 32 bits
  p->desc_ok = p->rows_per_cut >= 4 && p->tile_bound < (1 << 19) &&
               (int64_t)cfg->grid[0] * (2 * cfg->win[1] - 1) * (2 * cfg->win[2] - 1) < (1 << 24) && cfg->tau < 128;
  p->total = o;
  return DSVT_OK;
}

// Header value of a scratch buffer whose mark bitmaps (room for both axes) are zero for this geometry.
uint64_t ws_token(const PartPlan& p) { return kWsMagic ^ ((uint64_t)p.n_words * 0x9E3779B97F4A7C15ull); }

// What one window configuration asks for (host side).
struct PartRequest {
  const dsvt_part_cfg* cfg;
  int32_t n_axes, axis0;
  int32_t* set_inds[2];
  int32_t* voxel_slot[2];
  int32_t *n_sets, *set_win;
  int32_t max_sets;
  const dsvt_tile_list* tiles;
  int32_t* tile_desc_2;
  void* ws;
  size_t ws_bytes;
  int32_t* status;
};

struct Prepared {
  PartPlan p;
  Job job;
  bool want_tiles, front_ok;
  size_t front_lds;
};

// Checks one request and lays out its job.
int prepare(const PartRequest& r, int32_t n_voxels, Prepared* out) {
  PartPlan& p = out->p;
  int rc = make_plan(r.cfg, n_voxels, &p);
  if (rc != DSVT_OK) return rc;
  if (!r.n_sets || !r.ws || !r.status || r.max_sets <= 0) return DSVT_EINVAL;
  for (int32_t k = 0; k < r.n_axes; ++k)
    if (!r.set_inds[k] || !r.voxel_slot[k]) return DSVT_EINVAL;
  if ((int64_t)r.max_sets * r.cfg->tau >= (1ll << 31)) return DSVT_EINVAL;
  if (r.ws_bytes < p.total) return DSVT_ENOSPC;
  Job& J = out->job;
  J = Job{};
  TileOut& tout = J.out;
  out->want_tiles = r.tiles != nullptr;
  if (r.tiles != nullptr) {
    const dsvt_tile_list* t = r.tiles;
    if (!t->tile_first || !t->n_tiles || !t->tile_order || !t->tile_desc || t->max_tiles <= 0) return DSVT_EINVAL;
    if (r.n_axes == 2 && !r.tile_desc_2) return DSVT_EINVAL;
    if (((uintptr_t)t->tile_desc | (uintptr_t)r.tile_desc_2) & 7u) return DSVT_EINVAL;   // a row's two words go out as one 8-byte store
    if (!p.desc_ok) return DSVT_EUNSUPPORTED;
    tout.tile_first = t->tile_first; tout.n_tiles = t->n_tiles; tout.tile_order = t->tile_order;
    tout.tile_desc[0] = t->tile_desc;
    tout.tile_desc[1] = r.n_axes == 2 ? r.tile_desc_2 : nullptr;
    tout.max_tiles = t->max_tiles < p.tile_bound ? t->max_tiles : p.tile_bound;   // scratch is sized for the bound
  }
  char* base = (char*)r.ws;
  J.win_count = (int32_t*)(base + p.off_count);
  J.win_soff = (int32_t*)(base + p.off_soff);
  J.set_loc = (int32_t*)(base + p.off_setloc);
  J.n_sets = r.n_sets;
  J.status = r.status;
  // window key of every set: the caller's array, or scratch when it is not wanted (k_emit rewrites the same values there)
  J.set_win = r.set_win != nullptr ? r.set_win : (int32_t*)(base + p.off_setwin);
  J.n_words = (int32_t)p.n_words;
  J.max_sets = r.max_sets;
  J.set_cap = r.max_sets < p.set_bound ? r.max_sets : p.set_bound;
  J.rows_per_cut = p.rows_per_cut;
  J.tile_cap = p.tile_bound;
  AxisSet& ax = J.ax;
  ax.n = r.n_axes; ax.axis0 = r.axis0;
  for (int32_t k = 0; k < r.n_axes; ++k) {
    ax.a[k].mark = (uint32_t*)(base + p.off_mark) + (size_t)k * p.n_words;
    ax.a[k].bitmap = (uint32_t*)(base + p.off_bitmap) + (size_t)k * p.n_words;
    ax.a[k].prefix = (uint32_t*)(base + p.off_prefix) + (size_t)k * p.n_words;
    ax.a[k].set_inds = r.set_inds[k]; ax.a[k].voxel_slot = r.voxel_slot[k];
    ax.a[k].tile_desc = tout.tile_desc[k];
  }
  ax.ws_token = (const uint64_t*)base;
  ax.token = ws_token(p);
  // k_front divides by tau by multiplying: exact for x < 2^16 and d < 2^15 (tau against a window's volume + tau)
  const int32_t tau = r.cfg->tau;
  out->front_ok = (int64_t)p.g.words_per_win * 32 + tau < (1 << 16) && tau < (1 << 15) && tau > 1 &&
                  (int64_t)n_voxels + 4 * (int64_t)p.set_bound < (1 << 25) && p.g.n_windows < (1 << 22) &&
                  p.n_words * r.n_axes < (1 << 22) && (r.tiles == nullptr || p.rows_per_cut >= 2);
  if (out->front_ok) {
    p.g.magic_tau = (uint32_t)(((1ull << 32) + (uint64_t)tau - 1) / (uint64_t)tau);
  }
  out->front_lds = ((size_t)r.n_axes * p.n_words + 5 * (size_t)p.g.n_windows + 3 * (size_t)(p.tile_bound + 1)) * 4;
  out->front_ok = out->front_ok && out->front_lds <= kFrontLds;
  const size_t fill_lds = ((size_t)p.set_bound + 1) * 9 + 16;    // rows before every set, two jump tables, marks
  J.fill_sets = 0;
  if (r.tiles != nullptr && p.set_bound < 65535 && out->front_lds + fill_lds <= kFrontLds) {
    J.fill_sets = p.set_bound;
    out->front_lds += fill_lds;
  }
  // Frames for the general front end, X-/Y-axis pair of the plain or the "Sparse" order (their bitmaps are keyed alike):
  // the Y-order bits of a window are its X-order bits with x and y exchanged, so only the X-order bits are set by
  // atomics and k_window_count derives the others window by window (half the atomics of k_mark).
  J.derive_y = (!out->front_ok && r.n_axes == 2 && (r.axis0 & ~4) == 0 && p.g.vol <= (1u << 16)) ? 1 : 0;
  J.g = p.g;
  return DSVT_OK;
}

// The partitions of n window configurations over the same voxels (n_axes inner orders each): one
// launch per step when every configuration fits k_front, else one configuration after the other.
int run_partitions(const PartRequest* reqs, int32_t n, const int32_t* coords, int32_t n_voxels, void* stream) {
  if (n <= 0 || n > kMaxJobs || !reqs || !coords) return DSVT_EINVAL;
  Prepared prep[kMaxJobs];
  for (int32_t q = 0; q < n; ++q) {
    if (reqs[q].cfg == nullptr || reqs[q].n_axes != reqs[0].n_axes) return DSVT_EINVAL;
    int rc = prepare(reqs[q], n_voxels, &prep[q]);
    if (rc != DSVT_OK) return rc;
  }
  hipStream_t st = (hipStream_t)stream;
  const int tb = 256;
  const int32_t n_axes = reqs[0].n_axes;
  const int32_t vox_blocks = (int32_t)dsvt_ceil_div(n_voxels, tb);
  // One chain of launches for all jobs: mark, then the single-workgroup front end for the jobs it can hold and
  // the general one (three launches) for the others, then emit.
  Jobs jobs = {}, front_jobs = {}, gen_jobs = {};
  GenJobs gen = {};
  int32_t n_front = 0, n_gen = 0, max_tiles = 0, any_tiles = 0, any_merged = 0, tile_pieces = 0;
  size_t front_lds = 0, fill_lds = 0, count_lds = 0;
  int64_t count_threads = 0;
  for (int32_t q = 0; q < n; ++q) {
    const Prepared& P = prep[q];
    jobs.j[q] = P.job;
    max_tiles = P.job.out.max_tiles > max_tiles ? P.job.out.max_tiles : max_tiles;
    if (P.front_ok) {
      front_jobs.j[n_front++] = P.job;
      front_lds = P.front_lds > front_lds ? P.front_lds : front_lds;
    } else {
      const PartPlan& p = P.p;
      char* base = (char*)reqs[q].ws;
      GenJob& G = gen.j[n_gen];
      G.ws_setwin = (int32_t*)(base + p.off_setwin);
      G.piece_hist = (int32_t*)(base + p.off_piecehist);
      G.set_bound = p.set_bound;
      G.want_tiles = P.want_tiles ? 1 : 0;
      // LDS tables of the work-list builder (see build_tiles_lds; 9 bytes per set): for the whole frame if it has at
      // most kFillMax sets, else for the pieces it is taken in (see build_tiles)
      constexpr int32_t kFillMax = 16384;
      G.fill_sets = P.want_tiles ? (p.set_bound < kFillMax ? p.set_bound : kFillMax) : 0;
      const size_t need = ((size_t)G.fill_sets + 1) * 9 + 16;
      static_assert(((size_t)kFillMax + 1) * 9 + 16 <= kFrontLds && kTilePiece <= kFillMax, "the tables fit the LDS k_tiles may ask for");
      if (G.want_tiles && p.set_bound > G.fill_sets) {
        const int32_t pieces = (p.set_bound + kTilePiece - 1) / kTilePiece;
        tile_pieces = pieces > tile_pieces ? pieces : tile_pieces;
      }
      if (G.fill_sets) fill_lds = need > fill_lds ? need : fill_lds;
      // every set has a place in the tables: the scan of the windows builds the work list too (no k_tiles launch)
      G.merged = (G.want_tiles && p.set_bound <= G.fill_sets && p.set_bound < 65535 && p.g.tau > 1) ? 1 : 0;
      any_merged |= G.merged;
      any_tiles |= (G.want_tiles && !G.merged) ? 1 : 0;
      int32_t group = 1;
      while (group < 64 && group < p.g.words_per_win) group <<= 1;
      const int64_t threads = (int64_t)p.g.n_windows * group;
      count_threads = threads > count_threads ? threads : count_threads;
      if (P.job.derive_y) {
        const size_t need_y = (size_t)(tb / group) * p.g.words_per_win * 4;
        count_lds = need_y > count_lds ? need_y : count_lds;
      }
      gen_jobs.j[n_gen++] = P.job;
    }
  }
  // Everything that can fail on the host comes before the first launch: once k_mark has run, the mark bitmap
  // holds bits that only the rest of the chain takes out again.
  auto* front = n_axes == 2 ? k_front<2> : k_front<1>;
  if (n_front) {
    static std::atomic<uint64_t> front_allowed[2];
    if (int rc = dsvt_allow_lds((const void*)front, kFrontLds, front_allowed[n_axes - 1])) return rc;
  }
  if (n_gen && any_tiles && fill_lds) {
    static std::atomic<uint64_t> tiles_allowed{0};
    if (int rc = dsvt_allow_lds((const void*)k_tiles, kFrontLds, tiles_allowed)) return rc;
  }
  if (n_gen && any_merged) {
    static std::atomic<uint64_t> scan_allowed{0};
    if (int rc = dsvt_allow_lds((const void*)k_scan_windows, kFrontLds, scan_allowed)) return rc;
  }
  DSVT_HIP_TRY(hipGetLastError());                            // (an error left by an earlier call is not this chain's)
  {
    dsvt_prof_scope ps(DSVT_K_PART_MARK, st);
    k_mark<<<dim3((unsigned)vox_blocks, n), tb, 0, st>>>(jobs, (const int4*)coords, n_voxels);
  }
  if (hipGetLastError() != hipSuccess) return DSVT_EHIP;      // nothing was enqueued
  if (n_front) {
    dsvt_prof_scope ps(DSVT_K_PART_TILES, st);
    front<<<n_front, 1024, front_lds, st>>>(front_jobs);
  }
  if (n_gen) {
    {
      dsvt_prof_scope ps(DSVT_K_PART_COUNT, st);
      k_window_count<<<dim3((unsigned)dsvt_ceil_div(count_threads, tb), n_axes, n_gen), tb, count_lds, st>>>(gen_jobs);
    }
    {
      dsvt_prof_scope ps(DSVT_K_PART_SCAN, st);
      k_scan_windows<<<n_gen, 1024, any_merged ? fill_lds : 0, st>>>(gen_jobs, gen);
    }
    if (any_tiles) {
      dsvt_prof_scope ps(DSVT_K_PART_TILES, st);
      if (tile_pieces) k_tiles<<<dim3(n_gen, tile_pieces), 1024, fill_lds, st>>>(gen_jobs, gen, 0);
      k_tiles<<<dim3(n_gen, tile_pieces ? tile_pieces : 1), 1024, fill_lds, st>>>(gen_jobs, gen, 1);
    }
  }
  {
    dsvt_prof_scope ps(DSVT_K_PART_EMIT, st);
    const int32_t tail_blocks = (int32_t)dsvt_ceil_div((int64_t)max_tiles * 16, tb);
    k_emit<<<dim3((unsigned)(vox_blocks + tail_blocks), n_axes, n), tb, 0, st>>>(jobs, (const int4*)coords, n_voxels, vox_blocks);
  }
  if (hipGetLastError() != hipSuccess) {
    // A launch after k_mark failed: the marked bits may still be there.  The buffers' headers are taken back,
    // so that the next call on them reports DSVT_ST_WS_STATE instead of ranking voxels over stale bits.
    for (int32_t q = 0; q < n; ++q) k_ws_revoke<<<1, 64, 0, st>>>((uint64_t*)reqs[q].ws);
    (void)hipGetLastError();
    return DSVT_EHIP;
  }
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

extern "C" int dsvt_partition_ws_init(const dsvt_part_cfg* cfg, int32_t n_voxels, void* ws, size_t ws_bytes, void* stream) {
  PartPlan p;
  int rc = make_plan(cfg, n_voxels, &p);
  if (rc != DSVT_OK) return rc;
  if (!ws) return DSVT_EINVAL;
  if (ws_bytes < p.total) return DSVT_ENOSPC;
  const int64_t n_clear = p.n_words * 2;
  k_ws_init<<<(unsigned)dsvt_ceil_div(n_clear, 256), 256, 0, (hipStream_t)stream>>>(
      (uint32_t*)((char*)ws + p.off_mark), n_clear, (uint64_t*)ws, ws_token(p));
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}

extern "C" int dsvt_partition(const dsvt_part_cfg* cfg, const int32_t* coords, int32_t n_voxels, int32_t* set_inds,
                              int32_t* voxel_slot, int32_t* n_sets, int32_t max_sets, int32_t* set_win,
                              const dsvt_tile_list* tiles, void* ws, size_t ws_bytes, int32_t* status, void* stream) {
  if (cfg == nullptr) return DSVT_EINVAL;
  const PartRequest r = {cfg, 1, cfg->axis, {set_inds, nullptr}, {voxel_slot, nullptr}, n_sets, set_win, max_sets, tiles,
                         nullptr, ws, ws_bytes, status};
  return run_partitions(&r, 1, coords, n_voxels, stream);
}

extern "C" int dsvt_partition_xy(const dsvt_part_cfg* cfg, const int32_t* coords, int32_t n_voxels, int32_t* set_inds_x,
                                 int32_t* set_inds_y, int32_t* voxel_slot_x, int32_t* voxel_slot_y, int32_t* n_sets,
                                 int32_t max_sets, int32_t* set_win, const dsvt_tile_list* tiles, int32_t* tile_desc_y,
                                 void* ws, size_t ws_bytes, int32_t* status, void* stream) {
  if (cfg == nullptr) return DSVT_EINVAL;
  if (cfg->axis & 1) return DSVT_EINVAL;                      // the pair is (axis, axis + 1)
  const PartRequest r = {cfg, 2, cfg->axis, {set_inds_x, set_inds_y}, {voxel_slot_x, voxel_slot_y}, n_sets, set_win, max_sets,
                         tiles, tile_desc_y, ws, ws_bytes, status};
  return run_partitions(&r, 1, coords, n_voxels, stream);
}

extern "C" int dsvt_partition_xy_multi(const dsvt_xy_job* jobs, int32_t n_jobs, const int32_t* coords, int32_t n_voxels,
                                       void* stream) {
  if (jobs == nullptr || n_jobs <= 0 || n_jobs > kMaxJobs) return DSVT_EINVAL;
  PartRequest r[kMaxJobs];
  for (int32_t q = 0; q < n_jobs; ++q) {
    const dsvt_xy_job& j = jobs[q];
    if (j.cfg.axis & 1) return DSVT_EINVAL;
    r[q] = PartRequest{&j.cfg, 2, j.cfg.axis, {j.set_inds_x, j.set_inds_y}, {j.voxel_slot_x, j.voxel_slot_y}, j.n_sets,
                       j.set_win, j.max_sets, j.tiles, j.tile_desc_y, j.ws, j.ws_bytes, j.status};
  }
  return run_partitions(r, n_jobs, coords, n_voxels, stream);
}
