// dsvt_attn_pool: attention-style 3D pooling (Sec. 3.3, Eq. 6-7) on gfx950.
//
// Grouping: pooled cells are unique keys in a bounded grid, so -- as in the set partition -- the
// output order (ascending region key) comes from an occupancy bitmap and a pop-count prefix, with
// no sort.  Every voxel then writes its index into the dense slot table of its region (Sec. 3.3: a
// sparse pooling region is first laid out densely, one slot per cell).
// Attention: a workgroup takes 48 consecutive regions.  Only their occupied slots become rows of the
// <=96-row LDS tile that the K/V projection runs on (an empty slot's key and value are the two bias
// vectors, whatever the weights); regions whose occupied slots do not fit one tile are taken in
// several passes.  Max-pool over the occupied slots gives the query row (Eq. 6); K/V of the occupied
// slots and Q of the pooled rows are MFMA projections; the P-key softmax per head is plain ALU
// work; output projection, residual and LayerNorm follow the layer kernels (Eq. 7).
#include "common.h"
#include "block_scan.h"
#include "mma.h"

namespace {

constexpr int kMaxPool = 8;                       // slots of a pooling region
constexpr int kRegs = 48;                         // regions (pooled rows) of a workgroup: three MFMA row tiles
constexpr int kSlots = kRegs * kMaxPool;          // their dense slots at most
constexpr int kPoolGrid = 256;                    // workgroups of the attention kernel: the compute units of an MI355X

struct PoolGeom {
  int32_t grid[3], pool[3], pg[3];                // cells, region size, pooled cells per axis
  int32_t batch, P;
};

__global__ void kp_clear(uint32_t* __restrict__ words, int64_t n_words, int32_t* __restrict__ pool_inds, int64_t n_inds) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) words[i] = 0u;
  if (i < n_inds) pool_inds[i] = -1;
}

__device__ __forceinline__ bool pool_key(const PoolGeom& g, int4 c, uint32_t* key, int32_t* slot) {
  const bool ok = c.x >= 0 && c.x < g.batch && c.y >= 0 && c.y < g.grid[0] && c.z >= 0 && c.z < g.grid[1] &&
                  c.w >= 0 && c.w < g.grid[2];
  if (!ok) return false;
  const int32_t px = c.y / g.pool[0], py = c.z / g.pool[1], pz = c.w / g.pool[2];
  *key = (uint32_t)(((c.x * g.pg[0] + px) * g.pg[1] + py) * g.pg[2] + pz);
  *slot = ((c.y - px * g.pool[0]) * g.pool[1] + (c.z - py * g.pool[1])) * g.pool[2] + (c.w - pz * g.pool[2]);
  return true;
}

__global__ void kp_mark(PoolGeom g, const int4* __restrict__ coords, int32_t n, uint32_t* __restrict__ bitmap,
                        int32_t* __restrict__ status) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint32_t key; int32_t slot;
  if (!pool_key(g, coords[i], &key, &slot)) { atomicOr(status, DSVT_ST_COORD_RANGE); return; }
  atomicOr(&bitmap[key >> 5], 1u << (key & 31u));
}

__global__ void kp_emit(PoolGeom g, const int4* __restrict__ coords, int32_t n, const uint32_t* __restrict__ bitmap,
                        const int32_t* __restrict__ word_prefix, int32_t* __restrict__ pool_inds,
                        int32_t* __restrict__ out_coords) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int4 c = coords[i];
  uint32_t key; int32_t slot;
  if (!pool_key(g, c, &key, &slot)) return;
  const uint32_t word = key >> 5, bit = key & 31u;
  const int32_t m = word_prefix[word] + __popc(bitmap[word] & ((1u << bit) - 1u));   // m < number of regions <= n
  pool_inds[(int64_t)m * g.P + slot] = i;
  // every member of a region writes the same pooled coordinates
  reinterpret_cast<int4*>(out_coords)[m] = make_int4(c.x, c.y / g.pool[0], c.z / g.pool[1], c.w / g.pool[2]);
}

struct PoolDev {
  const void *w_kv, *w_q, *w_o;                   // packed: [2C, C] (K rows then V rows), [C, C], [C, C]
  const float *b_kv, *b_q, *b_o, *ln_g, *ln_b;    // b_kv: [2C] in scratch (b_k then b_v)
  float ln_eps;
  int32_t P, mask_empty;
};

// D consecutive elements of an LDS row as floats (16-byte reads when the head width allows).
template <typename T, int D>
__device__ __forceinline__ void load_row(float (&dst)[D], const T* src) {
  constexpr int EPC = 16 / (int)sizeof(T);
  if constexpr (D % EPC == 0) {
#pragma unroll
    for (int c = 0; c < D / EPC; ++c) {
      const uint4 raw = reinterpret_cast<const uint4*>(src)[c];
      const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
      for (int j = 0; j < EPC; ++j) dst[c * EPC + j] = to_f32<T>(e[j]);
    }
  } else {
#pragma unroll
    for (int j = 0; j < D; ++j) dst[j] = to_f32<T>(src[j]);
  }
}


template <typename T, int C> struct PoolLds {
  static constexpr int PAD = lds_pad<T>();
  static constexpr int LDX = C + PAD;
  static constexpr size_t kTile = (size_t)kRowsMax * LDX * sizeof(T);
  static constexpr size_t kQTile = (size_t)kRegs * LDX * sizeof(T);
  static constexpr size_t kStat = (size_t)2 * kStatGroupsMax * kRowsMax * 4;      // LayerNorm partial sums: over Xs, dead by then
  static constexpr size_t off_x = 0, off_k = kTile, off_v = 2 * kTile, off_p = 3 * kTile, off_q = off_p + kQTile;
  static constexpr size_t off_misc = off_q + kQTile;
  // misc: voxel of every slot, occupied slots before it (16 bit), occupied slots before every region, first
  // region of every pass, voxel of every tile row, the bias rows b_k and b_v, per-wavefront counts
  static constexpr size_t off_svox = off_misc, off_scum = off_svox + kSlots * 4, off_rcum = off_scum + kSlots * 2,
                          off_pass = off_rcum + (kRegs + 1) * 4, off_rvox = off_pass + (kMaxPool + 2) * 4,
                          off_bias = (off_rvox + kRowsMax * 4 + 15) / 16 * 16, off_wcnt = off_bias + 2 * C * sizeof(T);
  static constexpr size_t total = off_wcnt + 16 * 4;
  static_assert(kStat <= kTile && total <= 160 * 1024 && off_bias % 16 == 0, "pooling tile does not fit the LDS");
};

// A workgroup walks over groups of kRegs regions (group blockIdx.x, then every gridDim.x-th), software-pipelined: the
// slot table of the next group is requested during the softmax of the current one, and its occupancy scan and the
// request for its rows come before the current group's output projection and LayerNorm, so that the two memory
// round trips of a group (slots, then rows) are behind arithmetic of its predecessor.  One workgroup fits a CU.
template <typename T, int C, int HEADS, int NT_KV, int NT_C>
__global__ void __launch_bounds__(kWaves * 64)
kp_attention(PoolDev p, const int32_t* __restrict__ pool_inds, const int32_t* __restrict__ n_out_ptr,
             const T* __restrict__ x, T* __restrict__ out) {
  typedef PoolLds<T, C> L;
  typedef typename Mma<T>::Vec4 Vec4;
  constexpr int LDX = L::LDX, D = C / HEADS, NW = kWaves, NTHREADS = NW * 64;
  constexpr int CH = C * (int)sizeof(T) / 16, EPC = 16 / (int)sizeof(T);     // 16-byte chunks of a row, elements per chunk
  static_assert(kSlots <= NTHREADS, "one slot per thread");
  extern __shared__ __align__(16) unsigned char smem[];
  T* Xs = reinterpret_cast<T*>(smem + L::off_x);      // occupied slots of the pass, one row each
  T* Ks = reinterpret_cast<T*>(smem + L::off_k);
  T* Vs = reinterpret_cast<T*>(smem + L::off_v);
  T* Ps = reinterpret_cast<T*>(smem + L::off_p);      // pooled rows: query input, residual, finally the output
  T* Qs = reinterpret_cast<T*>(smem + L::off_q);      // Q, then O
  float* stat = reinterpret_cast<float*>(smem + L::off_x);
  int32_t* slot_vox = reinterpret_cast<int32_t*>(smem + L::off_svox);
  uint16_t* slot_cum = reinterpret_cast<uint16_t*>(smem + L::off_scum);
  int32_t* reg_cum = reinterpret_cast<int32_t*>(smem + L::off_rcum);
  int32_t* pass_first = reinterpret_cast<int32_t*>(smem + L::off_pass);
  int32_t* row_vox = reinterpret_cast<int32_t*>(smem + L::off_rvox);
  T* Kb = reinterpret_cast<T*>(smem + L::off_bias);   // key and value of an empty slot
  T* Vb = Kb + C;
  int32_t* wcnt = reinterpret_cast<int32_t*>(smem + L::off_wcnt);
  const int tid0 = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  const int P = p.P;
  const int n_out = __builtin_amdgcn_readfirstlane(*n_out_ptr);
  const int n_groups = (n_out + kRegs - 1) / kRegs;
  if ((int)blockIdx.x >= n_groups) return;
  const int W = kRowsMax + 1 - P;                  // a pass takes the regions whose first occupied slot number lies in one
                                                   // run of W: together at most W - 1 + P = 96 rows
  const float scale = rsqrtf((float)D);
  // (a wavefront's loads return in order: weights are requested after the loads whose results are needed first; the
  // barriers wait for LDS traffic only, so none of them waits for weights or rows still on their way)
  GemmPhase<T, NT_KV, C, 2 * C, NW> kv(reinterpret_cast<const T*>(p.w_kv), wave);
  GemmPhase<T, NT_C, C, C, NW, 2> qp(reinterpret_cast<const T*>(p.w_q), wave);   // C x C phases: 4 feature groups x 2 halves of the row tiles
  GemmPhase<T, NT_C, C, C, NW, 2> op(reinterpret_cast<const T*>(p.w_o), wave);
  constexpr int N_OG = C / (16 * NT_C), RH = kRowTiles / 2;
  static_assert(2 * N_OG == NW && kRegs / 16 <= 2 * RH - 1, "one output-projection item per wavefront");
  const int og_own = wave % N_OG, half = wave / N_OG;
  const int o_own = og_own * 16 * NT_C, rt_own = half ? 2 : 0, HC = half ? kRegs / 16 - 2 : 2;
  constexpr int G = (kRowsMax * CH + NTHREADS - 1) / NTHREADS;      // 16-byte pieces of a pass's rows per thread

  for (int c = tid0; c < 2 * C; c += NTHREADS) Kb[c] = (T)p.b_kv[c];
  auto slot_of = [&](int grp, int tid) {                              // this thread's slot of a group: its voxel or -1
    const int m0 = grp * kRegs, mr = (n_out - m0) < kRegs ? (n_out - m0) : kRegs;
    return tid < mr * P ? pool_inds[(size_t)m0 * P + tid] : -1;
  };
  int v_slot = slot_of((int)blockIdx.x, tid0);
  int m0_prev = 0, mr_prev = 0;

  for (int grp = (int)blockIdx.x;; grp += (int)gridDim.x) {
    // (the thread index is taken anew in every trip, or the compiler computes every address that depends on it
    // once, in front of the loop, and keeps -- spills -- them all)
    const int tid = opaque_tid(), lane = tid & 63, g = lane >> 4;
    const bool have = grp < n_groups, have_prev = grp != (int)blockIdx.x;     // (uniform)
    const int m0 = grp * kRegs;
    const int mr = have ? ((n_out - m0) < kRegs ? (n_out - m0) : kRegs) : 0;
    int n_pass = 0, RT0 = 0;
    uint4 val[G];
#pragma unroll
    for (int k = 0; k < G; ++k) opaque_def(val[k]);
    qp.forget();
    op.forget();
    if (have_prev) op.prefetch();                  // ahead of this group's rows in the queue
    if (have) {
      // ---- slots: voxel and number of occupied slots before it (what the row loads below need to know)
      const unsigned long long occ = __ballot(v_slot >= 0);
      if (lane == 0) wcnt[wave] = __popcll(occ);
      lds_barrier();
      int before = 0, all = 0;
      for (int k = 0; k < NW; ++k) { const int w = wcnt[k]; all += w; if (k < wave) before += w; }
      if (tid < mr * P) { slot_vox[tid] = v_slot; slot_cum[tid] = (uint16_t)(before + __popcll(occ & ((1ull << lane) - 1ull))); }
      lds_barrier();
      for (int mm = tid; mm <= mr; mm += NTHREADS) {
        const int cum = mm < mr ? slot_cum[mm * P] : all;
        reg_cum[mm] = cum;
        if (mm == mr) pass_first[(slot_cum[(mr - 1) * P] / W) + 1] = mr;
        else if (mm == 0 || slot_cum[(mm - 1) * P] / W != cum / W) pass_first[cum / W] = mm;
      }
      lds_barrier();
      n_pass = reg_cum[mr - 1] / W + 1;
      // ---- rows of the first pass: requested now, stored once the tile is free
      const int mb0 = pass_first[1], rows0 = reg_cum[mb0];
      RT0 = (rows0 + 15) >> 4;
      for (int r = rows0 + tid; r < RT0 * 16; r += NTHREADS) row_vox[r] = -1;
      if (tid < mb0 * P && v_slot >= 0) row_vox[slot_cum[tid]] = v_slot;
      lds_barrier();
#pragma unroll
      for (int k = 0; k < G; ++k) {
        const int idx = tid + k * NTHREADS, r = idx / CH, c = idx - r * CH;
        const int v = idx < RT0 * 16 * CH ? row_vox[r] : -1;
        val[k] = make_uint4(0u, 0u, 0u, 0u);
        if (v >= 0) val[k] = reinterpret_cast<const uint4*>(x + (size_t)v * C)[c];
      }
    }
    if (have_prev) {
      // ---- the group before: out = LN(P + O Wo^T + bo), its rows to memory
      f32x4 bo4[NT_C], ga[NT_C], be[NT_C];
#pragma unroll
      for (int nt = 0; nt < NT_C; ++nt) bo4[nt] = *reinterpret_cast<const f32x4*>(p.b_o + o_own + 16 * nt + 4 * g);
      f32x4 keep[NT_C][RH];
      if (HC == 1) op.template run_keep<1>(Qs, LDX, rt_own, bo4, keep);
      else op.template run_keep<2>(Qs, LDX, rt_own, bo4, keep);
#pragma unroll
      for (int nt = 0; nt < NT_C; ++nt) {
        ga[nt] = *reinterpret_cast<const f32x4*>(p.ln_g + o_own + 16 * nt + 4 * g);
        be[nt] = *reinterpret_cast<const f32x4*>(p.ln_b + o_own + 16 * nt + 4 * g);
      }
#pragma unroll
      for (int nt = 0; nt < NT_C; ++nt)
#pragma unroll
        for (int r = 0; r < RH; ++r)
          if (r < HC) {
            const Vec4 xr = *reinterpret_cast<const Vec4*>(Ps + (16 * (rt_own + r) + (lane & 15)) * LDX + o_own + 16 * nt + 4 * g);
            keep[nt][r] += f32x4{to_f32<T>(xr[0]), to_f32<T>(xr[1]), to_f32<T>(xr[2]), to_f32<T>(xr[3])};
          }
      layer_norm_tile<T, NT_C, C, RH>(keep, o_own, og_own, rt_own, HC, stat, ga, be, p.ln_eps, Ps, LDX);
      lds_barrier();
      for (int idx = tid; idx < mr_prev * CH; idx += NTHREADS) {
        const int r = idx / CH, c = idx - r * CH;
        reinterpret_cast<uint4*>(out + (size_t)(m0_prev + r) * C)[c] =
            *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(Ps) + (size_t)r * LDX * sizeof(T) + c * 16);
      }
      lds_barrier();                               // (the pooled rows and the statistics are free from here)
    }
    if (!have) break;
    m0_prev = m0; mr_prev = mr;
    kv.prefetch();
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const int idx = tid + k * NTHREADS, r = idx / CH, c = idx - r * CH;
      if (idx < RT0 * 16 * CH)
        *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(Xs) + (size_t)r * LDX * sizeof(T) + c * 16) = val[k];
    }
    if (mr < kRegs)
      for (int idx = tid; idx < kRegs * CH; idx += NTHREADS)     // pooled rows past the last region are zero
        if (idx / CH >= mr)
          *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(Ps) + (size_t)(idx / CH) * LDX * sizeof(T) + (idx % CH) * 16) =
              make_uint4(0u, 0u, 0u, 0u);

    // ---- passes: K, V of the occupied slots, then Eq. (7) per (region, head): softmax over the region's slots;
    // O replaces the head's Q entries
    for (int ps = 0; ps < n_pass; ++ps) {
      const int ma = pass_first[ps], mb = pass_first[ps + 1];
      const int base = reg_cum[ma], rows = reg_cum[mb] - base;
      const int RT = (rows + 15) >> 4;
      if (ps > 0) {                                // (the first pass's rows are on their way into the tile already)
        for (int r = rows + tid; r < RT * 16; r += NTHREADS) row_vox[r] = -1;
        for (int sl = ma * P + tid; sl < mb * P; sl += NTHREADS) {
          const int v = slot_vox[sl];
          if (v >= 0) row_vox[slot_cum[sl] - base] = v;
        }
        lds_barrier();
        uint4 val2[G];                             // gather: every load requested before the first store
#pragma unroll
        for (int k = 0; k < G; ++k) {
          const int idx = tid + k * NTHREADS, r = idx / CH, c = idx - r * CH;
          const int v = idx < RT * 16 * CH ? row_vox[r] : -1;
          val2[k] = make_uint4(0u, 0u, 0u, 0u);
          if (v >= 0) val2[k] = reinterpret_cast<const uint4*>(x + (size_t)v * C)[c];
        }
        kv.prefetch();
#pragma unroll
        for (int k = 0; k < G; ++k) {
          const int idx = tid + k * NTHREADS, r = idx / CH, c = idx - r * CH;
          if (idx < RT * 16 * CH)
            *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(Xs) + (size_t)r * LDX * sizeof(T) + c * 16) = val2[k];
        }
      }
      lds_barrier();
      // Eq. (6): channel-wise max over a region's occupied slots, which are consecutive rows of the tile
      for (int idx = tid; idx < (mb - ma) * CH; idx += NTHREADS) {
        const int mm = ma + idx / CH, c = idx % CH;
        const int r0 = reg_cum[mm] - base, cnt = reg_cum[mm + 1] - reg_cum[mm];
        float best[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) best[e] = -INFINITY;
        for (int r = r0; r < r0 + cnt; ++r) {
          const uint4 raw = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(Xs) + (size_t)r * LDX * sizeof(T) + c * 16);
          const T* e4 = reinterpret_cast<const T*>(&raw);
#pragma unroll
          for (int e = 0; e < EPC; ++e) best[e] = fmaxf(best[e], to_f32<T>(e4[e]));
        }
        uint4 packed;
        T* o4 = reinterpret_cast<T*>(&packed);
#pragma unroll
        for (int e = 0; e < EPC; ++e) o4[e] = (T)best[e];
        *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(Ps) + (size_t)mm * LDX * sizeof(T) + c * 16) = packed;
      }
      kv.run(Xs, LDX, RT, p.b_kv, [&](int o0, int r, f32x4 (&acc)[NT_KV], bool) {
        const int row = 16 * r + (lane & 15);
#pragma unroll
        for (int nt = 0; nt < NT_KV; ++nt) {
          const int ot = o0 + 16 * nt, o = ot + 4 * g;
          if (ot < C) *reinterpret_cast<Vec4*>(Ks + row * LDX + o) = pack4<T>(acc[nt]);
          else *reinterpret_cast<Vec4*>(Vs + row * LDX + (o - C)) = pack4<T>(acc[nt]);
        }
      });
      qp.prefetch();
      lds_barrier();
      // Q of the pooled rows of this pass (the rows of earlier passes hold their results already)
      qp.run(Ps, LDX, kRegs / 16, p.b_q, [&](int o0, int r, f32x4 (&acc)[NT_C], bool) {
        const int row = 16 * r + (lane & 15);
        if (row >= ma && row < mb) {
#pragma unroll
          for (int nt = 0; nt < NT_C; ++nt) *reinterpret_cast<Vec4*>(Qs + row * LDX + o0 + 16 * nt + 4 * g) = pack4<T>(acc[nt]);
        }
      });
      if (ps == n_pass - 1) v_slot = grp + (int)gridDim.x < n_groups ? slot_of(grp + (int)gridDim.x, tid) : -1;   // used after the softmax
      lds_barrier();
      // Eq. (7) per (region, head): softmax over the region's slots; O replaces the head's Q entries.  The
      // occupied slots are rows r0 .. r0 + cnt - 1; the P - cnt empty ones all have the bias vectors as key and
      // value, so they enter as one key of that weight (or not at all when empty slots are masked).
      for (int it = tid; it < (mb - ma) * HEADS; it += NTHREADS) {
        const int mm = ma + it / HEADS, h = it % HEADS;
        const int r0 = reg_cum[mm] - base, cnt = reg_cum[mm + 1] - reg_cum[mm];
        const float holes = p.mask_empty ? 0.f : (float)(P - cnt);
        T* q = Qs + mm * LDX + h * D;
        float qv[D], o[D], logit[kMaxPool + 1];
        load_row<T, D>(qv, q);
        float mx = -INFINITY;
#pragma unroll
        for (int s = 0; s <= kMaxPool; ++s) {
          logit[s] = -INFINITY;
          const bool real = s < cnt, hole = s == kMaxPool && holes > 0.f;
          if (real || hole) {
            float kvv[D];
            load_row<T, D>(kvv, real ? Ks + (r0 + s) * LDX + h * D : Kb + h * D);
            float acc = 0.f;
#pragma unroll
            for (int j = 0; j < D; ++j) acc = fmaf(qv[j], kvv[j], acc);
            logit[s] = acc * scale;
            mx = fmaxf(mx, logit[s]);
          }
        }
#pragma unroll
        for (int j = 0; j < D; ++j) o[j] = 0.f;
        float sum = 0.f;
#pragma unroll
        for (int s = 0; s <= kMaxPool; ++s) {
          const bool real = s < cnt, hole = s == kMaxPool && holes > 0.f;
          if (real || hole) {
            const float e = __expf(logit[s] - mx) * (hole ? holes : 1.f);
            sum += e;
            float kvv[D];
            load_row<T, D>(kvv, real ? Vs + (r0 + s) * LDX + h * D : Vb + h * D);
#pragma unroll
            for (int j = 0; j < D; ++j) o[j] = fmaf(e, kvv[j], o[j]);
          }
        }
        const float inv = 1.0f / sum;
#pragma unroll
        for (int j = 0; j < D; ++j) q[j] = (T)(o[j] * inv);
      }
      lds_barrier();
    }
  }
}

// ------------------------------------------------------------------------------------------
struct PoolPlan {
  PoolGeom g;
  int64_t n_words;
  size_t off_bitmap, off_prefix, off_inds, total;
};

bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

int make_plan(const dsvt_pool_cfg* cfg, int32_t n_voxels, PoolPlan* pl) {
  if (!cfg || n_voxels <= 0 || cfg->batch <= 0) return DSVT_EINVAL;
  PoolGeom& g = pl->g;
  int64_t cells = cfg->batch, P = 1;
  for (int a = 0; a < 3; ++a) {
    if (cfg->grid[a] <= 0 || cfg->pool[a] <= 0) return DSVT_EINVAL;
    g.grid[a] = cfg->grid[a]; g.pool[a] = cfg->pool[a];
    g.pg[a] = (int32_t)dsvt_ceil_div(cfg->grid[a], cfg->pool[a]);
    cells *= g.pg[a]; P *= cfg->pool[a];
    if (cells >= (1ll << 31) || P > kMaxPool) return cells >= (1ll << 31) ? DSVT_EINVAL : DSVT_EUNSUPPORTED;
  }
  g.batch = cfg->batch; g.P = (int32_t)P;
  pl->n_words = dsvt_ceil_div(cells, 32);
  size_t o = 0;
  pl->off_bitmap = o; o = dsvt_align_up(o + (size_t)pl->n_words * 4, 256);
  pl->off_prefix = o; o = dsvt_align_up(o + (size_t)pl->n_words * 4, 256);
  pl->off_inds = o;   o = dsvt_align_up(o + (size_t)n_voxels * P * 4, 256);
  pl->total = o;
  return DSVT_OK;
}

int check_pool(const dsvt_pool_cfg& c, bool need_packed) {
  if (!c.w_q || !c.w_k || !c.w_v || !c.w_o || !c.b_q || !c.b_k || !c.b_v || !c.b_o || !c.ln_g || !c.ln_b) return DSVT_EINVAL;
  if (c.dtype != DSVT_F32 && c.dtype != DSVT_BF16) return DSVT_EINVAL;
  if (c.mask_empty != 0 && c.mask_empty != 1) return DSVT_EINVAL;
  if (!((c.C == 64 && c.heads == 4) || (c.C == 128 && c.heads == 8) || (c.C == 192 && c.heads == 8))) return DSVT_EUNSUPPORTED;
  if (c.dtype == DSVT_F32 && c.C != 64) return DSVT_EUNSUPPORTED;
  if (need_packed && (!c.packed || !aligned16(c.packed))) return DSVT_EINVAL;
  const void* ptrs[] = {c.w_q, c.w_k, c.w_v, c.w_o, c.b_q, c.b_k, c.b_v, c.b_o, c.ln_g, c.ln_b};
  for (const void* q : ptrs) if (!aligned16(q)) return DSVT_EINVAL;
  return DSVT_OK;
}

// packed buffer: [w_k; w_v] as one [2C, C] matrix, w_q, w_o (fragment order), then b_k|b_v as floats
struct PoolPacked { size_t off_kv, off_q, off_o, off_bkv, total; };
PoolPacked pool_packed(const dsvt_pool_cfg& c) {
  const size_t es = c.dtype == DSVT_BF16 ? 2 : 4, cc = (size_t)c.C * c.C * es;
  PoolPacked pp;
  size_t o = 0;
  pp.off_kv = o; o = dsvt_align_up(o + 2 * cc, 256);
  pp.off_q = o;  o = dsvt_align_up(o + cc, 256);
  pp.off_o = o;  o = dsvt_align_up(o + cc, 256);
  pp.off_bkv = o; o = dsvt_align_up(o + (size_t)2 * c.C * 4, 256);
  pp.total = o;
  return pp;
}

__global__ void kp_copy_f32(const float* __restrict__ src, float* __restrict__ dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

template <typename T> void pack_matrix(const void* src, void* dst, int out, int k, hipStream_t st) {
  const long long slots = (long long)(out / 16) * (k / Mma<T>::KC) * 64;
  k_pack<T><<<(unsigned)dsvt_ceil_div(slots, 256), 256, 0, st>>>(reinterpret_cast<const T*>(src), reinterpret_cast<T*>(dst), out, k);
}

template <typename T, int C, int HEADS, int NT_KV, int NT_C>
int launch_pool_attention(const dsvt_pool_cfg& c, const PoolPlan& pl, const int32_t* pool_inds, const int32_t* n_out,
                          const void* x, void* out, int32_t n_voxels, hipStream_t st) {
  auto kern = kp_attention<T, C, HEADS, NT_KV, NT_C>;
  constexpr size_t lds = PoolLds<T, C>::total;
  static std::atomic<uint64_t> lds_allowed{0};
  if (int rc = dsvt_allow_lds(reinterpret_cast<const void*>(kern), lds, lds_allowed)) return rc;
  const PoolPacked pp = pool_packed(c);
  const char* pk = reinterpret_cast<const char*>(c.packed);
  PoolDev d;
  d.w_kv = pk + pp.off_kv; d.w_q = pk + pp.off_q; d.w_o = pk + pp.off_o;
  d.b_kv = reinterpret_cast<const float*>(pk + pp.off_bkv);
  d.b_q = c.b_q; d.b_o = c.b_o; d.ln_g = c.ln_g; d.ln_b = c.ln_b; d.ln_eps = c.ln_eps;
  d.P = pl.g.P; d.mask_empty = c.mask_empty;
  dsvt_prof_scope ps(DSVT_K_POOL_ATTN, st);
  // one workgroup per compute unit (the LDS tile fills it), each walking over every grid-th group of regions
  const int64_t groups = dsvt_ceil_div(n_voxels, kRegs);
  kern<<<(unsigned)(groups < kPoolGrid ? groups : kPoolGrid), kWaves * 64, lds, st>>>(d, pool_inds, n_out, reinterpret_cast<const T*>(x),
                                                                                    reinterpret_cast<T*>(out));
  return DSVT_OK;
}

}  // namespace


extern "C" int dsvt_pool_packed_size(const dsvt_pool_cfg* cfg, size_t* bytes) {
  if (!cfg || !bytes) return DSVT_EINVAL;
  int rc = check_pool(*cfg, false);
  if (rc != DSVT_OK) return rc;
  *bytes = pool_packed(*cfg).total;
  return DSVT_OK;
}

extern "C" int dsvt_pool_pack(const dsvt_pool_cfg* cfg, void* packed, size_t bytes, void* stream) {
  if (!cfg || !packed || !aligned16(packed)) return DSVT_EINVAL;
  int rc = check_pool(*cfg, false);
  if (rc != DSVT_OK) return rc;
  const PoolPacked pp = pool_packed(*cfg);
  if (bytes < pp.total) return DSVT_ENOSPC;
  hipStream_t st = (hipStream_t)stream;
  char* pk = reinterpret_cast<char*>(packed);
  const int C = cfg->C;
  const size_t es = cfg->dtype == DSVT_BF16 ? 2 : 4;
  const void* srcs[4] = {cfg->w_k, cfg->w_v, cfg->w_q, cfg->w_o};
  char* dsts[4] = {pk + pp.off_kv, pk + pp.off_kv + (size_t)C * C * es, pk + pp.off_q, pk + pp.off_o};
  for (int i = 0; i < 4; ++i) {
    // [w_k; w_v] is the row-wise concatenation, so its fragment order is w_k's followed by w_v's
    if (cfg->dtype == DSVT_BF16) pack_matrix<bf16_t>(srcs[i], dsts[i], C, C, st);
    else pack_matrix<float>(srcs[i], dsts[i], C, C, st);
  }
  float* bkv = reinterpret_cast<float*>(pk + pp.off_bkv);
  kp_copy_f32<<<(unsigned)dsvt_ceil_div(C, 256), 256, 0, st>>>(cfg->b_k, bkv, C);
  kp_copy_f32<<<(unsigned)dsvt_ceil_div(C, 256), 256, 0, st>>>(cfg->b_v, bkv + C, C);
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}

extern "C" int dsvt_attn_pool_workspace_size(const dsvt_pool_cfg* cfg, int32_t n_voxels, size_t* bytes) {
  if (!bytes) return DSVT_EINVAL;
  PoolPlan pl;
  int rc = make_plan(cfg, n_voxels, &pl);
  if (rc != DSVT_OK) return rc;
  *bytes = pl.total;
  return DSVT_OK;
}

namespace {

// The whole call on scratch memory `ws` of at least pl.total bytes (checked by the callers).
int run_attn_pool(const dsvt_pool_cfg* cfg, const PoolPlan& pl, const int32_t* coords, const void* x, int32_t n_voxels,
                  int32_t* out_coords, void* out, int32_t* n_out, void* ws, int32_t* status, hipStream_t st) {
  char* base = reinterpret_cast<char*>(ws);
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(base + pl.off_bitmap);
  int32_t* prefix = reinterpret_cast<int32_t*>(base + pl.off_prefix);
  int32_t* inds = reinterpret_cast<int32_t*>(base + pl.off_inds);
  const int tb = 256;
  {
    dsvt_prof_scope ps(DSVT_K_POOL_GROUP, st);
    const int64_t n_inds = (int64_t)n_voxels * pl.g.P;
    const int64_t n_clear = pl.n_words > n_inds ? pl.n_words : n_inds;
    kp_clear<<<(unsigned)dsvt_ceil_div(n_clear, tb), tb, 0, st>>>(bitmap, pl.n_words, inds, n_inds);
    kp_mark<<<(unsigned)dsvt_ceil_div(n_voxels, tb), tb, 0, st>>>(pl.g, reinterpret_cast<const int4*>(coords), n_voxels,
                                                                  bitmap, status);
    k_block_scan<true><<<block_scan_grid(pl.n_words), 1024, 0, st>>>(bitmap, prefix, pl.n_words, nullptr, n_out);
    kp_emit<<<(unsigned)dsvt_ceil_div(n_voxels, tb), tb, 0, st>>>(pl.g, reinterpret_cast<const int4*>(coords), n_voxels,
                                                                  bitmap, prefix, inds, out_coords);
  }
  int rc;
  if (cfg->dtype == DSVT_BF16) {
    if (cfg->C == 192) rc = launch_pool_attention<bf16_t, 192, 8, 3, 3>(*cfg, pl, inds, n_out, x, out, n_voxels, st);
    else if (cfg->C == 128) rc = launch_pool_attention<bf16_t, 128, 8, 2, 2>(*cfg, pl, inds, n_out, x, out, n_voxels, st);
    else rc = launch_pool_attention<bf16_t, 64, 4, 1, 1>(*cfg, pl, inds, n_out, x, out, n_voxels, st);
  } else {
    rc = launch_pool_attention<float, 64, 4, 1, 1>(*cfg, pl, inds, n_out, x, out, n_voxels, st);
  }
  if (rc != DSVT_OK) return rc;
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}

int check_pool_call(const dsvt_pool_cfg* cfg, const int32_t* coords, const void* x, int32_t n_voxels, int32_t* out_coords,
                    void* out, int32_t* n_out, int32_t* status, PoolPlan* pl) {
  int rc = make_plan(cfg, n_voxels, pl);
  if (rc != DSVT_OK) return rc;
  rc = check_pool(*cfg, true);
  if (rc != DSVT_OK) return rc;
  if (!coords || !x || !out_coords || !out || !n_out || !status || x == out) return DSVT_EINVAL;
  if (!aligned16(coords) || !aligned16(x) || !aligned16(out) || !aligned16(out_coords)) return DSVT_EINVAL;
  return DSVT_OK;
}

// Scratch of dsvt_attn_pool_static: one array per GPU, part of the loaded code object (never allocated, never
// freed).  In host code `scratch` is only a handle for hipGetSymbolAddress; the kernels get the device address
// that call returns, looked up once per device and kept in g_scratch.
constexpr size_t kStaticScratchBytes = DSVT_POOL_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch[kMaxDevices];

int static_scratch(void** ptr) {
  int dev = 0;
  DSVT_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return DSVT_EUNSUPPORTED;
  void* p = g_scratch[dev].load(std::memory_order_acquire);
  if (p == nullptr) {                                          // first call on this device (it is the current one)
    DSVT_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return DSVT_EHIP;
    g_scratch[dev].store(p, std::memory_order_release);        // (two threads racing here store the same address)
  }
  *ptr = p;
  return DSVT_OK;
}

}  // namespace

extern "C" int dsvt_attn_pool(const dsvt_pool_cfg* cfg, const int32_t* coords, const void* x, int32_t n_voxels,
                              int32_t* out_coords, void* out, int32_t* n_out, void* ws, size_t ws_bytes,
                              int32_t* status, void* stream) {
  PoolPlan pl;
  int rc = check_pool_call(cfg, coords, x, n_voxels, out_coords, out, n_out, status, &pl);
  if (rc != DSVT_OK) return rc;
  if (!ws) return DSVT_EINVAL;
  if (ws_bytes < pl.total) return DSVT_ENOSPC;
  return run_attn_pool(cfg, pl, coords, x, n_voxels, out_coords, out, n_out, ws, status, (hipStream_t)stream);
}

extern "C" int dsvt_attn_pool_static(const dsvt_pool_cfg* cfg, const int32_t* coords, const void* x, int32_t n_voxels,
                                     int32_t* out_coords, void* out, int32_t* n_out, int32_t* status, void* stream) {
  PoolPlan pl;
  int rc = check_pool_call(cfg, coords, x, n_voxels, out_coords, out, n_out, status, &pl);
  if (rc != DSVT_OK) return rc;
  if (pl.total > kStaticScratchBytes) return DSVT_ENOSPC;      // grid or voxel count beyond the built-in scratch
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != DSVT_OK) return rc;
  return run_attn_pool(cfg, pl, coords, x, n_voxels, out_coords, out, n_out, ws, status, (hipStream_t)stream);
}
