// dsvt_set_attention / dsvt_block: one DSVT layer per kernel launch on gfx950 (Sec. 3.2 Eq. 4-5;
// appendix "Network Architecture").
//
// k_layer: a workgroup owns a run of consecutive sets (a "tile" of at most 96 rows).  It takes the
// sets' distinct voxels -- from the tile descriptor the partition wrote, or, without a work list, by
// keeping the first occurrence of every voxel in the sets' slot rows (repeats are adjacent, Eq. 3 is
// monotone) -- and gathers those voxels' features into an LDS tile: the tau x C tiles of Eq. (4)
// with the repeated rows squeezed out, since a masked repeat contributes nothing as a key and its
// query row would be thrown away.  Q/K/V projection, per-(set, head) softmax(QK^T + PE)V,
// output projection, residual + LayerNorm, the MLP and the second residual + LayerNorm all run
// on that tile in LDS and registers; the rows then go straight back to the voxels' rows of the
// output (every voxel is in exactly one set, Thm A.2-A.3), so a layer reads and writes [N, C] once.
#include "common.h"
#include "mma.h"
#include "phase_clock.h"

namespace {

constexpr int kTauMax = 96;                     // a set's distinct voxels must fit one tile
constexpr int kMaxSets = kRowsMax / 4;           // every set takes at least 4 rows of a tile
constexpr int kRowsPad = kRowsMax + 16;          // per-row arrays are read 4 at a time up to 15 rows past a set's end
constexpr int kMaxItems = 128;                  // attention items: (set, query tile, group of heads); see item_groups()
// Sets per workgroup when no tile list is given.
__host__ __device__ constexpr int fixed_sets(int tau) { return tau <= kRowsMax / 2 ? 2 : 1; }
// A set of up to 3 key tiles (48 voxels) is split into items of half of the heads each; a larger one
// (its logits take more registers) into one item per head.  At most one set of a tile is that large,
// so a tile has at most 8 * 6 + 2 * (3 + 11) = 76 items.
__host__ __device__ constexpr int item_groups(int kts, int heads) { return kts <= 3 ? 2 : heads; }
constexpr int kHalfTiles = kRowTiles / 2;        // the LayerNorm-phase work items cover half of the row tiles
constexpr int kLayerWaves = 12;                  // three per SIMD: one workgroup per CU (LDS), the other wavefronts hide one's waits

// erf-GELU (appendix "Network Architecture": the MLP of a DSVT layer) for bf16 features by linear
// interpolation: kGeluKnots intervals of width 1 / kGeluScale over [-4, 4), each with the slope
// and intercept of the chord through the exact values at its ends; below -4 the result is 0, from
// 4 on it is x (both within 1.4e-4 of the exact function; the chords are within 3.5e-5).  The
// table (4 KB) sits in LDS during the MLP: a lookup and one fma replace a dozen ALU instructions.
constexpr int kGeluKnots = 512;
constexpr float kGeluScale = 64.f;
__global__ void k_pack_gelu_table(float2* __restrict__ tab) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= kGeluKnots) return;
  const double x0 = (i - kGeluKnots / 2) / (double)kGeluScale, x1 = x0 + 1.0 / kGeluScale;
  const double g0 = 0.5 * x0 * (1.0 + erf(x0 * 0.70710678118654752440)), g1 = 0.5 * x1 * (1.0 + erf(x1 * 0.70710678118654752440));
  const double sl = (g1 - g0) * kGeluScale;
  float2 e = make_float2((float)sl, (float)(g0 - sl * x0));
  if (i == 0) e = make_float2(0.f, 0.f);                      // x < -4 + 1/64 (and everything below)
  if (i == kGeluKnots - 1) e = make_float2(1.f, 0.f);         // x >= 4 - 1/64 (and everything above)
  tab[i] = e;
}
__device__ __forceinline__ float gelu_from_table(const float2* tab, float x) {
  const float t = __builtin_amdgcn_fmed3f(fmaf(x, kGeluScale, 0.5f * kGeluKnots), 0.f, (float)(kGeluKnots - 1));
  const float2 e = tab[(int)t];
  return fmaf(e.x, x, e.y);
}

struct LayerDev {
  const void *w_qkv, *w_o, *w_1, *w_2;       // packed (see mma.h)
  const float *b_qkv, *b_o, *b_1, *b_2, *ln1_g, *ln1_b, *ln2_g, *ln2_b, *rel_bias;
  const float2* gelu_tab;                    // kGeluKnots (slope, intercept) pairs, see k_pack_gelu_table
  float ln_eps;
  int rel_size, rel_const, rel_my, rel_mz;   // table entries per head; index = lin(q) - lin(k) + rel_const
  int dup_mode;
};


struct MapsDev {
  const int32_t *set_inds, *n_sets, *n_tiles, *tile_desc;
  int32_t max_sets, tau, n_voxels;
};

template <typename T, int C, int HEADS, int HID> struct LayerLds {
  static constexpr int D = C / HEADS;
  static constexpr int PAD = lds_pad<T>();
  static constexpr int LDX = C + PAD;            // pitch of [row][feature] tiles, elements of T
  static constexpr int LDV = kRowsMax + 16 / (int)sizeof(T);   // pitch of V^T [feature][row]
  static constexpr int LDH = HID + PAD;          // pitch of the MLP hidden tile
  static constexpr size_t kTile = (size_t)kRowsMax * LDX * sizeof(T);
  static constexpr size_t off_x = 0, off_q = kTile, off_k = 2 * kTile, off_v = 3 * kTile;
  static constexpr size_t kVt = (size_t)C * LDV * sizeof(T);
  static constexpr size_t off_h = off_q;         // hidden tile reuses Q and K once attention is done
  static constexpr size_t off_misc = off_v + kVt;
  static constexpr size_t kMisc = (size_t)(3 * kRowsPad + 2 * kMaxSets + 2 + kMaxItems + 1) * 4;
  // after attention the V^T region holds the GELU table and the LayerNorm statistics
  static constexpr size_t off_gelu = off_v, off_stat = off_v + 4096, kStat = (size_t)2 * kStatGroupsMax * kRowsMax * 4;
  static_assert(off_stat + kStat <= off_misc, "GELU table and LayerNorm statistics must fit in the V^T region");
  static constexpr size_t total = off_misc + kMisc;
  static_assert((size_t)kRowsMax * LDH * sizeof(T) <= 2 * kTile, "hidden tile must fit in Q + K");
  static_assert(C % 64 == 0 && D % Mma<T>::KL == 0 && D % 4 == 0, "shape");
  static_assert(total <= 160 * 1024, "LDS of one CU");
};

// Attention of one (set, query tile, group of heads) item (Eq. 5): for each of its heads,
// logits = Q K^T (+ PE), softmax over the set's distinct voxels, O = P V; O overwrites the Q
// entries it was computed from.  KTC = key tiles of the set (compile time: no branches inside).
// S^T is produced key-major (keys as MFMA rows) so that a lane holds 4 keys of ONE query: the
// softmax reductions are in-lane plus two cross-lane steps, and P^T is already laid out as the B
// operand of O^T = V^T P^T.  Q arrives scaled by log2(e) / sqrt(d) (the projection's epilogue does
// it), and the positional term -- which depends on (query, key) only through the coordinate
// difference, one table row [index][heads] per pair, fetched once for all heads -- is the MFMA's
// initial accumulator value, so the logits come out of the matrix cores finished.  The keys past
// the set's last voxel take the table's extra last row, which holds -inf: no mask arithmetic.
// DUP: repeated slots count as keys (the exponentials are multiplied by the slots' counts).
template <typename T, int C, int HEADS, int HID, int KTC, int HG, bool DUP>
__device__ __forceinline__ void attn_item(const LayerDev& p, T* Qs, const T* Ks, const T* Vt, const int32_t* row_lin,
                                          const float* row_mult, int r0, int nu, int qt, int hh, int rows_ready) {
  typedef LayerLds<T, C, HEADS, HID> L;
  typedef Mma<T> M;
  typedef typename M::Frag Frag;
  typedef typename M::Vec4 Vec4;
  constexpr int D = L::D, LDX = L::LDX, LDV = L::LDV, KC = M::KC, KL = M::KL;
  constexpr int TPC = KC / 16;                    // key tiles per PV fragment: 2 (bf16) or 1 (fp32)
  constexpr int NCH = (KTC + TPC - 1) / TPC;
  static_assert(HG == 1 || HG == 2 || HG == 4, "heads per item");
  const int lane = opaque_tid() & 63, m = lane & 15, g = lane >> 4;
  const int qi = 16 * qt + m;
  const int qrow = r0 + (qi < nu ? qi : nu - 1);

  f32x4 bias[HG][KTC];
  f32x4 mult[KTC];
  {
    const int ql = row_lin[qrow] + p.rel_const;
#pragma unroll
    for (int kt = 0; kt < KTC; ++kt) {
      const int4 kl = *reinterpret_cast<const int4*>(row_lin + r0 + 16 * kt + 4 * g);
      const int kls[4] = {kl.x, kl.y, kl.z, kl.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int idx = ql - kls[i];
        idx = idx < 0 ? 0 : (idx >= p.rel_size ? p.rel_size - 1 : idx);
        if (kt == KTC - 1) idx = 16 * kt + 4 * g + i < nu ? idx : p.rel_size;   // only the last key tile is ragged
        const float* tp = reinterpret_cast<const float*>(reinterpret_cast<const char*>(p.rel_bias) +
                                                         (unsigned)idx * (unsigned)(HEADS * 4) + (unsigned)(hh * HG * 4));
        if constexpr (HG == 4) {
          const f32x4 t = *reinterpret_cast<const f32x4*>(tp);
          bias[0][kt][i] = t[0]; bias[1][kt][i] = t[1]; bias[2][kt][i] = t[2]; bias[3][kt][i] = t[3];
        } else if constexpr (HG == 2) {
          const float2 t = *reinterpret_cast<const float2*>(tp);
          bias[0][kt][i] = t.x; bias[1][kt][i] = t.y;
        } else {
          bias[0][kt][i] = *tp;
        }
      }
    }
  }
  if constexpr (DUP) {
#pragma unroll
    for (int kt = 0; kt < KTC; ++kt) mult[kt] = *reinterpret_cast<const f32x4*>(row_mult + r0 + 16 * kt + 4 * g);
  }

#pragma unroll
  for (int hl = 0; hl < HG; ++hl) {
    const int h = hh * HG + hl;
    f32x4 S[KTC];                                 // S[kt][i]: key 16*kt + 4*g + i, query 16*qt + m
#pragma unroll
    for (int kt = 0; kt < KTC; ++kt) S[kt] = bias[hl][kt];
#pragma unroll
    for (int kc = 0; kc < D; kc += KC) {
      const int kk = kc + g * KL;
      const bool live = kk < D;                   // lanes past the head width feed zeros
      const int kkc = live ? kk : 0;
      Frag fb = *reinterpret_cast<const Frag*>(Qs + qrow * LDX + h * D + kkc);
      fb = live ? fb : M::zero();
#pragma unroll
      for (int kt = 0; kt < KTC; ++kt) {
        const int ki = 16 * kt + m;
        const Frag fa = *reinterpret_cast<const Frag*>(Ks + (r0 + (ki < nu ? ki : nu - 1)) * LDX + h * D + kkc);
        S[kt] = M::mma(fa, fb, S[kt]);                  // dead k lanes: finite K times the zeroed Q
      }
    }
    // S holds the logits in units of log2(e), -inf for the keys that do not exist: exp is a bare exp2
    float mx = S[0][0];
#pragma unroll
    for (int kt = 0; kt < KTC; ++kt)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (kt + i > 0) mx = fmaxf(mx, S[kt][i]);
    mx = col_max(mx);                             // (key 0 exists for every query: finite)
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < KTC; ++kt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float e = __builtin_amdgcn_exp2f(S[kt][i] - mx);       // exp2(-inf) = 0
        if constexpr (DUP) e *= mult[kt][i];
        S[kt][i] = e;
        sum += e;
      }
    sum = col_sum(sum);
    const float inv = __builtin_amdgcn_rcpf(sum);

    // O^T[dv][q] = sum_key V^T[dv][key] P^T[key][q].  Key columns past the tile's rows hold no V: their P is an
    // exact zero, so any finite column will do, and the set's first one is read instead.
#pragma unroll
    for (int dt = 0; dt < (D + 15) / 16; ++dt) {
      f32x4 O = f32x4{0.f, 0.f, 0.f, 0.f};
      const int dv = 16 * dt + m;
      const T* vrow = Vt + (h * D + (dv < D ? dv : 0)) * LDV;      // (rows past the head width: results thrown away)
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        Frag fa, fb;
        if constexpr (TPC == 2) {
          const int c0 = r0 + 32 * c + 4 * g, c1 = c0 + 16;
          const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vrow + (c0 < rows_ready ? c0 : r0));
          const f32x4 p0 = S[2 * c];
          if (2 * c + 1 < KTC) {
            const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vrow + (c1 < rows_ready ? c1 : r0));
            const f32x4 p1 = S[2 * c + 1 < KTC ? 2 * c + 1 : 0];
            fa = Frag{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            fb = Frag{(bf16_t)p0[0], (bf16_t)p0[1], (bf16_t)p0[2], (bf16_t)p0[3],
                      (bf16_t)p1[0], (bf16_t)p1[1], (bf16_t)p1[2], (bf16_t)p1[3]};
          } else {
            fa = Frag{lo[0], lo[1], lo[2], lo[3], 0, 0, 0, 0};
            fb = Frag{(bf16_t)p0[0], (bf16_t)p0[1], (bf16_t)p0[2], (bf16_t)p0[3], 0, 0, 0, 0};
          }
        } else {
          const int c0 = r0 + 16 * c + 4 * g;
          fa = *reinterpret_cast<const Frag*>(vrow + (c0 < rows_ready ? c0 : r0));
          fb = S[c];
        }
        O = M::mma(fa, fb, O);
      }
      if (qi < nu && 16 * dt + 4 * g < D)
        *reinterpret_cast<Vec4*>(Qs + (r0 + qi) * LDX + h * D + 16 * dt + 4 * g) = pack4<T>(O * inv);
    }
  }
}

// An item of a set with kts key tiles: up to three key tiles half of the heads per item, beyond that (BIG kernels
// only) one head.
template <typename T, int C, int HEADS, int HID, bool BIG, bool DUP>
__device__ __forceinline__ void attn_any(const LayerDev& p, T* Qs, const T* Ks, const T* Vt, const int32_t* row_lin,
                                         const float* row_mult, int r0, int nu, int qt, int hh, int kts, int rows_ready) {
  constexpr int HG2 = HEADS / 2;
  if (kts == 1) attn_item<T, C, HEADS, HID, 1, HG2, DUP>(p, Qs, Ks, Vt, row_lin, row_mult, r0, nu, qt, hh, rows_ready);
  else if (kts == 2) attn_item<T, C, HEADS, HID, 2, HG2, DUP>(p, Qs, Ks, Vt, row_lin, row_mult, r0, nu, qt, hh, rows_ready);
  else if (!BIG || kts == 3) attn_item<T, C, HEADS, HID, 3, HG2, DUP>(p, Qs, Ks, Vt, row_lin, row_mult, r0, nu, qt, hh, rows_ready);
  else if constexpr (BIG) {
    if (kts == 4) attn_item<T, C, HEADS, HID, 4, 1, DUP>(p, Qs, Ks, Vt, row_lin, row_mult, r0, nu, qt, hh, rows_ready);
    else if (kts == 5) attn_item<T, C, HEADS, HID, 5, 1, DUP>(p, Qs, Ks, Vt, row_lin, row_mult, r0, nu, qt, hh, rows_ready);
    else attn_item<T, C, HEADS, HID, 6, 1, DUP>(p, Qs, Ks, Vt, row_lin, row_mult, r0, nu, qt, hh, rows_ready);
  }
}

// BIG: the instantiation for tau > 48 (sets of four to six key tiles); the common one does not carry that code.
template <typename T, int C, int HEADS, int HID, int NT_QKV, int NT_O, int NT_1, int NT_2, bool BIG, bool DUP>
__global__ void __launch_bounds__(kLayerWaves * 64)
k_layer(LayerDev p, MapsDev mp, const int4* __restrict__ coords, const T* x, T* out, int full_layer) {
  // out may be x: a tile's rows are read, then written, by this workgroup only
  typedef LayerLds<T, C, HEADS, HID> L;
  typedef typename Mma<T>::Vec4 Vec4;
  constexpr int LDX = L::LDX, LDV = L::LDV, LDH = L::LDH;
  constexpr int NW = kLayerWaves, NTHREADS = NW * 64;
  constexpr int SG = C / (16 * NT_O);              // LayerNorm phases: SG feature groups x 2 halves of the row tiles, one item per wavefront
  static_assert(NT_O == NT_2 && SG * 16 * NT_O == C && 2 * SG <= NW && SG <= kStatGroupsMax, "LayerNorm phases: one item per wavefront");
  extern __shared__ __align__(16) unsigned char smem[];
  T* Xs = reinterpret_cast<T*>(smem + L::off_x);
  T* Qs = reinterpret_cast<T*>(smem + L::off_q);
  T* Ks = reinterpret_cast<T*>(smem + L::off_k);
  T* Vt = reinterpret_cast<T*>(smem + L::off_v);
  T* Hs = reinterpret_cast<T*>(smem + L::off_h);
  int32_t* row_vox = reinterpret_cast<int32_t*>(smem + L::off_misc);
  int32_t* row_lin = row_vox + kRowsPad;
  float* row_mult = reinterpret_cast<float*>(row_lin + kRowsPad);
  int32_t* set_r0 = reinterpret_cast<int32_t*>(row_mult + kRowsPad);   // [kMaxSets + 1]
  int32_t* set_nu = set_r0 + kMaxSets + 1;                              // [kMaxSets + 1]
  float* stat = reinterpret_cast<float*>(smem + L::off_stat);           // [2][kStatGroupsMax][kRowsMax], over V^T once attention is done
  int32_t* items = set_nu + kMaxSets + 1;                               // [kMaxItems + 1]

  // wave-uniform values are read back through readfirstlane so that the compiler keeps them in
  // scalar registers: branches on them are scalar branches, not exec-mask divergence
  int tid = threadIdx.x, lane = tid & 63, m = lane & 15, g = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#define DSVT_REFRESH_LANE() do { tid = opaque_tid(); lane = tid & 63; m = lane & 15; g = lane >> 4; } while (0)
  GemmPhase<T, NT_QKV, C, 3 * C, NW, 1, false> qkv(reinterpret_cast<const T*>(p.w_qkv), wave);

  DSVT_PHASE(0);
  int ns;
  if (mp.tile_desc != nullptr) {
    // ---- 1a. rows from the tile descriptor the partition wrote for this workgroup (1 KB, one load)
    const int n_tiles = *mp.n_tiles;
    const int word = tid < 256 ? mp.tile_desc[(size_t)blockIdx.x * 256 + tid] : 0;
    if ((int)blockIdx.x >= n_tiles) return;
    for (int r = kRowsMax + tid; r < kRowsPad; r += NTHREADS) { row_vox[r] = -1; row_lin[r] = 0; row_mult[r] = 0.f; }
    if (wave == 0) {
      int hdr_ns = __shfl(word, 1, 64), hdr_rows = __shfl(word, 0, 64);
      hdr_ns = hdr_ns < 0 ? 0 : (hdr_ns > kMaxSets ? kMaxSets : hdr_ns);
      hdr_rows = hdr_rows < 0 ? 0 : (hdr_rows > kRowsMax ? kRowsMax : hdr_rows);
      if (lane == 0) { set_nu[kMaxSets] = hdr_ns; set_r0[hdr_ns] = hdr_rows; }
      if (lane >= 2 && lane < 2 + kMaxSets && lane - 2 < hdr_ns) set_r0[lane - 2] = word < 0 ? 0 : (word > kRowsMax - 4 ? kRowsMax - 4 : word);
      constexpr int kNuMax = BIG ? kTauMax : 48;
      const int nu_s = word < 1 ? 1 : (word > kNuMax ? kNuMax : word);
      const int ls = lane - 2 - kMaxSets;        // the lanes holding the sets' sizes also list the sets' attention items
      if (ls >= 0 && ls < kMaxSets) set_nu[ls] = nu_s;
      const int kts = (ls >= 0 && ls < hdr_ns) ? (nu_s + 15) >> 4 : 0;
      const int ngr = item_groups(kts, HEADS);
      int incl = ngr * kts;                      // items: (set, query tile, group of heads)
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(incl, o, 64); if (lane >= o) incl += t; }
      int n = incl - ngr * kts;
      for (int qt = 0; qt < kts; ++qt)
        for (int hh = 0; hh < ngr; ++hh)
          if (n < kMaxItems) items[n++] = ls | (qt << 8) | (hh << 12) | (kts << 16);
      if (lane == 63) items[kMaxItems] = incl < kMaxItems ? incl : kMaxItems;   // published by the barrier below
    } else if (tid < 64 + 2 * kRowsMax) {           // words 64 + 2 r and 65 + 2 r: voxel and (slots << 24 | position code) of row r
      const int r = (tid - 64) >> 1;
      if ((tid & 1) == 0) {
        row_vox[r] = (word >= 0 && word < mp.n_voxels) ? word : -1;
      } else {
        row_lin[r] = word & 0xFFFFFF;
        row_mult[r] = (float)((unsigned)word >> 24);
      }
    }
    lds_barrier();
    ns = __builtin_amdgcn_readfirstlane(set_nu[kMaxSets]);
    if (ns <= 0) return;
  } else {
    // ---- 1b. no work list: two sets per workgroup, rows derived from set_inds and coords
    int n_sets = *mp.n_sets;
    n_sets = n_sets < mp.max_sets ? n_sets : mp.max_sets;
    const int per_wg = fixed_sets(mp.tau);
    const int s_begin = blockIdx.x * per_wg;
    ns = __builtin_amdgcn_readfirstlane((n_sets - s_begin) < per_wg ? (n_sets - s_begin) : per_wg);
    if (ns <= 0) return;
    const int tau = mp.tau;
    for (int r = tid; r < kRowsPad; r += NTHREADS) { row_vox[r] = -1; row_lin[r] = 0; row_mult[r] = 0.f; }
    for (int ls = wave; ls < ns; ls += NW) {
      const int v = lane < tau ? mp.set_inds[(size_t)(s_begin + ls) * tau + lane] : -2;
      const int prev = __shfl_up(v, 1, 64);
      const bool first = lane < tau && (lane == 0 || v != prev);   // repeats are adjacent
      const unsigned long long mask = __ballot(first);
      if (lane == 0) set_nu[ls] = __popcll(mask);
    }
    lds_barrier();
    if (tid == 0) {
      int r = 0, n = 0;
      for (int s = 0; s < ns; ++s) {             // each set starts on a multiple of 4 rows
        set_r0[s] = r; r += (set_nu[s] + 3) & ~3;
        const int kts = (set_nu[s] + 15) >> 4;
        for (int qt = 0; qt < kts; ++qt)
          for (int hh = 0; hh < item_groups(kts, HEADS); ++hh)
            if (n < kMaxItems) items[n++] = s | (qt << 8) | (hh << 12) | (kts << 16);
      }
      set_r0[ns] = r;
      items[kMaxItems] = n;
    }
    lds_barrier();
    for (int ls = wave; ls < ns; ls += NW) {
      const int v = lane < tau ? mp.set_inds[(size_t)(s_begin + ls) * tau + lane] : -2;
      const int prev = __shfl_up(v, 1, 64);
      const bool first = lane < tau && (lane == 0 || v != prev);
      const unsigned long long mask = __ballot(first);
      if (first && v >= 0 && v < mp.n_voxels) {
        const int r = set_r0[ls] + __popcll(mask & ((1ull << lane) - 1ull));
        const unsigned long long later = mask >> (lane + 1);
        const int run = later ? (__ffsll((long long)later)) : (tau - lane);   // slots holding this voxel
        const int4 c = coords[v];
        row_vox[r] = v;
        row_mult[r] = (float)run;
        row_lin[r] = (c.y * p.rel_my + c.z) * p.rel_mz + c.w;
      }
    }
    lds_barrier();
  }
  DSVT_PHASE(1);                                 // rows known
  const int R = __builtin_amdgcn_readfirstlane(set_r0[ns]);
  const int RT = (R + 15) >> 4;
  const int RTK = ((RT + 1) >> 1) << 1;          // the LayerNorm phases run on an even number of row tiles

  // ---- 2. gather (Eq. 4): rows of x -> Xs, 16 bytes per thread, dead rows zero.  The loads are
  // unconditional (clamped addresses).  The Q/K/V weights are requested after the barrier that
  // publishes the rows, not here: the compute unit's memory pipeline takes one 1 KB fragment every
  // ~19 cycles whether it hits the cache or not, a wavefront stands still until its requests are
  // taken, and 216 fragments in front of the stores to LDS kept every wavefront from the barrier
  // for 3.4 k cycles (measured: gather 5.7 k -> 1.6 k cycles, the tile 47.4 k -> 45.7 k).
  {
    constexpr int CH = C * (int)sizeof(T) / 16, G = (kRowsMax * CH + NTHREADS - 1) / NTHREADS;
    uint4 gv[G];
    bool live[G];
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const int idx = tid + k * NTHREADS;
      const int r = idx / CH, c = idx - r * CH;
      const int v = r < RTK * 16 ? row_vox[r] : -1;
      live[k] = v >= 0;
      gv[k] = reinterpret_cast<const uint4*>(x + (size_t)(v >= 0 ? v : 0) * C)[c];
    }
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const int idx = tid + k * NTHREADS;
      const int r = idx / CH, c = idx - r * CH;
      if (idx < RTK * 16 * CH)
        *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(Xs) + (size_t)r * LDX * sizeof(T) + c * 16) =
            live[k] ? gv[k] : make_uint4(0u, 0u, 0u, 0u);
    }
  }
  lds_barrier();
  DSVT_REFRESH_LANE();
  DSVT_PHASE(2);                                 // rows in LDS
  qkv.prefetch(p.b_qkv, 2 * C / (16 * NT_QKV));

  // ---- 3. Q, K, V = X W^T + b; V stored transposed
  {
    // the V items run with exchanged MFMA operands: a lane then holds four consecutive rows of one
    // feature, i.e. 8 contiguous bytes of V^T (a plain store instead of four 2-byte ones)
    static_assert((C / 16) % NT_QKV == 0, "an item never straddles the Q/K/V boundary");
    const float q_scale = rsqrtf((float)L::D) * 1.4426950408889634f;
    qkv.run(Xs, LDX, RT, p.b_qkv, [&](int o0, int r, f32x4 (&acc)[NT_QKV], bool swapped) {
      if (swapped) {
#pragma unroll
        for (int nt = 0; nt < NT_QKV; ++nt)
          *reinterpret_cast<Vec4*>(Vt + (o0 - 2 * C + 16 * nt + m) * LDV + 16 * r + 4 * g) = pack4<T>(acc[nt]);
      } else {
        const int row = 16 * r + m;
#pragma unroll
        for (int nt = 0; nt < NT_QKV; ++nt) {
          const int ot = o0 + 16 * nt;
          const int o = ot + 4 * g;
          if (ot < C) *reinterpret_cast<Vec4*>(Qs + row * LDX + o) = pack4<T>(acc[nt] * q_scale);   // logits in units of log2(e)
          else *reinterpret_cast<Vec4*>(Ks + row * LDX + (o - C)) = pack4<T>(acc[nt]);
        }
      }
    }, 2 * C / (16 * NT_QKV));
  }
  GemmPhase<T, NT_O, C, C, NW, 2> oproj(reinterpret_cast<const T*>(p.w_o), wave);
  oproj.prefetch();                              // in flight during the attention phase
  // LayerNorm phases (small weight matrices): every wavefront owns C / 4 features of one half of
  // the row tiles; the Q/K/V and first MLP projections (bandwidth-heavy) give a wavefront all rows
  // of its output tiles instead, so that each of their weight fragments is loaded only once
  const int og_own = wave % SG;
  const int rt_own = (wave / SG) * (RTK >> 1), HC = wave < 2 * SG ? RTK >> 1 : 0;   // HC = 0: a wavefront without an item
  const int o_own = og_own * 16 * NT_O;
  lds_barrier();
  DSVT_REFRESH_LANE();

  DSVT_PHASE(3);                                 // Q, K, V^T in LDS
  // ---- 4. attention inside every set; O overwrites Q
  {
    const int n_items = __builtin_amdgcn_readfirstlane(items[kMaxItems]);
    for (int it = wave; it < n_items; it += NW) {
      const int d = __builtin_amdgcn_readfirstlane(items[it]);
      const int s = d & 255, qt = (d >> 8) & 15, hh = (d >> 12) & 15, kts = d >> 16;
      const int r0 = __builtin_amdgcn_readfirstlane(set_r0[s]), nu = __builtin_amdgcn_readfirstlane(set_nu[s]);
      attn_any<T, C, HEADS, HID, BIG, DUP>(p, Qs, Ks, Vt, row_lin, row_mult, r0, nu, qt, hh, kts, RT * 16);
    }
  }
  f32x4 bo4[NT_O];
#pragma unroll
  for (int nt = 0; nt < NT_O; ++nt) bo4[nt] = *reinterpret_cast<const f32x4*>(p.b_o + o_own + 16 * nt + 4 * g);
  lds_barrier();
  DSVT_REFRESH_LANE();
  DSVT_PHASE(4);                                 // attention done
  // attention is done with V^T: the GELU table of the MLP takes its place (published by the
  // barriers of the LayerNorm below)
  constexpr bool kGeluTable = sizeof(T) == 2;
  static_assert(kGeluKnots * sizeof(float2) <= 4096, "GELU table slot");
  const float2* gelu_lds = reinterpret_cast<const float2*>(smem + L::off_gelu);
  if (kGeluTable && full_layer && tid < kGeluKnots / 2)
    reinterpret_cast<float4*>(smem + L::off_gelu)[tid] = reinterpret_cast<const float4*>(p.gelu_tab)[tid];

  // ---- 5. Y = O Wo^T + bo (+ x), then LayerNorm; result (or raw Y) replaces x in Xs
  // The first MLP matrix is requested during this phase, by a third of the wavefronts at a time
  // (before the projection, after it, after the residual): a CU takes a 16-byte load per
  // wavefront every ~16 cycles, a wavefront waits until its requests are taken, and twelve
  // wavefronts asking at once would all stand still for 3 k cycles.
  GemmPhase<T, NT_1, C, HID, NW, 1, false> ffn1(reinterpret_cast<const T*>(p.w_1), wave);
  const int pf_turn = full_layer ? wave / (NW / 3) : -1;
  if (pf_turn == 0) ffn1.prefetch();
  f32x4 keep[NT_O][kHalfTiles];
  if (HC == 1) oproj.template run_keep<1>(Qs, LDX, rt_own, bo4, keep);
  else if (HC == 2) oproj.template run_keep<2>(Qs, LDX, rt_own, bo4, keep);
  else if (HC == 3) oproj.template run_keep<3>(Qs, LDX, rt_own, bo4, keep);
  if (pf_turn == 1) ffn1.prefetch();
  f32x4 g1[NT_O], be1[NT_O];                       // fetched while the MFMAs above drain
#pragma unroll
  for (int nt = 0; nt < NT_O; ++nt) {
    g1[nt] = full_layer ? *reinterpret_cast<const f32x4*>(p.ln1_g + o_own + 16 * nt + 4 * g) : bo4[nt];
    be1[nt] = full_layer ? *reinterpret_cast<const f32x4*>(p.ln1_b + o_own + 16 * nt + 4 * g) : bo4[nt];
  }
#pragma unroll
  for (int nt = 0; nt < NT_O; ++nt) {
    const int o = o_own + 16 * nt + 4 * g;
#pragma unroll
    for (int r = 0; r < kHalfTiles; ++r) {
      if (r < HC) {
        if (full_layer) {
          const Vec4 xr = *reinterpret_cast<const Vec4*>(Xs + (16 * (rt_own + r) + m) * LDX + o);
          keep[nt][r] += f32x4{to_f32<T>(xr[0]), to_f32<T>(xr[1]), to_f32<T>(xr[2]), to_f32<T>(xr[3])};
        } else {
          *reinterpret_cast<Vec4*>(Xs + (16 * (rt_own + r) + m) * LDX + o) = pack4<T>(keep[nt][r]);
        }
      }
    }
  }
  if (full_layer) {
    if (pf_turn == 2) ffn1.prefetch();
    layer_norm_tile<T, NT_O, C, kHalfTiles>(keep, o_own, og_own, rt_own, HC, stat, g1, be1, p.ln_eps, Xs, LDX);
    lds_barrier();
    DSVT_REFRESH_LANE();

    DSVT_PHASE(5);                               // x1 in LDS
    // ---- 6. MLP: H = gelu(x1 W1^T + b1) over the dead Q/K tiles; x2 = LN(x1 + H W2^T + b2)
    ffn1.run(Xs, LDX, RT, p.b_1, [&](int o0, int r, f32x4 (&acc)[NT_1], bool) {
#pragma unroll
      for (int nt = 0; nt < NT_1; ++nt) {
        const int o = o0 + 16 * nt + 4 * g;
        f32x4 v = acc[nt];
        if constexpr (kGeluTable)
          v = f32x4{gelu_from_table(gelu_lds, v[0]), gelu_from_table(gelu_lds, v[1]), gelu_from_table(gelu_lds, v[2]), gelu_from_table(gelu_lds, v[3])};
        else
          v = f32x4{gelu_erf_fast<T>(v[0]), gelu_erf_fast<T>(v[1]), gelu_erf_fast<T>(v[2]), gelu_erf_fast<T>(v[3])};
        *reinterpret_cast<Vec4*>(Hs + (16 * r + m) * LDH + o) = pack4<T>(v);
      }
    });
    GemmPhase<T, NT_2, HID, C, NW, 2, true, (HID / Mma<T>::KC > 8 ? 2 : 1)> ffn2(reinterpret_cast<const T*>(p.w_2), wave);
    ffn2.prefetch();
    const int o_own2 = og_own * 16 * NT_2;
    f32x4 b24[NT_2];
#pragma unroll
    for (int nt = 0; nt < NT_2; ++nt) b24[nt] = *reinterpret_cast<const f32x4*>(p.b_2 + o_own2 + 16 * nt + 4 * g);
    lds_barrier();
    DSVT_REFRESH_LANE();
    DSVT_PHASE(6);                               // H in LDS
    f32x4 keep2[NT_2][kHalfTiles];
    if (HC == 1) ffn2.template run_keep<1>(Hs, LDH, rt_own, b24, keep2);
    else if (HC == 2) ffn2.template run_keep<2>(Hs, LDH, rt_own, b24, keep2);
    else if (HC == 3) ffn2.template run_keep<3>(Hs, LDH, rt_own, b24, keep2);
    f32x4 g2[NT_2], be2[NT_2];
#pragma unroll
    for (int nt = 0; nt < NT_2; ++nt) {
      g2[nt] = *reinterpret_cast<const f32x4*>(p.ln2_g + o_own2 + 16 * nt + 4 * g);
      be2[nt] = *reinterpret_cast<const f32x4*>(p.ln2_b + o_own2 + 16 * nt + 4 * g);
    }
#pragma unroll
    for (int nt = 0; nt < NT_2; ++nt) {
      const int o = o_own2 + 16 * nt + 4 * g;
#pragma unroll
      for (int r = 0; r < kHalfTiles; ++r) {
        if (r < HC) {
          const Vec4 xr = *reinterpret_cast<const Vec4*>(Xs + (16 * (rt_own + r) + m) * LDX + o);
          keep2[nt][r] += f32x4{to_f32<T>(xr[0]), to_f32<T>(xr[1]), to_f32<T>(xr[2]), to_f32<T>(xr[3])};
        }
      }
    }
    layer_norm_tile<T, NT_2, C, kHalfTiles>(keep2, o_own2, og_own, rt_own, HC, stat, g2, be2, p.ln_eps, Xs, LDX);
  }
  lds_barrier();
  DSVT_REFRESH_LANE();

  DSVT_PHASE(7);                                 // x2 in LDS
  // ---- 7. scatter: rows of Xs -> the voxels' rows of out, 16 bytes per thread
  {
    constexpr int CH = C * (int)sizeof(T) / 16;
    for (int idx = tid; idx < R * CH; idx += NTHREADS) {
      const int r = idx / CH, c = idx - r * CH;
      const int v = row_vox[r];
      if (v >= 0)
        reinterpret_cast<uint4*>(out + (size_t)v * C)[c] =
            *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(Xs) + (size_t)r * LDX * sizeof(T) + c * 16);
    }
  }
  DSVT_PHASE(8);
}

// ------------------------------------------------------------------------------------------
// Packed buffer of a layer: the four matrices in fragment order, each on a 256-byte boundary.
struct PackedLayout { size_t off[6], total; int out[4], k[4]; int rel_size; };   // off[4]: position table [index][heads], off[5]: GELU table
PackedLayout packed_layout(const dsvt_layer_w& w) {
  PackedLayout pl;
  const size_t es = w.dtype == DSVT_BF16 ? 2 : 4;
  const int out[4] = {3 * w.C, w.C, w.hidden, w.C}, k[4] = {w.C, w.C, w.C, w.hidden};
  size_t o = 0;
  for (int i = 0; i < 4; ++i) { pl.off[i] = o; pl.out[i] = out[i]; pl.k[i] = k[i]; o = dsvt_align_up(o + (size_t)out[i] * k[i] * es, 256); }
  // position table [index][heads] plus one last row of -inf (the row of a key that does not exist); without a
  // positional term the table is one row of zeros and that last row
  pl.rel_size = w.rel_bias != nullptr ? (2 * w.win[0] - 1) * (2 * w.win[1] - 1) * (2 * w.win[2] - 1) : 1;
  pl.off[4] = o;
  o = dsvt_align_up(o + (size_t)(pl.rel_size + 1) * w.heads * 4, 256);
  pl.off[5] = o;
  o = dsvt_align_up(o + (size_t)kGeluKnots * sizeof(float2), 256);
  pl.total = o;
  return pl;
}

// [heads][size] -> [size + 1][heads], in units of log2(e) (the softmax works with exp2); row `size` holds -inf.
// src == nullptr (no positional term): zeros.
__global__ void k_pack_table(const float* __restrict__ src, float* __restrict__ dst, int heads, int size) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < heads * size) dst[(i % size) * heads + i / size] = src != nullptr ? src[i] * 1.4426950408889634f : 0.f;
  else if (i < heads * (size + 1)) dst[i] = -INFINITY;
}

LayerDev to_dev(const dsvt_layer_w& w) {
  LayerDev d;
  const PackedLayout pl = packed_layout(w);
  const char* pk = reinterpret_cast<const char*>(w.packed);
  d.w_qkv = pk + pl.off[0]; d.w_o = pk + pl.off[1]; d.w_1 = pk + pl.off[2]; d.w_2 = pk + pl.off[3];
  d.b_qkv = w.b_qkv; d.b_o = w.b_o; d.b_1 = w.b_1; d.b_2 = w.b_2;
  d.ln1_g = w.ln1_g; d.ln1_b = w.ln1_b; d.ln2_g = w.ln2_g; d.ln2_b = w.ln2_b;
  d.rel_bias = reinterpret_cast<const float*>(pk + pl.off[4]);
  d.gelu_tab = reinterpret_cast<const float2*>(pk + pl.off[5]);
  d.ln_eps = w.ln_eps; d.dup_mode = w.dup_mode;
  const int my = 2 * w.win[1] - 1, mz = 2 * w.win[2] - 1;
  d.rel_my = my; d.rel_mz = mz;
  d.rel_size = pl.rel_size;
  d.rel_const = w.rel_bias != nullptr ? ((w.win[0] - 1) * my + (w.win[1] - 1)) * mz + (w.win[2] - 1) : 0;
  return d;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_layer(const dsvt_layer_w& w, bool need_mlp, bool need_packed = true) {
  if (!w.w_qkv || !w.w_o || !w.b_qkv || !w.b_o) return DSVT_EINVAL;
  if (need_packed && (!w.packed || !aligned16(w.packed))) return DSVT_EINVAL;
  if (need_mlp && (!w.w_1 || !w.w_2 || !w.b_1 || !w.b_2 || !w.ln1_g || !w.ln1_b || !w.ln2_g || !w.ln2_b)) return DSVT_EINVAL;
  if (w.dtype != DSVT_F32 && w.dtype != DSVT_BF16) return DSVT_EINVAL;
  if (w.dup_mode != 0 && w.dup_mode != 1) return DSVT_EINVAL;
  for (int a = 0; a < 3; ++a) if (w.win[a] <= 0) return DSVT_EINVAL;
  if (!((w.C == 64 && w.heads == 4 && w.hidden == 128) || (w.C == 128 && w.heads == 8 && w.hidden == 256) ||
        (w.C == 192 && w.heads == 8 && w.hidden == 384)))
    return DSVT_EUNSUPPORTED;
  if (w.dtype == DSVT_F32 && w.C != 64) return DSVT_EUNSUPPORTED;   // wider fp32 tiles exceed the 160 KB LDS
  const void* ptrs[] = {w.w_qkv, w.w_o, w.w_1, w.w_2, w.b_qkv, w.b_o, w.b_1, w.b_2, w.ln1_g, w.ln1_b, w.ln2_g, w.ln2_b};
  for (const void* q : ptrs) if (q && !aligned16(q)) return DSVT_EINVAL;
  return DSVT_OK;
}

int check_maps(const dsvt_maps& mp) {
  if (!mp.set_inds || !mp.n_sets || mp.n_voxels <= 0 || mp.max_sets <= 0 || mp.tau <= 0) return DSVT_EINVAL;
  if (mp.tau > kTauMax) return DSVT_EUNSUPPORTED;
  if (mp.tiles.tile_desc == nullptr && mp.tau > 64) return DSVT_EUNSUPPORTED;   // without a work list a wavefront scans a set's tau slots
  const dsvt_tile_list& tl = mp.tiles;
  const bool any = tl.tile_first || tl.n_tiles || tl.tile_order || tl.tile_desc;
  const bool all = tl.tile_first && tl.n_tiles && tl.tile_order && tl.tile_desc;
  if (any && (!all || tl.max_tiles <= 0)) return DSVT_EINVAL;
  return DSVT_OK;
}

template <typename T, int C, int HEADS, int HID, int NT_QKV, int NT_O, int NT_1, int NT_2, bool BIG, bool DUP>
int launch_layer_v(const dsvt_layer_w& w, const dsvt_maps& mp, const int32_t* coords, const void* x, void* out, int full,
                   hipStream_t st) {
  auto kern = k_layer<T, C, HEADS, HID, NT_QKV, NT_O, NT_1, NT_2, BIG, DUP>;
  constexpr size_t lds = LayerLds<T, C, HEADS, HID>::total;
  static std::atomic<uint64_t> lds_allowed{0};
  if (int rc = dsvt_allow_lds(reinterpret_cast<const void*>(kern), lds, lds_allowed)) return rc;
  MapsDev md;
  md.set_inds = mp.set_inds; md.n_sets = mp.n_sets; md.n_tiles = mp.tiles.n_tiles; md.tile_desc = mp.tiles.tile_desc;
  md.max_sets = mp.max_sets; md.tau = mp.tau; md.n_voxels = mp.n_voxels;
  const unsigned grid = mp.tiles.tile_desc ? (unsigned)mp.tiles.max_tiles : (unsigned)dsvt_ceil_div(mp.max_sets, fixed_sets(mp.tau));
  dsvt_prof_scope ps(DSVT_K_LAYER, st);
  kern<<<grid, kLayerWaves * 64, lds, st>>>(to_dev(w), md, reinterpret_cast<const int4*>(coords),
                                       reinterpret_cast<const T*>(x), reinterpret_cast<T*>(out), full);
  return DSVT_OK;
}

template <typename T, int C, int HEADS, int HID, int NT_QKV, int NT_O, int NT_1, int NT_2>
int launch_layer(const dsvt_layer_w& w, const dsvt_maps& mp, const int32_t* coords, const void* x, void* out, int full,
                 hipStream_t st) {
  // four instantiations per shape: sets of more than 48 voxels (tau > 48) take one head per attention item, and
  // repeated slots that count as keys (dup_mode 1) multiply the exponentials by the slots' counts
  const bool big = mp.tau > 48, dup = w.dup_mode != 0;
  if (big && dup) return launch_layer_v<T, C, HEADS, HID, NT_QKV, NT_O, NT_1, NT_2, true, true>(w, mp, coords, x, out, full, st);
  if (big) return launch_layer_v<T, C, HEADS, HID, NT_QKV, NT_O, NT_1, NT_2, true, false>(w, mp, coords, x, out, full, st);
  if (dup) return launch_layer_v<T, C, HEADS, HID, NT_QKV, NT_O, NT_1, NT_2, false, true>(w, mp, coords, x, out, full, st);
  return launch_layer_v<T, C, HEADS, HID, NT_QKV, NT_O, NT_1, NT_2, false, false>(w, mp, coords, x, out, full, st);
}

int run_layer(const dsvt_layer_w& w, const dsvt_maps& mp, const int32_t* coords, const void* x, void* out, int full,
              hipStream_t st) {
  if (w.dtype == DSVT_BF16) {
    if (w.C == 192) return launch_layer<bf16_t, 192, 8, 384, 3, 2, 2, 2>(w, mp, coords, x, out, full, st);
    if (w.C == 128) return launch_layer<bf16_t, 128, 8, 256, 2, 2, 2, 2>(w, mp, coords, x, out, full, st);
    return launch_layer<bf16_t, 64, 4, 128, 1, 1, 1, 1>(w, mp, coords, x, out, full, st);
  }
  return launch_layer<float, 64, 4, 128, 1, 1, 1, 1>(w, mp, coords, x, out, full, st);
}

}  // namespace


extern "C" int dsvt_layer_packed_size(const dsvt_layer_w* layer, size_t* bytes) {
  if (!layer || !bytes) return DSVT_EINVAL;
  int rc = check_layer(*layer, true, false);
  if (rc != DSVT_OK) return rc;
  *bytes = packed_layout(*layer).total;
  return DSVT_OK;
}

extern "C" int dsvt_layer_pack(const dsvt_layer_w* layer, void* packed, size_t bytes, void* stream) {
  if (!layer || !packed || !aligned16(packed)) return DSVT_EINVAL;
  int rc = check_layer(*layer, true, false);
  if (rc != DSVT_OK) return rc;
  const PackedLayout pl = packed_layout(*layer);
  if (bytes < pl.total) return DSVT_ENOSPC;
  const void* src[4] = {layer->w_qkv, layer->w_o, layer->w_1, layer->w_2};
  hipStream_t st = (hipStream_t)stream;
  for (int i = 0; i < 4; ++i) {
    char* dst = reinterpret_cast<char*>(packed) + pl.off[i];
    if (layer->dtype == DSVT_BF16) {
      const long long slots = (long long)(pl.out[i] / 16) * (pl.k[i] / Mma<bf16_t>::KC) * 64;
      k_pack<bf16_t><<<(unsigned)dsvt_ceil_div(slots, 256), 256, 0, st>>>(reinterpret_cast<const bf16_t*>(src[i]),
                                                                        reinterpret_cast<bf16_t*>(dst), pl.out[i], pl.k[i]);
    } else {
      const long long slots = (long long)(pl.out[i] / 16) * (pl.k[i] / Mma<float>::KC) * 64;
      k_pack<float><<<(unsigned)dsvt_ceil_div(slots, 256), 256, 0, st>>>(reinterpret_cast<const float*>(src[i]),
                                                                       reinterpret_cast<float*>(dst), pl.out[i], pl.k[i]);
    }
  }
  k_pack_gelu_table<<<(unsigned)dsvt_ceil_div(kGeluKnots, 256), 256, 0, st>>>(
      reinterpret_cast<float2*>(reinterpret_cast<char*>(packed) + pl.off[5]));
  {
    const int n = (pl.rel_size + 1) * layer->heads;
    k_pack_table<<<(unsigned)dsvt_ceil_div(n, 256), 256, 0, st>>>(
        layer->rel_bias, reinterpret_cast<float*>(reinterpret_cast<char*>(packed) + pl.off[4]), layer->heads, pl.rel_size);
  }
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}

extern "C" int dsvt_set_attention_workspace_size(const dsvt_layer_w* layer, int32_t n_voxels, size_t* bytes) {
  if (!layer || !bytes || n_voxels <= 0) return DSVT_EINVAL;
  *bytes = 0;
  return DSVT_OK;
}

extern "C" int dsvt_block_workspace_size(const dsvt_layer_w* layer, int32_t n_voxels, size_t* bytes) {
  if (!layer || !bytes || n_voxels <= 0) return DSVT_EINVAL;
  *bytes = 0;
  return DSVT_OK;
}

extern "C" int dsvt_set_attention(const dsvt_layer_w* layer, const dsvt_maps* maps, const int32_t* coords,
                                  const void* x, void* y, void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  if (!layer || !maps || !coords || !x || !y || x == y) return DSVT_EINVAL;
  int rc = check_layer(*layer, false);
  if (rc != DSVT_OK) return rc;
  rc = check_maps(*maps);
  if (rc != DSVT_OK) return rc;
  if (!aligned16(x) || !aligned16(y) || !aligned16(coords)) return DSVT_EINVAL;
  rc = run_layer(*layer, *maps, coords, x, y, 0, (hipStream_t)stream);
  if (rc != DSVT_OK) return rc;
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}

extern "C" int dsvt_block(const dsvt_layer_w layer[2], const dsvt_maps maps[2], const int32_t* coords,
                          const void* x_in, void* x_out, void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  if (!layer || !maps || !coords || !x_in || !x_out) return DSVT_EINVAL;
  for (int l = 0; l < 2; ++l) {
    int rc = check_layer(layer[l], true);
    if (rc != DSVT_OK) return rc;
    rc = check_maps(maps[l]);
    if (rc != DSVT_OK) return rc;
    if (layer[l].C != layer[0].C || layer[l].dtype != layer[0].dtype || maps[l].n_voxels != maps[0].n_voxels)
      return DSVT_EINVAL;
  }
  if (!aligned16(x_in) || !aligned16(x_out) || !aligned16(coords)) return DSVT_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const void* src = x_in;
  for (int l = 0; l < 2; ++l) {
    int rc = run_layer(layer[l], maps[l], coords, src, x_out, 1, st);
    if (rc != DSVT_OK) return rc;
    src = x_out;
  }
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}
