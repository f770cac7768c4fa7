// dsvt_set_attention / dsvt_block: one DSVT layer per kernel launch on gfx950 (Sec. 3.2 Eq. 4-5;
// appendix "Network Architecture").
//
// k_layer: a workgroup owns a run of consecutive sets (a "tile" of at most 96 rows).  It reads
// their slot rows of set_inds, keeps the first occurrence of every voxel (repeats are adjacent,
// Eq. 3 is monotone), and gathers those voxels' features into an LDS tile -- the tau x C tiles of
// Eq. (4) with the repeated rows squeezed out, since a masked repeat contributes nothing as a key
// and its query row would be thrown away.  Q/K/V projection, per-(set, head) softmax(QK^T + PE)V,
// output projection, residual + LayerNorm, the MLP and the second residual + LayerNorm all run
// on that tile in LDS and registers; the rows then go straight back to the voxels' rows of the
// output (every voxel is in exactly one set, Thm A.2-A.3), so a layer reads and writes [N, C] once.
#include "common.h"
#include "mma.h"

namespace {

constexpr int kTauMax = 48;
constexpr int kRowsMax = 96;                     // rows of a tile = 6 MFMA row tiles
constexpr int kKeyTiles = kTauMax / 16;          // 3
constexpr int kMaxSets = kRowsMax / 4;           // every set takes at least 4 rows of a tile
constexpr int kFixedSets = kRowsMax / kTauMax;   // sets per workgroup when no tile list is given
constexpr int kWaves = 8;
constexpr int kStatGroups = 4;                   // output-tile groups of the LayerNorm phases

struct LayerDev {
  const void *w_qkv, *w_o, *w_1, *w_2;
  const float *b_qkv, *b_o, *b_1, *b_2, *ln1_g, *ln1_b, *ln2_g, *ln2_b, *rel_bias;
  float ln_eps;
  int rel_size, rel_const, rel_my, rel_mz;   // table entries per head; index = lin(q) - lin(k) + rel_const
  int dup_mode;
};

struct MapsDev {
  const int32_t *set_inds, *n_sets, *tile_first, *n_tiles;
  int32_t max_sets, tau, n_voxels;
};

template <typename T, int C, int HEADS, int HID> struct LayerLds {
  static constexpr int D = C / HEADS;
  static constexpr int PAD = lds_pad<T>();
  static constexpr int LDX = C + PAD;            // pitch of [row][feature] tiles, elements of T
  static constexpr int LDV = kRowsMax + PAD;     // pitch of V^T [feature][row]
  static constexpr int LDH = HID + PAD;          // pitch of the MLP hidden tile
  static constexpr size_t kTile = (size_t)kRowsMax * LDX * sizeof(T);
  static constexpr size_t off_x = 0, off_q = kTile, off_k = 2 * kTile, off_v = 3 * kTile;
  static constexpr size_t kVt = (size_t)C * LDV * sizeof(T);
  static constexpr size_t off_h = off_q;         // hidden tile reuses Q and K once attention is done
  static constexpr size_t off_misc = off_v + kVt;
  static constexpr size_t kMisc = (size_t)(3 * kRowsMax + 2 * kMaxSets + 2 + 2 * kStatGroups * kRowsMax) * 4;
  static constexpr size_t total = off_misc + kMisc;
  static_assert((size_t)kRowsMax * LDH * sizeof(T) <= 2 * kTile, "hidden tile must fit in Q + K");
  static_assert(C % 64 == 0 && D % Mma<T>::KL == 0 && D % 4 == 0, "shape");
};

// LayerNorm over the C features of every row, for values spread over the workgroup in
// accumulator layout: this wavefront holds features o0 .. o0 + 16*NT - 1 (group og of
// kStatGroups) of rows 16*(rt0 + r) + m, r < cnt.  Two-pass (mean, then centred squares) with
// the per-group partial sums exchanged through LDS.  Every thread of the workgroup must call it.
template <typename T, int NT>
__device__ __forceinline__ void layer_norm_tile(f32x4 (&v)[NT][3], int C, int o0, int og, int rt0, int cnt, float* stat,
                                                const float* __restrict__ gamma, const float* __restrict__ beta,
                                                float eps, T* dst, int ldd) {
  typedef typename Mma<T>::Vec4 Vec4;
  const int lane = threadIdx.x & 63, m = lane & 15, g = lane >> 4;
  float* stat1 = stat;
  float* stat2 = stat + kStatGroups * kRowsMax;
  float mean[3], rs[3];
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    float s = 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) s += v[nt][r][0] + v[nt][r][1] + v[nt][r][2] + v[nt][r][3];
    s += __shfl_xor(s, 16, 64);
    s += __shfl_xor(s, 32, 64);
    if (g == 0 && r < cnt) stat1[og * kRowsMax + 16 * (rt0 + r) + m] = s;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    mean[r] = 0.f;
    if (r < cnt) {
      const int row = 16 * (rt0 + r) + m;
      float t = 0.f;
#pragma unroll
      for (int k = 0; k < kStatGroups; ++k) t += stat1[k * kRowsMax + row];
      mean[r] = t / (float)C;
    }
    float s = 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      v[nt][r] -= mean[r];
      s += v[nt][r][0] * v[nt][r][0] + v[nt][r][1] * v[nt][r][1] + v[nt][r][2] * v[nt][r][2] + v[nt][r][3] * v[nt][r][3];
    }
    s += __shfl_xor(s, 16, 64);
    s += __shfl_xor(s, 32, 64);
    if (g == 0 && r < cnt) stat2[og * kRowsMax + 16 * (rt0 + r) + m] = s;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    if (r < cnt) {
      const int row = 16 * (rt0 + r) + m;
      float t = 0.f;
#pragma unroll
      for (int k = 0; k < kStatGroups; ++k) t += stat2[k * kRowsMax + row];
      rs[r] = rsqrtf(t / (float)C + eps);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int o = o0 + 16 * nt + 4 * g;
        const f32x4 ga = *reinterpret_cast<const f32x4*>(gamma + o), be = *reinterpret_cast<const f32x4*>(beta + o);
        *reinterpret_cast<Vec4*>(dst + row * ldd + o) = pack4<T>(v[nt][r] * rs[r] * ga + be);
      }
    }
  }
}

template <typename T, int C, int HEADS, int HID, int NT_QKV, int NT_O, int NT_1, int NT_2, int KSPLIT_2>
__global__ void __launch_bounds__(kWaves * 64)
k_layer(LayerDev p, MapsDev mp, const int4* __restrict__ coords, const T* x, T* out, int full_layer) {
  // out may be x: a tile's rows are read, then written, by this workgroup only
  typedef LayerLds<T, C, HEADS, HID> L;
  typedef Mma<T> M;
  typedef typename M::Frag Frag;
  typedef typename M::Vec4 Vec4;
  constexpr int D = L::D, LDX = L::LDX, LDV = L::LDV, LDH = L::LDH, KC = M::KC, KL = M::KL;
  constexpr int NW = kWaves, NTHREADS = NW * 64;
  static_assert(C / (16 * NT_O) == kStatGroups && C / (16 * NT_2) == kStatGroups, "LayerNorm phases: one item per wave");
  extern __shared__ __align__(16) unsigned char smem[];
  T* Xs = reinterpret_cast<T*>(smem + L::off_x);
  T* Qs = reinterpret_cast<T*>(smem + L::off_q);
  T* Ks = reinterpret_cast<T*>(smem + L::off_k);
  T* Vt = reinterpret_cast<T*>(smem + L::off_v);
  T* Hs = reinterpret_cast<T*>(smem + L::off_h);
  int32_t* row_vox = reinterpret_cast<int32_t*>(smem + L::off_misc);
  int32_t* row_lin = row_vox + kRowsMax;
  float* row_mult = reinterpret_cast<float*>(row_lin + kRowsMax);
  int32_t* set_r0 = reinterpret_cast<int32_t*>(row_mult + kRowsMax);   // [kMaxSets + 1]
  int32_t* set_nu = set_r0 + kMaxSets + 1;                              // [kMaxSets + 1]
  float* stat = reinterpret_cast<float*>(set_nu + kMaxSets + 1);        // [2][kStatGroups][kRowsMax]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, m = lane & 15, g = lane >> 4;

  // The first Q/K/V weight fragments are requested before anything else: their latency hides
  // behind the row bookkeeping and the gather.
  GemmPhase<T, NT_QKV, C, 3 * C, NW, 1> qkv(p.w_qkv, wave);
  qkv.issue(0);

  int n_sets = *mp.n_sets;
  n_sets = n_sets < mp.max_sets ? n_sets : mp.max_sets;
  int s_begin, s_end;
  if (mp.tile_first != nullptr) {
    if ((int)blockIdx.x >= *mp.n_tiles) return;
    s_begin = mp.tile_first[blockIdx.x];
    s_end = mp.tile_first[blockIdx.x + 1];
  } else {
    s_begin = blockIdx.x * kFixedSets;
    s_end = s_begin + kFixedSets;
  }
  s_end = s_end < n_sets ? s_end : n_sets;
  int ns = s_end - s_begin;
  if (ns <= 0 || s_begin < 0) return;
  ns = ns < kMaxSets ? ns : kMaxSets;
  const int tau = mp.tau;

  // ---- 1. slots -> compact rows (first occurrences only; each set starts on a multiple of 4 rows)
  for (int r = tid; r < kRowsMax; r += NTHREADS) { row_vox[r] = -1; row_lin[r] = 0; row_mult[r] = 0.f; }
  for (int ls = wave; ls < ns; ls += NW) {
    const int v = lane < tau ? mp.set_inds[(size_t)(s_begin + ls) * tau + lane] : -2;
    const int prev = __shfl_up(v, 1, 64);
    const bool first = lane < tau && (lane == 0 || v != prev);
    const unsigned long long mask = __ballot(first);
    if (lane == 0) set_nu[ls] = __popcll(mask);
  }
  __syncthreads();
  if (tid == 0) {
    int r = 0, keep = 0;
    for (int s = 0; s < ns; ++s) {
      const int padded = (set_nu[s] + 3) & ~3;
      if (r + padded > kRowsMax) break;          // cannot happen with a tile list built for 96 rows
      set_r0[s] = r; r += padded; keep = s + 1;
    }
    set_r0[keep] = r;
    set_nu[kMaxSets] = keep;
  }
  __syncthreads();
  ns = set_nu[kMaxSets];
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
  __syncthreads();
  const int R = set_r0[ns];
  const int RT = (R + 15) >> 4;

  // ---- 2. gather (Eq. 4): rows of x -> Xs, 16 bytes per thread, dead rows zero
  {
    constexpr int CH = C * (int)sizeof(T) / 16;
    for (int idx = tid; idx < RT * 16 * CH; idx += NTHREADS) {
      const int r = idx / CH, c = idx - r * CH;
      const int v = row_vox[r];
      uint4 val = make_uint4(0u, 0u, 0u, 0u);
      if (v >= 0) val = reinterpret_cast<const uint4*>(x + (size_t)v * C)[c];
      *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(Xs) + (size_t)r * LDX * sizeof(T) + c * 16) = val;
    }
  }
  __syncthreads();

  // ---- 3. Q, K, V = X W^T + b; Q pre-scaled by 1/sqrt(d); V stored transposed
  {
    const float scale = rsqrtf((float)D);
    qkv.run(Xs, LDX, RT, [&](int o0, int rt0, int cnt, f32x4 (&acc)[NT_QKV][3]) {
#pragma unroll
      for (int nt = 0; nt < NT_QKV; ++nt) {
        const int ot = o0 + 16 * nt;             // a tile never straddles the Q/K/V boundary (C % 16 == 0)
        const int o = ot + 4 * g;
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.b_qkv + o);
        const int sel = ot / C;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
          if (r < cnt) {
            const int row = 16 * (rt0 + r) + m;
            f32x4 v = acc[nt][r] + b4;
            if (sel == 0) {
              v *= scale;
              *reinterpret_cast<Vec4*>(Qs + row * LDX + o) = pack4<T>(v);
            } else if (sel == 1) {
              *reinterpret_cast<Vec4*>(Ks + row * LDX + (o - C)) = pack4<T>(v);
            } else {
#pragma unroll
              for (int i = 0; i < 4; ++i) Vt[(o - 2 * C + i) * LDV + row] = (T)v[i];
            }
          }
        }
      }
    });
  }
  GemmPhase<T, NT_O, C, C, NW, 1> oproj(p.w_o, wave);
  oproj.issue(0);                                // in flight during the attention phase
  __syncthreads();

  // ---- 4. per (set, head): P = softmax(Q K^T + PE), O = P V; O overwrites the head's Q columns
  for (int item = wave; item < ns * HEADS; item += NW) {
    const int s = item / HEADS, h = item - s * HEADS;
    const int r0 = set_r0[s], nu = set_nu[s];
    const int KT = (nu + 15) >> 4;
    f32x4 S[kKeyTiles][kKeyTiles];               // S[kt][qt][i]: key 16kt+4g+i, query 16qt+m
#pragma unroll
    for (int a = 0; a < kKeyTiles; ++a)
#pragma unroll
      for (int b = 0; b < kKeyTiles; ++b) S[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < D; kc += KC) {
      const int kk = kc + g * KL;
      Frag fa[kKeyTiles], fb[kKeyTiles];
#pragma unroll
      for (int t = 0; t < kKeyTiles; ++t) {
        fa[t] = M::zero(); fb[t] = M::zero();
        if (t < KT && kk < D) {
          int rr = 16 * t + m; rr = r0 + (rr < nu ? rr : nu - 1);
          fa[t] = *reinterpret_cast<const Frag*>(Ks + rr * LDX + h * D + kk);
          fb[t] = *reinterpret_cast<const Frag*>(Qs + rr * LDX + h * D + kk);
        }
      }
#pragma unroll
      for (int kt = 0; kt < kKeyTiles; ++kt)
#pragma unroll
        for (int qt = 0; qt < kKeyTiles; ++qt)
          if (kt < KT && qt < KT) S[kt][qt] = M::mma(fa[kt], fb[qt], S[kt][qt]);
    }
    float inv[kKeyTiles];
    const float* table = p.rel_bias ? p.rel_bias + (size_t)h * p.rel_size : nullptr;
#pragma unroll
    for (int qt = 0; qt < kKeyTiles; ++qt) {
      inv[qt] = 0.f;
      if (qt < KT) {
        int q = 16 * qt + m; q = q < nu ? q : nu - 1;
        const int ql = row_lin[r0 + q] + p.rel_const;
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < kKeyTiles; ++kt) {
          if (kt < KT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int key = 16 * kt + 4 * g + i;
              float l = -INFINITY;
              if (key < nu) {
                l = S[kt][qt][i];
                if (table) {
                  int idx = ql - row_lin[r0 + key];
                  idx = idx < 0 ? 0 : (idx >= p.rel_size ? p.rel_size - 1 : idx);
                  l += table[idx];
                }
              }
              S[kt][qt][i] = l;
              mx = fmaxf(mx, l);
            }
          }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float sum = 0.f;
#pragma unroll
        for (int kt = 0; kt < kKeyTiles; ++kt) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float e = 0.f;
            if (kt < KT) {
              const int key = 16 * kt + 4 * g + i;
              if (key < nu) {
                e = __expf(S[kt][qt][i] - mx);
                if (p.dup_mode) e *= row_mult[r0 + key];
              }
            }
            S[kt][qt][i] = e;
            sum += e;
          }
        }
        sum += __shfl_xor(sum, 16, 64);
        sum += __shfl_xor(sum, 32, 64);
        inv[qt] = 1.0f / sum;
      }
    }
    // O^T[dv][q] = sum_key V^T[dv][key] P^T[key][q]; P^T comes straight from the registers above.
    constexpr int TPC = KC / 16;                  // key tiles per fragment: 2 (bf16) or 1 (fp32)
    constexpr int NCH = (kKeyTiles + TPC - 1) / TPC;
#pragma unroll
    for (int dt = 0; dt < (D + 15) / 16; ++dt) {
      f32x4 O[kKeyTiles];
#pragma unroll
      for (int qt = 0; qt < kKeyTiles; ++qt) O[qt] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int dv = 16 * dt + m;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        if (c * TPC < KT) {
          Frag fa = M::zero();
          if (dv < D) {
            const T* vrow = Vt + (h * D + dv) * LDV + r0 + 4 * g;
            if constexpr (TPC == 2) {
              bf16x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
              if (r0 + 32 * c + 4 * g < RT * 16) lo = *reinterpret_cast<const bf16x4*>(vrow + 32 * c);
              if (2 * c + 1 < KT && r0 + 32 * c + 16 + 4 * g < RT * 16)
                hi = *reinterpret_cast<const bf16x4*>(vrow + 32 * c + 16);
              fa = Frag{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            } else {
              if (r0 + 16 * c + 4 * g < RT * 16) fa = *reinterpret_cast<const Frag*>(vrow + 16 * c);
            }
          }
#pragma unroll
          for (int qt = 0; qt < kKeyTiles; ++qt) {
            if (qt < KT) {
              Frag fb;
              if constexpr (TPC == 2) {
                const f32x4 p0 = S[2 * c][qt];
                const f32x4 p1 = (2 * c + 1 < kKeyTiles) ? S[(2 * c + 1 < kKeyTiles) ? 2 * c + 1 : 0][qt]
                                                         : f32x4{0.f, 0.f, 0.f, 0.f};
                fb = Frag{(bf16_t)p0[0], (bf16_t)p0[1], (bf16_t)p0[2], (bf16_t)p0[3],
                          (bf16_t)p1[0], (bf16_t)p1[1], (bf16_t)p1[2], (bf16_t)p1[3]};
              } else {
                fb = S[c][qt];
              }
              O[qt] = M::mma(fa, fb, O[qt]);
            }
          }
        }
      }
#pragma unroll
      for (int qt = 0; qt < kKeyTiles; ++qt) {
        const int q = 16 * qt + m;
        if (qt < KT && q < nu && 16 * dt + 4 * g < D) {
          const f32x4 o4 = O[qt] * inv[qt];
          *reinterpret_cast<Vec4*>(Qs + (r0 + q) * LDX + h * D + 16 * dt + 4 * g) = pack4<T>(o4);
        }
      }
    }
  }
  __syncthreads();

  // ---- 5. Y = O Wo^T + bo (+ x), then LayerNorm; result (or raw Y) replaces x in Xs
  f32x4 keep[NT_O][3];
  int k_o0 = 0, k_rt0 = 0, k_cnt = 0;
  oproj.run(Qs, LDX, RT, [&](int o0, int rt0, int cnt, f32x4 (&acc)[NT_O][3]) {
    k_o0 = o0; k_rt0 = rt0; k_cnt = cnt;
#pragma unroll
    for (int nt = 0; nt < NT_O; ++nt) {
      const int o = o0 + 16 * nt + 4 * g;
      const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.b_o + o);
#pragma unroll
      for (int r = 0; r < 3; ++r) {
        keep[nt][r] = acc[nt][r] + b4;
        if (full_layer && r < cnt) {
          const Vec4 xr = *reinterpret_cast<const Vec4*>(Xs + (16 * (rt0 + r) + m) * LDX + o);
          keep[nt][r] += f32x4{to_f32<T>(xr[0]), to_f32<T>(xr[1]), to_f32<T>(xr[2]), to_f32<T>(xr[3])};
        }
      }
    }
  });
  if (!full_layer) {
#pragma unroll
    for (int nt = 0; nt < NT_O; ++nt)
#pragma unroll
      for (int r = 0; r < 3; ++r)
        if (r < k_cnt)
          *reinterpret_cast<Vec4*>(Xs + (16 * (k_rt0 + r) + m) * LDX + k_o0 + 16 * nt + 4 * g) = pack4<T>(keep[nt][r]);
  } else {
    GemmPhase<T, NT_1, C, HID, NW, 1> ffn1(p.w_1, wave);
    ffn1.issue(0);                               // in flight during the LayerNorm exchange
    layer_norm_tile<T, NT_O>(keep, C, k_o0, k_o0 / (16 * NT_O), k_rt0, k_cnt, stat, p.ln1_g, p.ln1_b, p.ln_eps, Xs, LDX);
    __syncthreads();

    // ---- 6. MLP: H = gelu(x1 W1^T + b1) over the dead Q/K tiles; x2 = LN(x1 + H W2^T + b2)
    ffn1.run(Xs, LDX, RT, [&](int o0, int rt0, int cnt, f32x4 (&acc)[NT_1][3]) {
#pragma unroll
      for (int nt = 0; nt < NT_1; ++nt) {
        const int o = o0 + 16 * nt + 4 * g;
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.b_1 + o);
#pragma unroll
        for (int r = 0; r < 3; ++r) {
          if (r < cnt) {
            f32x4 v = acc[nt][r] + b4;
            v = f32x4{gelu_erf(v[0]), gelu_erf(v[1]), gelu_erf(v[2]), gelu_erf(v[3])};
            *reinterpret_cast<Vec4*>(Hs + (16 * (rt0 + r) + m) * LDH + o) = pack4<T>(v);
          }
        }
      }
    });
    GemmPhase<T, NT_2, HID, C, NW, KSPLIT_2> ffn2(p.w_2, wave);
    ffn2.issue(0);
    __syncthreads();
    f32x4 keep2[NT_2][3];
    ffn2.run(Hs, LDH, RT, [&](int o0, int rt0, int cnt, f32x4 (&acc)[NT_2][3]) {
      k_o0 = o0; k_rt0 = rt0; k_cnt = cnt;
#pragma unroll
      for (int nt = 0; nt < NT_2; ++nt) {
        const int o = o0 + 16 * nt + 4 * g;
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.b_2 + o);
#pragma unroll
        for (int r = 0; r < 3; ++r) {
          keep2[nt][r] = acc[nt][r] + b4;
          if (r < cnt) {
            const Vec4 xr = *reinterpret_cast<const Vec4*>(Xs + (16 * (rt0 + r) + m) * LDX + o);
            keep2[nt][r] += f32x4{to_f32<T>(xr[0]), to_f32<T>(xr[1]), to_f32<T>(xr[2]), to_f32<T>(xr[3])};
          }
        }
      }
    });
    layer_norm_tile<T, NT_2>(keep2, C, k_o0, k_o0 / (16 * NT_2), k_rt0, k_cnt, stat, p.ln2_g, p.ln2_b, p.ln_eps, Xs, LDX);
  }
  __syncthreads();

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
}

// ------------------------------------------------------------------------------------------
LayerDev to_dev(const dsvt_layer_w& w) {
  LayerDev d;
  d.w_qkv = w.w_qkv; d.w_o = w.w_o; d.w_1 = w.w_1; d.w_2 = w.w_2;
  d.b_qkv = w.b_qkv; d.b_o = w.b_o; d.b_1 = w.b_1; d.b_2 = w.b_2;
  d.ln1_g = w.ln1_g; d.ln1_b = w.ln1_b; d.ln2_g = w.ln2_g; d.ln2_b = w.ln2_b;
  d.rel_bias = w.rel_bias; d.ln_eps = w.ln_eps; d.dup_mode = w.dup_mode;
  const int my = 2 * w.win[1] - 1, mz = 2 * w.win[2] - 1;
  d.rel_my = my; d.rel_mz = mz;
  d.rel_size = (2 * w.win[0] - 1) * my * mz;
  d.rel_const = ((w.win[0] - 1) * my + (w.win[1] - 1)) * mz + (w.win[2] - 1);
  return d;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_layer(const dsvt_layer_w& w, bool need_mlp) {
  if (!w.w_qkv || !w.w_o || !w.b_qkv || !w.b_o) return DSVT_EINVAL;
  if (need_mlp && (!w.w_1 || !w.w_2 || !w.b_1 || !w.b_2 || !w.ln1_g || !w.ln1_b || !w.ln2_g || !w.ln2_b)) return DSVT_EINVAL;
  if (w.dtype != DSVT_F32 && w.dtype != DSVT_BF16) return DSVT_EINVAL;
  if (w.dup_mode != 0 && w.dup_mode != 1) return DSVT_EINVAL;
  for (int a = 0; a < 3; ++a) if (w.win[a] <= 0) return DSVT_EINVAL;
  if (!((w.C == 64 && w.heads == 4 && w.hidden == 128) || (w.C == 192 && w.heads == 8 && w.hidden == 384)))
    return DSVT_EUNSUPPORTED;
  if (w.dtype == DSVT_F32 && w.C != 64) return DSVT_EUNSUPPORTED;   // the fp32 C=192 tiles exceed the 160 KB LDS
  const void* ptrs[] = {w.w_qkv, w.w_o, w.w_1, w.w_2, w.b_qkv, w.b_o, w.b_1, w.b_2, w.ln1_g, w.ln1_b, w.ln2_g, w.ln2_b};
  for (const void* q : ptrs) if (q && !aligned16(q)) return DSVT_EINVAL;
  return DSVT_OK;
}

int check_maps(const dsvt_maps& mp) {
  if (!mp.set_inds || !mp.n_sets || mp.n_voxels <= 0 || mp.max_sets <= 0 || mp.tau <= 0) return DSVT_EINVAL;
  if (mp.tau > kTauMax) return DSVT_EUNSUPPORTED;
  if ((mp.tile_first != nullptr) != (mp.n_tiles != nullptr)) return DSVT_EINVAL;
  if (mp.tile_first != nullptr && mp.max_tiles <= 0) return DSVT_EINVAL;
  return DSVT_OK;
}

template <typename K> int allow_lds(K kernel, size_t bytes) {
  DSVT_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)bytes));
  return DSVT_OK;
}

template <typename T, int C, int HEADS, int HID, int NT_QKV, int NT_O, int NT_1, int NT_2, int KSPLIT_2>
int launch_layer(const dsvt_layer_w& w, const dsvt_maps& mp, const int32_t* coords, const void* x, void* out, int full,
                 hipStream_t st) {
  auto kern = k_layer<T, C, HEADS, HID, NT_QKV, NT_O, NT_1, NT_2, KSPLIT_2>;
  constexpr size_t lds = LayerLds<T, C, HEADS, HID>::total;
  static int prepared = allow_lds(kern, lds);
  if (prepared != DSVT_OK) return prepared;
  MapsDev md;
  md.set_inds = mp.set_inds; md.n_sets = mp.n_sets; md.tile_first = mp.tile_first; md.n_tiles = mp.n_tiles;
  md.max_sets = mp.max_sets; md.tau = mp.tau; md.n_voxels = mp.n_voxels;
  const unsigned grid = mp.tile_first ? (unsigned)mp.max_tiles : (unsigned)dsvt_ceil_div(mp.max_sets, kFixedSets);
  dsvt_prof_scope ps(DSVT_K_LAYER, st);
  kern<<<grid, kWaves * 64, lds, st>>>(to_dev(w), md, reinterpret_cast<const int4*>(coords),
                                       reinterpret_cast<const T*>(x), reinterpret_cast<T*>(out), full);
  return DSVT_OK;
}

int run_layer(const dsvt_layer_w& w, const dsvt_maps& mp, const int32_t* coords, const void* x, void* out, int full,
              hipStream_t st) {
  if (w.dtype == DSVT_BF16) {
    if (w.C == 192) return launch_layer<bf16_t, 192, 8, 384, 3, 3, 3, 3, 2>(w, mp, coords, x, out, full, st);
    return launch_layer<bf16_t, 64, 4, 128, 3, 1, 2, 1, 1>(w, mp, coords, x, out, full, st);
  }
  return launch_layer<float, 64, 4, 128, 3, 1, 2, 1, 1>(w, mp, coords, x, out, full, st);
}

}  // namespace

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
