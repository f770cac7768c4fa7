// dsvt_set_attention / dsvt_block: one DSVT layer on gfx950 (Sec. 3.2 Eq. 4-5; appendix
// "Network Architecture").
//
// k_set_attention: a workgroup owns SETS_PER_WG consecutive sets.  It reads their slot rows of
// set_inds, keeps the first occurrence of every voxel (repeats are adjacent, Eq. 3 is monotone),
// and gathers those voxels' features into an LDS tile -- the tau x C tile of Eq. (4) with the
// repeated rows squeezed out, since a masked repeat contributes nothing as a key and its query
// row would be thrown away.  Q/K/V projection, per-(set, head) softmax(QK^T + PE)V, the output
// projection, the residual and LayerNorm all run on that tile; the result rows go straight back
// to the voxels' rows of the output (every voxel is in exactly one set, Thm A.2-A.3).
// k_ffn: row tiles of LN(x + W2 gelu(W1 x + b1) + b2).
#include "common.h"
#include "mma.h"

namespace {

constexpr int kSetsPerWg = 2;
constexpr int kTauMax = 48;
constexpr int kRowsMax = kSetsPerWg * kTauMax;   // 96 rows = 6 MFMA row tiles
constexpr int kRtMax = kRowsMax / 16;
constexpr int kKeyTiles = kTauMax / 16;          // 3

struct LayerDev {
  const void *w_qkv, *w_o, *w_1, *w_2;
  const float *b_qkv, *b_o, *b_1, *b_2, *ln1_g, *ln1_b, *ln2_g, *ln2_b, *rel_bias;
  float ln_eps;
  int rel_size, rel_const, rel_my, rel_mz;   // table entries per head; index = lin(q) - lin(k) + rel_const
  int dup_mode;
};

template <typename T, int C, int HEADS> struct AttnLds {
  static constexpr int D = C / HEADS;
  static constexpr int PAD = lds_pad<T>();
  static constexpr int LDX = C + PAD;            // pitch of [row][feature] tiles, elements of T
  static constexpr int LDV = kRowsMax + PAD;     // pitch of V^T [feature][row]
  static constexpr int LDY = C + 4;              // pitch of the fp32 staging tile
  static constexpr size_t kTile = (size_t)kRowsMax * LDX * sizeof(T);
  static constexpr size_t off_x = 0, off_q = kTile, off_k = 2 * kTile, off_v = 3 * kTile;
  static constexpr size_t kVt = (size_t)C * LDV * sizeof(T);
  static constexpr size_t off_y = off_k;         // fp32 staging reuses K and V^T once attention is done
  static constexpr size_t off_misc = off_v + kVt;
  static constexpr size_t kMisc = (size_t)(kSetsPerWg * kTauMax + 3 * kRowsMax + 2 * kSetsPerWg + 2) * 4;
  static constexpr size_t total = off_misc + kMisc;
  static_assert((size_t)kRowsMax * LDY * 4 <= kTile + kVt, "fp32 staging must fit in K + V^T");
  static_assert(C % 64 == 0 && D % Mma<T>::KL == 0 && D % 4 == 0, "shape");
};

template <typename T, int C, int HEADS, int NW, int NT_QKV, int NT_O>
__global__ void __launch_bounds__(NW * 64)
k_set_attention(LayerDev p, const int32_t* __restrict__ set_inds, const int32_t* __restrict__ n_sets_ptr,
                int32_t max_sets, int32_t tau, int32_t n_voxels, const int4* __restrict__ coords,
                const T* x, T* out, int full_layer) {   // out may be x (rows are read, then written, by one workgroup)
  typedef AttnLds<T, C, HEADS> L;
  typedef Mma<T> M;
  typedef typename M::Frag Frag;
  typedef typename M::Vec4 Vec4;
  constexpr int D = L::D, LDX = L::LDX, LDV = L::LDV, LDY = L::LDY, KC = M::KC, KL = M::KL;
  constexpr int NTHREADS = NW * 64;
  extern __shared__ __align__(16) unsigned char smem[];
  T* Xs = reinterpret_cast<T*>(smem + L::off_x);
  T* Qs = reinterpret_cast<T*>(smem + L::off_q);
  T* Ks = reinterpret_cast<T*>(smem + L::off_k);
  T* Vt = reinterpret_cast<T*>(smem + L::off_v);
  float* Yf = reinterpret_cast<float*>(smem + L::off_y);
  int32_t* inds = reinterpret_cast<int32_t*>(smem + L::off_misc);
  int32_t* row_vox = inds + kSetsPerWg * kTauMax;
  int32_t* row_lin = row_vox + kRowsMax;
  float* row_mult = reinterpret_cast<float*>(row_lin + kRowsMax);
  int32_t* set_r0 = reinterpret_cast<int32_t*>(row_mult + kRowsMax);   // [kSetsPerWg + 1]
  int32_t* set_nu = set_r0 + kSetsPerWg + 1;                            // [kSetsPerWg]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, m = lane & 15, g = lane >> 4;
  int n_sets = *n_sets_ptr;
  n_sets = n_sets < max_sets ? n_sets : max_sets;
  const int s_base = blockIdx.x * kSetsPerWg;
  const int ns = (n_sets - s_base) < kSetsPerWg ? (n_sets - s_base) : kSetsPerWg;
  if (ns <= 0) return;

  // ---- 1. slots -> compact rows (first occurrences only; each set starts on a multiple of 4 rows)
  for (int r = tid; r < kRowsMax; r += NTHREADS) { row_vox[r] = -1; row_lin[r] = 0; row_mult[r] = 0.f; }
  const int nslots = ns * tau;
  if (tid < nslots) inds[tid] = set_inds[(size_t)s_base * tau + tid];
  __syncthreads();
  int my_set = 0, my_rank = 0, my_mult = 0, my_v = -1;
  bool my_first = false;
  if (tid < nslots) {
    my_set = tid / tau;
    const int k = tid - my_set * tau;
    const int32_t* row = inds + my_set * tau;
    my_v = row[k];
    my_first = (k == 0) || (row[k - 1] != my_v);
    for (int k2 = 0; k2 < tau; ++k2) {
      const int u = row[k2];
      const bool f2 = (k2 == 0) || (row[k2 - 1] != u);
      my_rank += (k2 < k && f2) ? 1 : 0;
      my_mult += (u == my_v) ? 1 : 0;
    }
    if (k == tau - 1) set_nu[my_set] = my_rank + (my_first ? 1 : 0);
  }
  __syncthreads();
  if (tid == 0) {
    int r = 0;
    for (int s = 0; s < ns; ++s) { set_r0[s] = r; r += (set_nu[s] + 3) & ~3; }
    set_r0[ns] = r;
  }
  __syncthreads();
  if (tid < nslots && my_first && my_v >= 0 && my_v < n_voxels) {
    const int r = set_r0[my_set] + my_rank;
    const int4 c = coords[my_v];
    row_vox[r] = my_v;
    row_mult[r] = (float)my_mult;
    row_lin[r] = (c.y * p.rel_my + c.z) * p.rel_mz + c.w;
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
    const T* W = reinterpret_cast<const T*>(p.w_qkv);
    for (int og = wave; og < 3 * C / (16 * NT_QKV); og += NW) {
      const int o0 = og * 16 * NT_QKV;
      f32x4 acc[NT_QKV][kRtMax];
      zero_acc(acc);
      gemm_wx<T, NT_QKV, kRtMax>(W, C, o0, Xs, LDX, C, RT, acc);
#pragma unroll
      for (int nt = 0; nt < NT_QKV; ++nt) {
        const int ot = o0 + 16 * nt;             // tile never straddles the Q/K/V boundary (C % 16 == 0)
        const int o = ot + 4 * g;
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.b_qkv + o);
        const int sel = ot / C;
#pragma unroll
        for (int rt = 0; rt < kRtMax; ++rt) {
          if (rt < RT) {
            const int row = 16 * rt + m;
            f32x4 v = acc[nt][rt] + b4;
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
    }
  }
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

  // ---- 5. Y = O Wo^T + bo (+ x), staged in fp32 over the dead K / V^T tiles
  {
    const T* W = reinterpret_cast<const T*>(p.w_o);
    for (int og = wave; og < C / (16 * NT_O); og += NW) {
      const int o0 = og * 16 * NT_O;
      f32x4 acc[NT_O][kRtMax];
      zero_acc(acc);
      gemm_wx<T, NT_O, kRtMax>(W, C, o0, Qs, LDX, C, RT, acc);
#pragma unroll
      for (int nt = 0; nt < NT_O; ++nt) {
        const int o = o0 + 16 * nt + 4 * g;
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.b_o + o);
#pragma unroll
        for (int rt = 0; rt < kRtMax; ++rt) {
          if (rt < RT) {
            const int row = 16 * rt + m;
            f32x4 v = acc[nt][rt] + b4;
            if (full_layer) {
              const Vec4 xr = *reinterpret_cast<const Vec4*>(Xs + row * LDX + o);
              v += f32x4{to_f32<T>(xr[0]), to_f32<T>(xr[1]), to_f32<T>(xr[2]), to_f32<T>(xr[3])};
            }
            *reinterpret_cast<f32x4*>(Yf + row * LDY + o) = v;
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- 6. LayerNorm per row and scatter back to the voxel's row
  for (int r = wave; r < R; r += NW) {
    const int v = row_vox[r];
    if (v < 0) continue;
    float vals[C / 64];
    float s1 = 0.f;
#pragma unroll
    for (int j = 0; j < C / 64; ++j) { vals[j] = Yf[r * LDY + lane + 64 * j]; s1 += vals[j]; }
    if (full_layer) {
      const float mean = wave_sum(s1) * (1.0f / C);
      float s2 = 0.f;
#pragma unroll
      for (int j = 0; j < C / 64; ++j) { vals[j] -= mean; s2 += vals[j] * vals[j]; }
      const float rs = rsqrtf(wave_sum(s2) * (1.0f / C) + p.ln_eps);
#pragma unroll
      for (int j = 0; j < C / 64; ++j) vals[j] = vals[j] * rs * p.ln1_g[lane + 64 * j] + p.ln1_b[lane + 64 * j];
    }
#pragma unroll
    for (int j = 0; j < C / 64; ++j) out[(size_t)v * C + lane + 64 * j] = (T)vals[j];
  }
}

// ------------------------------------------------------------------------------------------
constexpr int kFfnRows = 64;

template <typename T, int C, int HID> struct FfnLds {
  static constexpr int PAD = lds_pad<T>();
  static constexpr int LDX = C + PAD, LDH = HID + PAD, LDY = C + 4;
  static constexpr size_t off_x = 0;
  static constexpr size_t off_h = off_x + (size_t)kFfnRows * LDX * sizeof(T);
  static constexpr size_t off_y = off_h + (size_t)kFfnRows * LDH * sizeof(T);
  static constexpr size_t total = off_y + (size_t)kFfnRows * LDY * 4;
};

template <typename T, int C, int HID, int NW, int NT_1, int NT_2>
__global__ void __launch_bounds__(NW * 64)
k_ffn(LayerDev p, const T* x1, T* out, int32_t n) {   // out may be x1
  typedef FfnLds<T, C, HID> L;
  typedef typename Mma<T>::Vec4 Vec4;
  constexpr int LDX = L::LDX, LDH = L::LDH, LDY = L::LDY, RT = kFfnRows / 16, NTHREADS = NW * 64;
  extern __shared__ __align__(16) unsigned char smem[];
  T* Xs = reinterpret_cast<T*>(smem + L::off_x);
  T* Hs = reinterpret_cast<T*>(smem + L::off_h);
  float* Yf = reinterpret_cast<float*>(smem + L::off_y);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, m = lane & 15, g = lane >> 4;
  const int row0 = blockIdx.x * kFfnRows;
  {
    constexpr int CH = C * (int)sizeof(T) / 16;
    for (int idx = tid; idx < kFfnRows * CH; idx += NTHREADS) {
      const int r = idx / CH, c = idx - r * CH;
      uint4 val = make_uint4(0u, 0u, 0u, 0u);
      if (row0 + r < n) val = reinterpret_cast<const uint4*>(x1 + (size_t)(row0 + r) * C)[c];
      *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(Xs) + (size_t)r * LDX * sizeof(T) + c * 16) = val;
    }
  }
  __syncthreads();
  {
    const T* W = reinterpret_cast<const T*>(p.w_1);
    for (int og = wave; og < HID / (16 * NT_1); og += NW) {
      const int o0 = og * 16 * NT_1;
      f32x4 acc[NT_1][RT];
      zero_acc(acc);
      gemm_wx<T, NT_1, RT>(W, C, o0, Xs, LDX, C, RT, acc);
#pragma unroll
      for (int nt = 0; nt < NT_1; ++nt) {
        const int o = o0 + 16 * nt + 4 * g;
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.b_1 + o);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          f32x4 v = acc[nt][rt] + b4;
          v = f32x4{gelu_erf(v[0]), gelu_erf(v[1]), gelu_erf(v[2]), gelu_erf(v[3])};
          *reinterpret_cast<Vec4*>(Hs + (16 * rt + m) * LDH + o) = pack4<T>(v);
        }
      }
    }
  }
  __syncthreads();
  {
    const T* W = reinterpret_cast<const T*>(p.w_2);
    for (int og = wave; og < C / (16 * NT_2); og += NW) {
      const int o0 = og * 16 * NT_2;
      f32x4 acc[NT_2][RT];
      zero_acc(acc);
      gemm_wx<T, NT_2, RT>(W, HID, o0, Hs, LDH, HID, RT, acc);
#pragma unroll
      for (int nt = 0; nt < NT_2; ++nt) {
        const int o = o0 + 16 * nt + 4 * g;
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.b_2 + o);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          const int row = 16 * rt + m;
          const Vec4 xr = *reinterpret_cast<const Vec4*>(Xs + row * LDX + o);
          f32x4 v = acc[nt][rt] + b4 + f32x4{to_f32<T>(xr[0]), to_f32<T>(xr[1]), to_f32<T>(xr[2]), to_f32<T>(xr[3])};
          *reinterpret_cast<f32x4*>(Yf + row * LDY + o) = v;
        }
      }
    }
  }
  __syncthreads();
  for (int r = wave; r < kFfnRows; r += NW) {
    if (row0 + r >= n) break;
    float vals[C / 64];
    float s1 = 0.f;
#pragma unroll
    for (int j = 0; j < C / 64; ++j) { vals[j] = Yf[r * LDY + lane + 64 * j]; s1 += vals[j]; }
    const float mean = wave_sum(s1) * (1.0f / C);
    float s2 = 0.f;
#pragma unroll
    for (int j = 0; j < C / 64; ++j) { vals[j] -= mean; s2 += vals[j] * vals[j]; }
    const float rs = rsqrtf(wave_sum(s2) * (1.0f / C) + p.ln_eps);
#pragma unroll
    for (int j = 0; j < C / 64; ++j)
      out[(size_t)(row0 + r) * C + lane + 64 * j] = (T)(vals[j] * rs * p.ln2_g[lane + 64 * j] + p.ln2_b[lane + 64 * j]);
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
  const void* ptrs[] = {w.w_qkv, w.w_o, w.w_1, w.w_2, w.b_qkv, w.b_o, w.b_1, w.b_2};
  for (const void* q : ptrs) if (q && !aligned16(q)) return DSVT_EINVAL;
  return DSVT_OK;
}

int check_maps(const dsvt_maps& mp) {
  if (!mp.set_inds || !mp.n_sets || mp.n_voxels <= 0 || mp.max_sets <= 0 || mp.tau <= 0) return DSVT_EINVAL;
  if (mp.tau > kTauMax) return DSVT_EUNSUPPORTED;
  return DSVT_OK;
}

template <typename K> int allow_lds(K kernel, size_t bytes) {
  DSVT_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)bytes));
  return DSVT_OK;
}

constexpr int kAttnWaves = 4, kFfnWaves = 4;

template <typename T, int C, int HEADS, int NT_QKV, int NT_O>
int launch_attention(const dsvt_layer_w& w, const dsvt_maps& mp, const int32_t* coords, const void* x, void* out,
                     int full, hipStream_t st) {
  auto kern = k_set_attention<T, C, HEADS, kAttnWaves, NT_QKV, NT_O>;
  constexpr size_t lds = AttnLds<T, C, HEADS>::total;
  static int prepared = allow_lds(kern, lds);
  if (prepared != DSVT_OK) return prepared;
  const unsigned grid = (unsigned)dsvt_ceil_div(mp.max_sets, kSetsPerWg);
  dsvt_prof_scope ps(DSVT_K_ATTN, st);
  kern<<<grid, kAttnWaves * 64, lds, st>>>(to_dev(w), mp.set_inds, mp.n_sets, mp.max_sets, mp.tau, mp.n_voxels,
                                           reinterpret_cast<const int4*>(coords), reinterpret_cast<const T*>(x),
                                           reinterpret_cast<T*>(out), full);
  return DSVT_OK;
}

template <typename T, int C, int HID, int NT_1, int NT_2>
int launch_ffn(const dsvt_layer_w& w, const void* x1, void* out, int32_t n, hipStream_t st) {
  auto kern = k_ffn<T, C, HID, kFfnWaves, NT_1, NT_2>;
  constexpr size_t lds = FfnLds<T, C, HID>::total;
  static int prepared = allow_lds(kern, lds);
  if (prepared != DSVT_OK) return prepared;
  dsvt_prof_scope ps(DSVT_K_FFN, st);
  kern<<<(unsigned)dsvt_ceil_div(n, kFfnRows), kFfnWaves * 64, lds, st>>>(to_dev(w), reinterpret_cast<const T*>(x1),
                                                                         reinterpret_cast<T*>(out), n);
  return DSVT_OK;
}

int run_attention(const dsvt_layer_w& w, const dsvt_maps& mp, const int32_t* coords, const void* x, void* out, int full,
                  hipStream_t st) {
  if (w.dtype == DSVT_BF16) {
    if (w.C == 192) return launch_attention<bf16_t, 192, 8, 3, 3>(w, mp, coords, x, out, full, st);
    return launch_attention<bf16_t, 64, 4, 3, 1>(w, mp, coords, x, out, full, st);
  }
  return launch_attention<float, 64, 4, 3, 1>(w, mp, coords, x, out, full, st);
}

int run_ffn(const dsvt_layer_w& w, const void* x1, void* out, int32_t n, hipStream_t st) {
  if (w.dtype == DSVT_BF16) {
    if (w.C == 192) return launch_ffn<bf16_t, 192, 384, 3, 3>(w, x1, out, n, st);
    return launch_ffn<bf16_t, 64, 128, 2, 1>(w, x1, out, n, st);
  }
  return launch_ffn<float, 64, 128, 2, 1>(w, x1, out, n, st);
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
  rc = run_attention(*layer, *maps, coords, x, y, 0, (hipStream_t)stream);
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
    // A set's workgroup reads its voxels' rows before it writes them and no other workgroup
    // touches those rows, so the attention half may run in place; so may the row-tiled FFN.
    int rc = run_attention(layer[l], maps[l], coords, src, x_out, 1, st);
    if (rc != DSVT_OK) return rc;
    rc = run_ffn(layer[l], x_out, x_out, maps[l].n_voxels, st);
    if (rc != DSVT_OK) return rc;
    src = x_out;
  }
  DSVT_HIP_TRY(hipGetLastError());
  return DSVT_OK;
}
