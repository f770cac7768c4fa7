// MFMA building blocks for gfx950 (64-lane wavefronts).
//
// All dense contractions of the path are skinny GEMMs  Out^T[o][r] = sum_k W[o][k] * X[r][k]:
// the weight matrix W ([out,in], in global memory, cache resident) is the MFMA "A" operand and
// the activations X ([rows, features], staged in LDS) are the "B" operand.  With 16x16 output
// tiles lane l = 16*g + m holds
//     A fragment: row m of the tile, the k-slice owned by lane group g (16 contiguous bytes)
//     B fragment: column m of the tile, the same k-slice                (16 contiguous bytes)
//     accumulator: acc[i] = Out^T[4*g + i][m]  -- four consecutive output features of one row,
// so results go back to a [rows, features] LDS tile with one vector store per lane and can be
// the B operand of the next contraction without a transpose.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct Mma;

// bf16: one v_mfma_f32_16x16x32_bf16 per fragment pair; a lane owns 8 consecutive k.
template <> struct Mma<bf16_t> {
  typedef bf16x8 Frag;
  typedef bf16x4 Vec4;                 // four values = one accumulator's worth, 8 bytes
  static constexpr int KC = 32;        // k extent of a fragment over the whole wavefront
  static constexpr int KL = 8;         // k per lane
  static __device__ __forceinline__ f32x4 mma(Frag a, Frag b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ Frag zero() { Frag z = {0, 0, 0, 0, 0, 0, 0, 0}; return z; }
};

// fp32: four v_mfma_f32_16x16x4_f32 per fragment pair; a lane owns 4 consecutive k and step e of
// the four consumes element e of every lane (the k order inside a fragment is irrelevant as long
// as A and B agree, which they do).
template <> struct Mma<float> {
  typedef f32x4 Frag;
  typedef f32x4 Vec4;
  static constexpr int KC = 16;
  static constexpr int KL = 4;
  static __device__ __forceinline__ f32x4 mma(Frag a, Frag b, f32x4 c) {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], c, 0, 0, 0);
    return c;
  }
  static __device__ __forceinline__ Frag zero() { Frag z = {0.f, 0.f, 0.f, 0.f}; return z; }
};

template <typename T> __device__ __forceinline__ typename Mma<T>::Vec4 pack4(f32x4 v);
template <> __device__ __forceinline__ bf16x4 pack4<bf16_t>(f32x4 v) {
  bf16x4 r = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
  return r;
}
template <> __device__ __forceinline__ f32x4 pack4<float>(f32x4 v) { return v; }

template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }

// threadIdx.x behind an empty asm: values derived from it (lane, row and feature offsets) are
// recomputed where they are used -- a couple of ALU instructions -- instead of being kept in
// registers from the top of a long kernel, where they end up spilled to scratch memory (and a
// reload from scratch waits for every outstanding global load, the weights requested ahead).
__device__ __forceinline__ int opaque_tid() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

// Elements of T that pad every LDS row by 32 bytes.  Rows of K elements (K * sizeof(T) a multiple
// of 64 bytes) then have a pitch that is an odd multiple of 32 bytes, the one pitch at which the
// 16-byte fragment loads of a wavefront (16 rows x 4 k-slices) run at the full LDS rate; measured
// on gfx950: 225 B/clk per CU against 125-150 B/clk for pitches of 16, 48 or 0 mod 64 bytes.
// Declares v defined, with whatever its registers hold and without an instruction.  For variables that are assigned
// on some paths only and read on those paths only: in a loop, the compiler otherwise moves the "undefined" definition
// of the other paths in front of the loop and keeps registers for it through every iteration.
template <typename V> __device__ __forceinline__ void opaque_def(V& v) { asm volatile("" : "=v"(v)); }

template <typename T> constexpr int lds_pad() { return 32 / (int)sizeof(T); }

// Packed weights.  A matrix W [OUT, K] is stored fragment by fragment in the order the MFMA "A"
// operand wants it: fragment (tile, kf) -- output rows 16*tile .. +15, k in [kf*KC, (kf+1)*KC) --
// is 1 KB, lane l's 16 bytes at offset 16*l, fragments ordered [tile][kf].  A wavefront's load of
// one fragment is then one fully coalesced 1 KB read (the [out, in] layout would touch 16 rows
// of 64 bytes each, which the L1/L2 path serves about 3x slower).
template <typename T> __host__ __device__ constexpr size_t packed_elems(int out, int k) { return (size_t)out * k; }

// Workgroup barrier for data exchanged through LDS: waits for this wavefront's LDS operations
// only.  __syncthreads() also drains the outstanding global loads (on this target loads and
// stores share one counter, and its release fence waits for stores), which would turn every
// barrier into a wait for the weight fragments requested ahead for the following phase.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// A-operand fragments of NT output tiles over the whole K, kept in registers: every weight
// fragment is loaded from memory once per workgroup tile and reused for all its rows.
template <typename T, int NT, int NKF> struct AFull { typename Mma<T>::Frag f[NKF][NT]; };
// B-operand fragments of one row tile (16 rows) over the whole K.
template <typename T, int NKF> struct BRow { typename Mma<T>::Frag f[NKF]; };

// Wp: packed matrix with NKF_ALL = K / KC fragments per tile; tiles tile0 .. tile0 + NT - 1,
// k-fragments kf0 .. kf0 + NKF - 1.
template <typename T, int NT, int NKF, int NKF_ALL = NKF>
__device__ __forceinline__ void load_a(AFull<T, NT, NKF>& a, const T* __restrict__ Wp, int tile0, int kf0 = 0) {
  typedef typename Mma<T>::Frag Frag;
  const int lane = opaque_tid() & 63;
  const Frag* fp = reinterpret_cast<const Frag*>(Wp) + ((size_t)tile0 * NKF_ALL + kf0) * 64 + lane;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int kf = 0; kf < NKF; ++kf) a.f[kf][nt] = fp[(nt * NKF_ALL + kf) * 64];
}

// Xs: LDS [rows][ldx]; row tile r, k from k0.
template <typename T, int NKF>
__device__ __forceinline__ void load_b(BRow<T, NKF>& b, const T* Xs, int ldx, int r, int k0 = 0) {
  typedef typename Mma<T>::Frag Frag;
  const int lane = opaque_tid() & 63, m = lane & 15, g = lane >> 4;
  const T* xp = Xs + (16 * r + m) * ldx + k0 + g * Mma<T>::KL;
#pragma unroll
  for (int kf = 0; kf < NKF; ++kf) b.f[kf] = *reinterpret_cast<const Frag*>(xp + kf * Mma<T>::KC);
}

template <typename T, int NT, int NKF>
__device__ __forceinline__ void mma_row(f32x4 (&acc)[NT], const AFull<T, NT, NKF>& a, const BRow<T, NKF>& b) {
#pragma unroll
  for (int kf = 0; kf < NKF; ++kf)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = Mma<T>::mma(a.f[kf][nt], b.f[kf], acc[nt]);
}

// Operands exchanged: the activations are the MFMA "A" operand and the weights "B" (their fragment
// layouts are identical), so acc[nt][i] = Out[row 4*g + i][feature 16*nt + m]: a lane holds four
// consecutive ROWS of one feature -- what a transposed store of the result wants.
template <typename T, int NT, int NKF>
__device__ __forceinline__ void mma_row_swapped(f32x4 (&acc)[NT], const AFull<T, NT, NKF>& a, const BRow<T, NKF>& b) {
#pragma unroll
  for (int kf = 0; kf < NKF; ++kf)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = Mma<T>::mma(b.f[kf], a.f[kf][nt], acc[nt]);
}

constexpr int kRowTiles = 6;                     // row tiles of a workgroup tile
constexpr int kRowsMax = 16 * kRowTiles;         // 96 rows
constexpr int kWaves = 8;                        // wavefronts of a pooling workgroup, two per SIMD
constexpr int kStatGroupsMax = 6;                // LayerNorm phases: the C features are split over at most 6 groups of output tiles

// One GEMM phase of a workgroup of NW wavefronts: Out^T[NOUT x rows] = W[NOUT x K] . X^T.
// A work item is a group of NT output tiles over all row tiles (RSPLIT = 1) or over one half of
// them (RSPLIT = 2, for workgroups with two wavefronts per SIMD); wavefront w takes items
// w, w + NW, ...  An item's weight fragments sit in registers for the whole item, the next item's
// are requested before the current one is consumed, and inside an item the activations of row
// tile r + 1 are read from LDS while row tile r is in the matrix cores.  Every activation
// fragment read from LDS feeds NT MFMAs; a weight fragment is loaded by RSPLIT wavefronts.
template <typename T, int NT, int K, int NOUT, int NW, int RSPLIT = 1, bool DOUBLE_A = true, int KSPLIT = 1>
struct GemmPhase {
  static constexpr int KC = Mma<T>::KC;
  static constexpr int NKF_ALL = K / KC;
  static constexpr int NKF = NKF_ALL / KSPLIT;          // fragments held at a time (KSPLIT > 1: run_keep only)
  static constexpr int N_OG = NOUT / (16 * NT);
  static constexpr int N_ITEMS = RSPLIT * N_OG;
  static constexpr int IPW = (N_ITEMS + NW - 1) / NW;   // items per wavefront (the last round may be partial)
  static constexpr int RH = kRowTiles / RSPLIT;          // row tiles an item can cover
  static_assert(K % KC == 0 && NOUT % (16 * NT) == 0 && (RSPLIT == 1 || RSPLIT == 2), "phase shape");
  AFull<T, NT, NKF> a[(IPW > 1 && DOUBLE_A) ? 2 : 1];   // DOUBLE_A: the next item's weights load during the current item
  const T* Wp;
  int wave;
  struct Bias { f32x4 v[NT]; float s[NT]; };          // both forms of an item's bias, see load_bias()
  Bias bias0;                                            // first item's bias when prefetch() fetched it
  bool bias0_set = false;

  __device__ __forceinline__ GemmPhase(const T* wp, int wave_) : Wp(wp), wave(wave_) {}

  // In a loop that requests the weights anew in every trip: called at the top of the trip, it ends the life of the
  // weight registers of the trip before (see opaque_def).
  __device__ __forceinline__ void forget() {
#pragma unroll
    for (int k = 0; k < (int)(sizeof(a) / sizeof(a[0])); ++k)
#pragma unroll
      for (int kf = 0; kf < NKF; ++kf)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) opaque_def(a[k].f[kf][nt]);
  }

  // Request the weights of this wavefront's first item (may be called long before run()), and
  // with them, if given, the bias run() starts that item from.
  __device__ __forceinline__ void prefetch(const float* __restrict__ bias = nullptr, int swap_og = N_OG) {
    if (N_ITEMS >= NW || wave < N_ITEMS) {
      load_a<T, NT, NKF, NKF_ALL>(a[0], Wp, (wave % N_OG) * NT);
      if (bias != nullptr) { load_bias(bias0, bias, wave % N_OG, swap_og < N_OG); bias0_set = true; }
    }
  }

  // Accumulator start values of output group og: feature 16*nt + 4*g + i for element i, or, with
  // exchanged operands, feature 16*nt + m for all four.  Both forms are loaded (no branch, no
  // wait at the point of the request) and select() picks one when the item starts.
  __device__ __forceinline__ void load_bias(Bias& b, const float* __restrict__ bias, int og, bool need_s) const {
    const int tl = opaque_tid(), lane16 = tl & 15, g4 = ((tl & 63) >> 4) * 4;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      b.v[nt] = *reinterpret_cast<const f32x4*>(bias + og * 16 * NT + 16 * nt + g4);
      b.s[nt] = need_s ? bias[og * 16 * NT + 16 * nt + lane16] : 0.f;
    }
  }
  static __device__ __forceinline__ void select_bias(f32x4 (&b4)[NT], const Bias& b, bool sw) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) b4[nt] = sw ? f32x4{b.s[nt], b.s[nt], b.s[nt], b.s[nt]} : b.v[nt];
  }

  // Row tiles in a rolled loop, two per trip.  epi(o0, r, acc, swapped): acc[nt][i] is output
  // feature o0 + 16*nt + 4*g + i of row 16*r + m, bias included -- or, for the items whose output
  // group is >= swap_og ("swapped": operands exchanged), feature o0 + 16*nt + m of row
  // 16*r + 4*g + i.  The bias is fetched before the next item's weights are requested, so waiting
  // for it never waits for them.
  template <typename Epi>
  __device__ __forceinline__ void run(const T* Xs, int ldx, int RT, const float* __restrict__ bias, Epi epi, int swap_og = N_OG) {
    static_assert(KSPLIT == 1, "run() holds the whole K");
    const int h0 = RSPLIT == 1 ? RT : (RT + 1) >> 1;
#pragma unroll
    for (int it = 0; it < IPW; ++it) {
      const int item = wave + it * NW;
      if (item >= N_ITEMS) break;
      const int og = item % N_OG, half = item / N_OG;
      const int rt0 = half ? h0 : 0, cnt = half ? RT - h0 : h0;
      const bool sw = og >= swap_og;                 // wave-uniform
      f32x4 b4[NT];
      if (it == 0 && bias0_set) {
        select_bias(b4, bias0, sw);
      } else {
        Bias bl;
        load_bias(bl, bias, og, swap_og < N_OG);
        select_bias(b4, bl, sw);
      }
      if (DOUBLE_A && it + 1 < IPW && item + NW < N_ITEMS) load_a<T, NT, NKF>(a[(it + 1) & 1], Wp, ((item + NW) % N_OG) * NT);
      const AFull<T, NT, NKF>& A = a[DOUBLE_A ? (it & 1) : 0];
      if constexpr (DOUBLE_A && RSPLIT == 2) {
        // two wavefronts per SIMD: the other one covers the LDS latency, so one row tile at a
        // time keeps the registers for the second weight buffer
        for (int r = 0; r < cnt; ++r) {
          BRow<T, NKF> b0;
          load_b<T, NKF>(b0, Xs, ldx, rt0 + r);
          f32x4 acc0[NT];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) acc0[nt] = b4[nt];
          if (sw) mma_row_swapped<T, NT, NKF>(acc0, A, b0); else mma_row<T, NT, NKF>(acc0, A, b0);
          epi(og * 16 * NT, rt0 + r, acc0, sw);
        }
      } else {
        BRow<T, NKF> b0, b1;
        if (cnt > 0) load_b<T, NKF>(b0, Xs, ldx, rt0);
        for (int r = 0; r < cnt; r += 2) {
          const bool two = r + 1 < cnt;
          if (two) load_b<T, NKF>(b1, Xs, ldx, rt0 + r + 1);
          f32x4 acc0[NT], acc1[NT];              // the bias is the accumulators' initial value
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) { acc0[nt] = b4[nt]; acc1[nt] = b4[nt]; }
          if (sw) mma_row_swapped<T, NT, NKF>(acc0, A, b0); else mma_row<T, NT, NKF>(acc0, A, b0);
          if (two) {
            if (r + 2 < cnt) load_b<T, NKF>(b0, Xs, ldx, rt0 + r + 2);
            if (sw) mma_row_swapped<T, NT, NKF>(acc1, A, b1); else mma_row<T, NT, NKF>(acc1, A, b1);
          }
          epi(og * 16 * NT, rt0 + r, acc0, sw);
          if (two) epi(og * 16 * NT, rt0 + r + 1, acc1, sw);
        }
      }
      if (!DOUBLE_A && it + 1 < IPW && item + NW < N_ITEMS) load_a<T, NT, NKF>(a[0], Wp, ((item + NW) % N_OG) * NT);
    }
  }

  // One item per wavefront: row tiles rt0 .. rt0 + HC - 1 unrolled, all accumulators returned
  // (the LayerNorm phases need a row's values in registers across a workgroup barrier).  With
  // KSPLIT > 1 the weights pass through the registers one K-slice at a time.
  template <int HC>
  __device__ __forceinline__ void run_keep(const T* Xs, int ldx, int rt0, const f32x4 (&b4)[NT], f32x4 (&acc)[NT][RH]) {
    static_assert(IPW == 1 && HC <= RH, "one item per wavefront");
    if (wave >= N_ITEMS) return;                       // wavefronts beyond the items only take part in the barriers
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int r = 0; r < HC; ++r) acc[nt][r] = b4[nt];
#pragma unroll
    for (int ks = 0; ks < KSPLIT; ++ks) {
      if (ks > 0) load_a<T, NT, NKF, NKF_ALL>(a[0], Wp, (wave % N_OG) * NT, ks * NKF);
      BRow<T, NKF> b[2];
      load_b<T, NKF>(b[0], Xs, ldx, rt0, ks * NKF * KC);
#pragma unroll
      for (int r = 0; r < HC; ++r) {
        if (r + 1 < HC) load_b<T, NKF>(b[(r + 1) & 1], Xs, ldx, rt0 + r + 1, ks * NKF * KC);
        f32x4 t[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) t[nt] = acc[nt][r];
        mma_row<T, NT, NKF>(t, a[0], b[r & 1]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt][r] = t[nt];
      }
    }
  }
};

template <int NT, int RT_MAX> __device__ __forceinline__ void zero_acc(f32x4 (&acc)[NT][RT_MAX]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int rt = 0; rt < RT_MAX; ++rt) acc[nt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// Reductions over the four lanes m, m + 16, m + 32, m + 48 (one accumulator column) with the
// gfx950 lane-swap instructions: permlane16_swap(x, x) returns x's 16-lane rows (0,0,2,2) and
// (1,1,3,3), permlane32_swap(x, x) its halves (lo,lo) and (hi,hi); no LDS round trip.
__device__ __forceinline__ float col_sum(float v) {
  const unsigned u = __float_as_uint(v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float s = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const unsigned w = __float_as_uint(s);
  const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
// (the maxima are taken by the instruction itself: fmaxf() on values that come out of a lane swap as plain bits
// is compiled with an extra quieting operation per operand)
__device__ __forceinline__ float raw_max(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float col_max(float v) {
  const unsigned u = __float_as_uint(v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float s = raw_max(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const unsigned w = __float_as_uint(s);
  const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return raw_max(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

// erf-GELU, x * Phi(x) = 0.5 x (1 + erf(x / sqrt 2)), with erf(z) = 1 - 1 / p(z)^(2^n) from
// Abramowitz & Stegun: 7.1.28 (six coefficients, ^16, |error| <= 3e-7) for fp32 features, 7.1.27
// (four coefficients, ^4, |error| <= 5e-4, below bf16 resolution) for bf16 features.
// 0.5 x + 0.5 |x| erf(|x|/sqrt 2) = max(x, 0) - |x| / (2 p^(2^n)); the polynomial is taken in
// a = |x| directly, q(a) = 2^(1/2^n) p(a / sqrt 2), so that q^(2^n) = 2 p^(2^n).
template <int POW_LOG2> constexpr double gelu_coef(double c, int deg) {
  double r = c;
  for (int i = 0; i < deg; ++i) r *= 0.70710678118654752440;              // (1 / sqrt 2)^deg
  double root = 2.0;                                                        // 2^(1 / 2^POW_LOG2)
  for (int i = 0; i < POW_LOG2; ++i) {                                      // Newton square roots, constexpr-friendly
    double y = root > 1.0 ? root : 1.0;
    for (int k = 0; k < 60; ++k) y = 0.5 * (y + root / y);
    root = y;
  }
  return r * root;
}
template <typename T> __device__ __forceinline__ float gelu_erf_fast(float x);
template <> __device__ __forceinline__ float gelu_erf_fast<float>(float x) {
  constexpr float k0 = (float)gelu_coef<4>(1.0, 0), k1 = (float)gelu_coef<4>(0.0705230784, 1),
                  k2 = (float)gelu_coef<4>(0.0422820123, 2), k3 = (float)gelu_coef<4>(0.0092705272, 3),
                  k4 = (float)gelu_coef<4>(0.0001520143, 4), k5 = (float)gelu_coef<4>(0.0002765672, 5),
                  k6 = (float)gelu_coef<4>(0.0000430638, 6);
  const float a = fabsf(x);
  float q = fmaf(k6, a, k5);
  q = fmaf(q, a, k4);
  q = fmaf(q, a, k3);
  q = fmaf(q, a, k2);
  q = fmaf(q, a, k1);
  q = fmaf(q, a, k0);
  q = q * q; q = q * q; q = q * q; q = q * q;
  return fmaf(-a, __builtin_amdgcn_rcpf(q), fmaxf(x, 0.f));
}
template <> __device__ __forceinline__ float gelu_erf_fast<bf16_t>(float x) {
  constexpr float k0 = (float)gelu_coef<2>(1.0, 0), k1 = (float)gelu_coef<2>(0.278393, 1),
                  k2 = (float)gelu_coef<2>(0.230389, 2), k3 = (float)gelu_coef<2>(0.000972, 3),
                  k4 = (float)gelu_coef<2>(0.078108, 4);
  const float a = fabsf(x);
  float q = fmaf(k4, a, k3);
  q = fmaf(q, a, k2);
  q = fmaf(q, a, k1);
  q = fmaf(q, a, k0);
  q = q * q; q = q * q;
  return fmaf(-a, __builtin_amdgcn_rcpf(q), fmaxf(x, 0.f));
}

// LayerNorm over the C features of every row, for values spread over the workgroup in
// accumulator layout: this wavefront holds features o0 .. o0 + 16*NT - 1 (group og of
// SG = C / (16*NT)) of rows 16*(rt0 + r) + m, r < cnt (cnt = 0: only the barrier).  Per-group sums of x and x^2 (fp32) are
// exchanged through LDS; variance = E[x^2] - mean^2.  Every thread of the workgroup must call it.
template <typename T, int NT, int C, int RH>
__device__ __forceinline__ void layer_norm_tile(f32x4 (&v)[NT][RH], int o0, int og, int rt0, int cnt, float* stat,
                                                const f32x4 (&ga)[NT], const f32x4 (&be)[NT], float eps, T* dst,
                                                int ldd) {
  typedef typename Mma<T>::Vec4 Vec4;
  constexpr int SG = C / (16 * NT);
  static_assert(SG * 16 * NT == C && SG <= kStatGroupsMax, "LayerNorm feature groups");
  const int lane = opaque_tid() & 63, m = lane & 15, g = lane >> 4;
  float* stat1 = stat;
  float* stat2 = stat + kStatGroupsMax * kRowsMax;
#pragma unroll
  for (int r = 0; r < RH; ++r) {
    if (r < cnt) {
      float s = 0.f, q = 0.f;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { s += v[nt][r][i]; q = fmaf(v[nt][r][i], v[nt][r][i], q); }
      }
      s = col_sum(s);
      q = col_sum(q);
      if (g == 0) { stat1[og * kRowsMax + 16 * (rt0 + r) + m] = s; stat2[og * kRowsMax + 16 * (rt0 + r) + m] = q; }
    }
  }
  lds_barrier();
#pragma unroll
  for (int r = 0; r < RH; ++r) {
    if (r < cnt) {
      const int row = 16 * (rt0 + r) + m;
      float s = 0.f, q = 0.f;
#pragma unroll
      for (int k = 0; k < SG; ++k) { s += stat1[k * kRowsMax + row]; q += stat2[k * kRowsMax + row]; }
      const float mean = s * (1.0f / C);
      const float rs = __builtin_amdgcn_rsqf(fmaxf(fmaf(-mean, mean, q * (1.0f / C)), 0.f) + eps);
      const float sh = -mean * rs;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int o = o0 + 16 * nt + 4 * g;
        f32x4 y;
#pragma unroll
        for (int i = 0; i < 4; ++i) y[i] = fmaf(fmaf(v[nt][r][i], rs, sh), ga[nt][i], be[nt][i]);
        *reinterpret_cast<Vec4*>(dst + row * ldd + o) = pack4<T>(y);
      }
    }
  }
}

// dst fragment order <- src [out, in]; one thread per 16-byte lane slot.
template <typename T>
__global__ void k_pack(const T* __restrict__ src, T* __restrict__ dst, int out, int k) {
  constexpr int KC = Mma<T>::KC, KL = Mma<T>::KL;
  const int nkf = k / KC;
  const long long slot = (long long)blockIdx.x * blockDim.x + threadIdx.x;     // (tile, kf, lane)
  if (slot >= (long long)(out / 16) * nkf * 64) return;
  const int lane = (int)(slot & 63), kf = (int)((slot >> 6) % nkf), tile = (int)((slot >> 6) / nkf);
  const T* s = src + (size_t)(tile * 16 + (lane & 15)) * k + kf * KC + (lane >> 4) * KL;
  T* d = dst + (size_t)slot * KL;
#pragma unroll
  for (int e = 0; e < KL; ++e) d[e] = s[e];
}

