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

// Elements of T that pad every LDS row by 16 bytes, so that the 16 rows a fragment load touches
// start in different banks.
template <typename T> constexpr int lds_pad() { return 16 / (int)sizeof(T); }

// A-operand fragments of NT output tiles over KF consecutive k-fragments, kept in registers so
// that all of a tile group's weight loads are in flight at once.
template <typename T, int NT, int KF> struct AReg { typename Mma<T>::Frag f[KF][NT]; };

// W: global [out, in] with row pitch ldw; rows o0 .. o0 + 16*NT - 1, k from k0.
template <typename T, int NT, int KF>
__device__ __forceinline__ void load_a(AReg<T, NT, KF>& a, const T* __restrict__ W, int ldw, int o0, int k0) {
  typedef typename Mma<T>::Frag Frag;
  const int lane = threadIdx.x & 63, m = lane & 15, g = lane >> 4;
  const T* wp = W + (size_t)(o0 + m) * ldw + k0 + g * Mma<T>::KL;
#pragma unroll
  for (int kf = 0; kf < KF; ++kf)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      a.f[kf][nt] = *reinterpret_cast<const Frag*>(wp + (size_t)(16 * nt) * ldw + kf * Mma<T>::KC);
}

// acc[nt][r] += W-fragments . X[16*(rt0+r) + .][k0 ...) for r < rt_cnt (<= RH).  X: LDS, pitch ldx.
template <typename T, int NT, int KF, int RH>
__device__ __forceinline__ void mma_rows(const AReg<T, NT, KF>& a, const T* Xs, int ldx, int k0, int rt0, int rt_cnt,
                                         f32x4 (&acc)[NT][RH]) {
  typedef typename Mma<T>::Frag Frag;
  const int lane = threadIdx.x & 63, m = lane & 15, g = lane >> 4;
  const T* xp = Xs + (16 * rt0 + m) * ldx + k0 + g * Mma<T>::KL;
#pragma unroll
  for (int kf = 0; kf < KF; ++kf) {
#pragma unroll
    for (int r = 0; r < RH; ++r) {
      if (r < rt_cnt) {
        const Frag b = *reinterpret_cast<const Frag*>(xp + (16 * r) * ldx + kf * Mma<T>::KC);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt][r] = Mma<T>::mma(a.f[kf][nt], b, acc[nt][r]);
      }
    }
  }
}

// One GEMM phase of a workgroup of NW wavefronts: Out^T[NOUT x rows] = W[NOUT x K] . X^T.
// Work items are (group of NT output tiles, half of the row tiles); wavefront w takes items
// w, w + NW, ...  Each item's weights are loaded in KSPLIT units of K/KSPLIT columns, and unit
// u + 1 is requested before unit u is consumed, so global-load latency overlaps the MFMAs.
template <typename T, int NT, int K, int NOUT, int NW, int KSPLIT> struct GemmPhase {
  static constexpr int KC = Mma<T>::KC;
  static constexpr int KFU = K / KC / KSPLIT;
  static constexpr int N_OG = NOUT / (16 * NT);
  static constexpr int N_ITEMS = 2 * N_OG;
  static constexpr int IPW = N_ITEMS / NW;
  static constexpr int UNITS = IPW * KSPLIT;
  static constexpr int RH = 3;               // row tiles per item: half of at most 6
  static_assert(N_ITEMS % NW == 0 && K % (KC * KSPLIT) == 0 && NOUT % (16 * NT) == 0, "phase shape");
  AReg<T, NT, KFU> a[2];
  const T* W;
  int wave;

  __device__ __forceinline__ GemmPhase(const void* w, int wave_) : W(reinterpret_cast<const T*>(w)), wave(wave_) {}

  __device__ __forceinline__ void issue(int u) {
    const int item = wave + (u / KSPLIT) * NW;
    load_a<T, NT, KFU>(a[u & 1], W, K, (item % N_OG) * 16 * NT, (u % KSPLIT) * KFU * KC);
  }

  // Needs issue(0) beforehand.  epi(o0, rt0, cnt, acc): acc[nt][r][i] is output feature
  // o0 + 16*nt + 4*g + i of row 16*(rt0 + r) + m, for r < cnt.
  template <typename Epi> __device__ __forceinline__ void run(const T* Xs, int ldx, int RT, Epi epi) {
    const int h0 = (RT + 1) >> 1;
#pragma unroll
    for (int it = 0; it < IPW; ++it) {
      const int item = wave + it * NW;
      const int og = item % N_OG, half = item / N_OG;
      const int rt0 = half ? h0 : 0, cnt = half ? RT - h0 : h0;
      f32x4 acc[NT][RH];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int r = 0; r < RH; ++r) acc[nt][r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kh = 0; kh < KSPLIT; ++kh) {
        const int u = it * KSPLIT + kh;
        if (u + 1 < UNITS) issue(u + 1);
        mma_rows<T, NT, KFU, RH>(a[u & 1], Xs, ldx, kh * KFU * KC, rt0, cnt, acc);
      }
      epi(og * 16 * NT, rt0, cnt, acc);
    }
  }
};

template <int NT, int RT_MAX> __device__ __forceinline__ void zero_acc(f32x4 (&acc)[NT][RT_MAX]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int rt = 0; rt < RT_MAX; ++rt) acc[nt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
