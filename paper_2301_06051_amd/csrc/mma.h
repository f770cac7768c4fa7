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

// acc[nt][rt] += W[o0 + 16*nt + .][0..K) . X[16*rt + .][0..K) for nt < NT, rt < rt_count.
// W: global, row pitch ldw elements.  X: LDS, row pitch ldx elements (16-byte multiple).
template <typename T, int NT, int RT_MAX>
__device__ __forceinline__ void gemm_wx(const T* __restrict__ W, int ldw, int o0, const T* Xs, int ldx, int K,
                                        int rt_count, f32x4 (&acc)[NT][RT_MAX]) {
  typedef typename Mma<T>::Frag Frag;
  constexpr int KC = Mma<T>::KC, KL = Mma<T>::KL;
  const int lane = threadIdx.x & 63, m = lane & 15, g = lane >> 4;
  const T* wp = W + (size_t)(o0 + m) * ldw + g * KL;
  const T* xp = Xs + m * ldx + g * KL;
#pragma unroll 2
  for (int k0 = 0; k0 < K; k0 += KC) {
    Frag a[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) a[nt] = *reinterpret_cast<const Frag*>(wp + (size_t)(16 * nt) * ldw + k0);
#pragma unroll
    for (int rt = 0; rt < RT_MAX; ++rt) {
      if (rt < rt_count) {
        Frag b = *reinterpret_cast<const Frag*>(xp + (16 * rt) * ldx + k0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt][rt] = Mma<T>::mma(a[nt], b, acc[nt][rt]);
      }
    }
  }
}

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
