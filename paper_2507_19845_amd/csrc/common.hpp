// Shared device/host helpers of libgptstage (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gpts {

using bf16 = __bf16;  // hardware round-to-nearest-even conversions (v_cvt_pk_bf16_f32)

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
// fp16: the storage type of the forward activations when cfg.fwd_fp16 is set (3 more
// significand bits than bf16 at the same size and the same matrix-core rate)
using f16 = _Float16;
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// ---- storage <-> fp32 -------------------------------------------------------
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return static_cast<float>(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return static_cast<bf16>(v); }
__device__ __forceinline__ float to_f32(f16 v) { return static_cast<float>(v); }
// fp32 -> fp16, round to nearest even, saturating at the largest finite fp16 value
// instead of overflowing to infinity
__device__ __forceinline__ f16 sat_f16(float v) {
  return static_cast<f16>(__builtin_fminf(__builtin_fmaxf(v, -65504.f), 65504.f));
}
template <> __device__ __forceinline__ f16 from_f32<f16>(float v) { return sat_f16(v); }

// A 16-byte vector of storage elements: 4 x fp32 or 8 x bf16.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  f32x4 v;
  __device__ __forceinline__ float get(int i) const { return v[i]; }
  __device__ __forceinline__ void set(int i, float x) { v[i] = x; }
};
template <> struct Vec16<bf16> {
  static constexpr int N = 8;
  bf16x8 v;
  __device__ __forceinline__ float get(int i) const { return static_cast<float>(v[i]); }
  __device__ __forceinline__ void set(int i, float x) { v[i] = static_cast<bf16>(x); }
};
template <typename T> __device__ __forceinline__ Vec16<T> load16(const T* p) {
  return *reinterpret_cast<const Vec16<T>*>(p);
}
template <typename T> __device__ __forceinline__ void store16(T* p, const Vec16<T>& v) {
  *reinterpret_cast<Vec16<T>*>(p) = v;
}

// ---- wavefront / workgroup reductions (64-wide) ------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Sum over a workgroup of NW waves; every thread gets the result.  `red` is
// NW floats of LDS.  Fixed combination order -> deterministic.
template <int NW> __device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  if constexpr (NW == 1) return v;
  const int w = threadIdx.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) red[w] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) s += red[i];
  return s;
}

// ---- GeLU (fp32 evaluation) -----------------------------------------------------
// tanh form: 0.5 u (1 + tanh z), z = k (u + 0.044715 u^3), k = sqrt(2/pi).  Since
// 0.5 (1 + tanh z) = sigma(2z) (logistic function) it is evaluated as u * sigma(2z)
// with one hardware exp2 and one hardware reciprocal.  erf form: u Phi(u).
__device__ __forceinline__ float sigmoid2z(float u) {
  // sigma(2z) = 1 / (1 + 2^(-2 z log2 e)); exact limits 0 and 1 for large |u|
  const float z2 = (-2.f * 0.7978845608028654f * 1.4426950408889634f) * (u + 0.044715f * u * u * u);
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(z2));
}
template <int KIND> __device__ __forceinline__ float gelu_f(float u) {
  if constexpr (KIND == 0) {
    return u * sigmoid2z(u);
  } else {
    return 0.5f * u * (1.f + erff(u * 0.7071067811865476f));
  }
}
template <int KIND> __device__ __forceinline__ float gelu_grad_f(float u) {
  if constexpr (KIND == 0) {
    // d/du [u sigma(2z)] = sigma + u sigma (1 - sigma) 2 z'(u),  z' = k (1 + 3*0.044715 u^2)
    const float s = sigmoid2z(u);
    const float dz2 = (2.f * 0.7978845608028654f) * (1.f + 3.f * 0.044715f * u * u);
    return s + u * s * (1.f - s) * dz2;
  } else {
    const float cdf = 0.5f * (1.f + erff(u * 0.7071067811865476f));
    const float pdf = 0.3989422804014327f * __expf(-0.5f * u * u);
    return cdf + u * pdf;
  }
}

}  // namespace gpts
