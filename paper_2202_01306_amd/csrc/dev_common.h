// Device-side helpers shared by the kernels: element types, 16-byte vector
// access, wavefront (64 lanes) and block reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hmy {

typedef __bf16 bf16_t;

template <typename E> struct ElemTraits;
template <> struct ElemTraits<float> { static constexpr int VEC = 4; };
template <> struct ElemTraits<bf16_t> { static constexpr int VEC = 8; };

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return static_cast<float>(x); }
template <typename E> __device__ __forceinline__ E from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return static_cast<bf16_t>(x); }  // RNE

// 16 bytes of E, register-resident
template <typename E> struct alignas(16) Vec16 {
  E v[ElemTraits<E>::VEC];
};
template <typename E> __device__ __forceinline__ Vec16<E> load16(const E *p) {
  return *reinterpret_cast<const Vec16<E> *>(p);
}
template <typename E> __device__ __forceinline__ void store16(E *p, const Vec16<E> &x) {
  *reinterpret_cast<Vec16<E> *>(p) = x;
}

constexpr int kWave = 64;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// tanh-form GELU and its derivative, fp32
__device__ __forceinline__ float gelu_f(float u) {
  const float c = 0.7978845608028654f, a = 0.044715f;
  return 0.5f * u * (1.f + tanhf(c * (u + a * u * u * u)));
}
__device__ __forceinline__ float gelu_grad_f(float u) {
  const float c = 0.7978845608028654f, a = 0.044715f;
  const float th = tanhf(c * (u + a * u * u * u));
  return 0.5f * (1.f + th) + 0.5f * u * (1.f - th * th) * c * (1.f + 3.f * a * u * u);
}

}  // namespace hmy
