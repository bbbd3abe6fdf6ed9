// Shared device/host helpers for the attention-softmax kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asx {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
  return __builtin_bit_cast(float, bits16 << 16);
}
__device__ __forceinline__ float lo_bf16(uint32_t packed) { return __builtin_bit_cast(float, packed << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t packed) { return __builtin_bit_cast(float, packed & 0xffff0000u); }

// round-to-nearest-even float -> bf16 bit pattern
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  bf16_t h = (bf16_t)f;
  return (uint32_t)__builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// element load/store by storage type
template <typename T> __device__ __forceinline__ float ld_elem(const T* p, int64_t i);
template <> __device__ __forceinline__ float ld_elem<float>(const float* p, int64_t i) { return p[i]; }
template <> __device__ __forceinline__ float ld_elem<uint16_t>(const uint16_t* p, int64_t i) {
  return bf16_bits_to_f32(p[i]);
}
template <typename T> __device__ __forceinline__ void st_elem(T* p, int64_t i, float v);
template <> __device__ __forceinline__ void st_elem<float>(float* p, int64_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void st_elem<uint16_t>(uint16_t* p, int64_t i, float v) {
  p[i] = (uint16_t)f32_to_bf16_bits(v);
}

// value of v after rounding to the storage type
template <typename T> __device__ __forceinline__ float round_elem(float v);
template <> __device__ __forceinline__ float round_elem<float>(float v) { return v; }
template <> __device__ __forceinline__ float round_elem<uint16_t>(float v) {
  return bf16_bits_to_f32(f32_to_bf16_bits(v));
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace asx
