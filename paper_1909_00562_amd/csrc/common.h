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

// philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11): counter (c0..c3), key (k0,k1) -> w[4]
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&w)[4]) {
#pragma unroll 1   // kept as a loop: unrolled, 32 copies of it stop the GEMM epilogue around it from unrolling
  for (int r = 0; r < 10; ++r) {
    if (r > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
  }
  w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}
// the four random words of the elements with flat indices 4q .. 4q+3
__device__ __forceinline__ void dropout_words4(uint64_t q, uint64_t seed, uint32_t (&w)[4]) {
  philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), w);
}
// multiplier of the element with flat index i: scale if kept, 0 if dropped
__device__ __forceinline__ float dropout_mult(uint64_t i, uint64_t seed, uint32_t thr, float scale) {
  uint32_t w[4];
  dropout_words4(i >> 2, seed, w);
  const uint32_t k = (uint32_t)i & 3u;
  const uint32_t word = k == 0 ? w[0] : k == 1 ? w[1] : k == 2 ? w[2] : w[3];
  return word >= thr ? scale : 0.f;
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
