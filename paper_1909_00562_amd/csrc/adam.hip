// Fused Adam update of one parameter tensor (paper section 4.2, "Parameter
// settings"; Kingma and Ba, Algorithm 1).  One streaming pass: per element 16
// bytes read (gradient, both moments, master weight), 12 written back and the
// 2- or 4-byte copy in the storage type of the forward pass; HBM-bound.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.h"
#include "kernels.h"

namespace asx {

template <bool OUT_BF16, bool HAS_OUT>
__global__ __launch_bounds__(256) void adam_step_kernel(size_t n4, size_t n, const float* __restrict__ grad,
                                                        float* __restrict__ master, float* __restrict__ m,
                                                        float* __restrict__ v, void* __restrict__ wout, float lr,
                                                        float beta1, float beta2, float eps, float inv_bc1,
                                                        float inv_bc2) {
  const float omb1 = 1.f - beta1, omb2 = 1.f - beta2;
  auto upd = [&](float g, float& mm, float& vv, float& w) {
    mm = beta1 * mm + omb1 * g;
    vv = beta2 * vv + omb2 * g * g;
    w -= lr * (mm * inv_bc1) / (sqrtf(vv * inv_bc2) + eps);
  };
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    const f32x4_t g4 = reinterpret_cast<const f32x4_t*>(grad)[i];
    f32x4_t m4 = reinterpret_cast<f32x4_t*>(m)[i], v4 = reinterpret_cast<f32x4_t*>(v)[i];
    f32x4_t w4 = reinterpret_cast<f32x4_t*>(master)[i];
    float mm[4] = {m4[0], m4[1], m4[2], m4[3]}, vv[4] = {v4[0], v4[1], v4[2], v4[3]};
    float w[4] = {w4[0], w4[1], w4[2], w4[3]};
#pragma unroll
    for (int c = 0; c < 4; ++c) upd(g4[c], mm[c], vv[c], w[c]);
    reinterpret_cast<f32x4_t*>(m)[i] = f32x4_t{mm[0], mm[1], mm[2], mm[3]};
    reinterpret_cast<f32x4_t*>(v)[i] = f32x4_t{vv[0], vv[1], vv[2], vv[3]};
    reinterpret_cast<f32x4_t*>(master)[i] = f32x4_t{w[0], w[1], w[2], w[3]};
    if constexpr (HAS_OUT) {
      if constexpr (OUT_BF16)
        reinterpret_cast<uint2*>(wout)[i] = make_uint2(pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3]));
      else
        reinterpret_cast<f32x4_t*>(wout)[i] = f32x4_t{w[0], w[1], w[2], w[3]};
    }
  }
  // ragged tail (n % 4 elements), one thread each
  const size_t t = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t < n) {
    float mm = m[t], vv = v[t], w = master[t];
    upd(grad[t], mm, vv, w);
    m[t] = mm;
    v[t] = vv;
    master[t] = w;
    if constexpr (HAS_OUT) {
      if constexpr (OUT_BF16) reinterpret_cast<uint16_t*>(wout)[t] = (uint16_t)f32_to_bf16_bits(w);
      else reinterpret_cast<float*>(wout)[t] = w;
    }
  }
}

hipError_t launch_adam_step(size_t n, const float* grad, float* master, float* m, float* v, void* wout,
                            bool out_bf16, float lr, float beta1, float beta2, float eps, float inv_bc1,
                            float inv_bc2, hipStream_t st) {
  const size_t n4 = n / 4;
  size_t blocks = (n4 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;   // 16 resident blocks per CU, grid-stride beyond
  if (blocks < 1) blocks = 1;
  dim3 grid((unsigned)blocks), blk(256);
#define ASX_ADAM(BF, HO) \
  hipLaunchKernelGGL((adam_step_kernel<BF, HO>), grid, blk, 0, st, n4, n, grad, master, m, v, wout, lr, beta1, beta2, \
                     eps, inv_bc1, inv_bc2)
  if (!wout) ASX_ADAM(false, false);
  else if (out_bf16) ASX_ADAM(true, true);
  else ASX_ADAM(false, true);
#undef ASX_ADAM
  return hipGetLastError();
}

}  // namespace asx
