// Masked softmax over source positions (Eq. 1 of section 3.2) and its Jacobian.
// One 64-lane wavefront owns one (sentence, decoder step) row; reductions are
// wavefront shuffles, no LDS.
#include "common.h"
#include "kernels.h"

namespace asx {

template <typename TE>
__global__ __launch_bounds__(256) void attn_softmax_rows_kernel(const float* __restrict__ score,
                                                               const int32_t* __restrict__ src_len, int B, int T,
                                                               int S, float* __restrict__ alpha32,
                                                               TE* __restrict__ alphaE,
                                                               TE* __restrict__ alphaE_lo, int64_t ldS,
                                                               uint8_t* __restrict__ attn_mask) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);   // row = b*T + t
  if (row >= B * T) return;
  const int b = row / T, t = row - b * T;
  int L = src_len[b];
  L = L < 0 ? 0 : (L > S ? S : L);
  const float* x = score + (int64_t)row * S;
  float m = -INFINITY;
  for (int s = lane; s < L; s += 64) m = fmaxf(m, x[s]);
  m = wave_max(m);
  float sum = 0.f;
  for (int s = lane; s < L; s += 64) sum += expf(x[s] - m);
  sum = wave_sum(sum);
  const float inv = L > 0 ? 1.f / sum : 0.f;
  float* a32 = alpha32 + (int64_t)row * S;
  TE* aE = alphaE + (int64_t)row * ldS;
  for (int s = lane; s < (int)ldS; s += 64) {
    const float a = s < L ? expf(x[s] - m) * inv : 0.f;   // masked positions: exactly 0
    if (s < S) a32[s] = a;
    st_elem<TE>(aE, s, a);
    if (alphaE_lo) st_elem<TE>(alphaE_lo + (int64_t)row * ldS, s, a - round_elem<TE>(a));
  }
  if (attn_mask && t == 0)
    for (int s = lane; s < S; s += 64) attn_mask[(int64_t)b * S + s] = s < L ? 1 : 0;
}

template <typename TE>
__global__ __launch_bounds__(256) void attn_softmax_rows_bwd_kernel(const float* __restrict__ alpha32,
                                                                   const float* __restrict__ dalpha, int rows,
                                                                   int S, TE* __restrict__ dscoreE,
                                                                   TE* __restrict__ dscoreE_lo, int64_t ldS) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float* a = alpha32 + (int64_t)row * S;
  const float* da = dalpha + (int64_t)row * S;
  float r = 0.f;
  for (int s = lane; s < S; s += 64) r += a[s] * da[s];
  r = wave_sum(r);
  TE* d = dscoreE + (int64_t)row * ldS;
  for (int s = lane; s < (int)ldS; s += 64) {
    const float v = s < S ? a[s] * (da[s] - r) : 0.f;      // alpha = 0 at masked positions -> 0
    st_elem<TE>(d, s, v);
    if (dscoreE_lo) st_elem<TE>(dscoreE_lo + (int64_t)row * ldS, s, v - round_elem<TE>(v));
  }
}

hipError_t launch_attn_softmax_rows(const float* score, const int32_t* src_len, int B, int T, int S,
                                    float* alpha32, void* alphaE, void* alphaE_lo, int64_t ldS, bool e_bf16,
                                    uint8_t* attn_mask, hipStream_t st) {
  const int rows = B * T;
  dim3 grid((rows + 3) / 4);
  if (e_bf16)
    hipLaunchKernelGGL(attn_softmax_rows_kernel<uint16_t>, grid, dim3(256), 0, st, score, src_len, B, T, S,
                       alpha32, reinterpret_cast<uint16_t*>(alphaE), reinterpret_cast<uint16_t*>(alphaE_lo), ldS,
                       attn_mask);
  else
    hipLaunchKernelGGL(attn_softmax_rows_kernel<float>, grid, dim3(256), 0, st, score, src_len, B, T, S, alpha32,
                       reinterpret_cast<float*>(alphaE), reinterpret_cast<float*>(alphaE_lo), ldS, attn_mask);
  return hipGetLastError();
}

hipError_t launch_attn_softmax_rows_bwd(const float* alpha32, const float* dalpha, int B, int T, int S,
                                        void* dscoreE, void* dscoreE_lo, int64_t ldS, bool e_bf16,
                                        hipStream_t st) {
  const int rows = B * T;
  dim3 grid((rows + 3) / 4);
  if (e_bf16)
    hipLaunchKernelGGL(attn_softmax_rows_bwd_kernel<uint16_t>, grid, dim3(256), 0, st, alpha32, dalpha, rows, S,
                       reinterpret_cast<uint16_t*>(dscoreE), reinterpret_cast<uint16_t*>(dscoreE_lo), ldS);
  else
    hipLaunchKernelGGL(attn_softmax_rows_bwd_kernel<float>, grid, dim3(256), 0, st, alpha32, dalpha, rows, S,
                       reinterpret_cast<float*>(dscoreE), reinterpret_cast<float*>(dscoreE_lo), ldS);
  return hipGetLastError();
}

}  // namespace asx
