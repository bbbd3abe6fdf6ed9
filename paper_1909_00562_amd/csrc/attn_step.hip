// Attention for ONE decoder step (T = 1), fused: scores (Eq. 2), masked softmax
// (Eq. 1) and context vector (Eq. 3) of section 3.2 in one kernel, one workgroup
// per sentence.  The encoder-side half of the score, K'[s,b,:] = W_a h_enc[s,b,:],
// does not depend on the decoder step and is computed once per batch of sentences,
// so a step costs one pass over K' (float) and one over h_enc:
//   score[s] = h_t[b] . K'[s,b]      alpha = softmax_{s < src_len[b]}      ctx = sum_s alpha[s] h_enc[s,b]
// Used by the per-step mode (decoding, scoring, the input-feeding variant of the
// paper's section 4, where step t+1 needs the attentional state of step t).
#include "common.h"
#include "kernels.h"

namespace asx {

typedef uint32_t u32x4_raw __attribute__((ext_vector_type(4)));
constexpr int kStepThreads = 512, kStepWaves = kStepThreads / 64;

template <typename TE>
__global__ __launch_bounds__(kStepThreads) void attn_step_kernel(const TE* __restrict__ h_t, const float* __restrict__ kprime,
                                                       const TE* __restrict__ h_enc,
                                                       const int32_t* __restrict__ src_len, int B, int S, int H,
                                                       float* __restrict__ alpha, TE* __restrict__ ctx,
                                                       TE* __restrict__ ctx_lo, uint8_t* __restrict__ attn_mask) {
  extern __shared__ float sm[];          // h_t as float [H], scores / alpha [S], context partial sums [G][H]
  float* hs = sm;
  float* sc = sm + H;
  __shared__ float red[2 * kStepWaves];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int L = src_len[b];
  L = L < 0 ? 0 : (L > S ? S : L);
  for (int c = tid; c < H; c += kStepThreads) hs[c] = ld_elem<TE>(h_t, (int64_t)b * H + c);
  __syncthreads();

  // scores: one wavefront per source position (two at a time, so that the loads of both are in flight),
  // lanes across H
  auto dot = [&](int s) {
    const float* kp = kprime + ((int64_t)s * B + b) * H;
    float acc = 0.f;
    if ((H & 3) == 0) {
      for (int c = lane * 4; c < H; c += 256) {
        const f32x4_t k4 = *reinterpret_cast<const f32x4_t*>(kp + c);
        const f32x4_t h4 = *reinterpret_cast<const f32x4_t*>(hs + c);
        acc += k4[0] * h4[0] + k4[1] * h4[1] + k4[2] * h4[2] + k4[3] * h4[3];
      }
    } else {
      for (int c = lane; c < H; c += 64) acc += kp[c] * hs[c];
    }
    return acc;
  };
  for (int s = wave; s < L; s += 2 * kStepWaves) {
    const int s2 = s + kStepWaves;
    float a0 = dot(s), a1 = s2 < L ? dot(s2) : 0.f;
    a0 = wave_sum(a0);
    a1 = wave_sum(a1);
    if (lane == 0) {
      sc[s] = a0;
      if (s2 < L) sc[s2] = a1;
    }
  }
  __syncthreads();

  // masked softmax over the L valid positions
  float m = -INFINITY;
  for (int s = tid; s < L; s += kStepThreads) m = fmaxf(m, sc[s]);
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = red[0];
#pragma unroll
  for (int i = 1; i < kStepWaves; ++i) m = fmaxf(m, red[i]);
  float sum = 0.f;
  for (int s = tid; s < L; s += kStepThreads) sum += expf(sc[s] - m);
  sum = wave_sum(sum);
  if (lane == 0) red[kStepWaves + wave] = sum;
  __syncthreads();
  sum = 0.f;
#pragma unroll
  for (int i = 0; i < kStepWaves; ++i) sum += red[kStepWaves + i];
  const float inv = L > 0 ? 1.f / sum : 0.f;
  for (int s = tid; s < S; s += kStepThreads) {
    const float a = s < L ? expf(sc[s] - m) * inv : 0.f;   // masked positions: exactly 0
    alpha[(int64_t)b * S + s] = a;
    if (attn_mask) attn_mask[(int64_t)b * S + s] = s < L ? 1 : 0;
  }
  __syncthreads();                        // every thread has read sc[] (its max / sum passes) before it is overwritten
  for (int s = tid; s < L; s += kStepThreads) sc[s] = expf(sc[s] - m) * inv;
  __syncthreads();

  // context: the threads form G groups; a group covers all of H with 16-byte vectors and takes every G-th
  // source position; the G partial sums are added in a fixed order
  constexpr int VEC = 16 / (int)sizeof(TE);
  float* part = sc + S;                   // [G][H]
  if (H % VEC == 0 && H / VEC <= kStepThreads) {
    const int per = H / VEC;              // threads of one group
    const int G = kStepThreads / per < 8 ? kStepThreads / per : 8;
    const int grp = tid / per, c = (tid - grp * per) * VEC;
    if (grp < G) {
      float acc[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
      for (int s = grp; s < L; s += G) {
        const TE* src = h_enc + ((int64_t)s * B + b) * H + c;
        const float a = sc[s];
        if constexpr (sizeof(TE) == 2) {
          const u32x4_raw raw = *reinterpret_cast<const u32x4_raw*>(src);
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            acc[2 * v] += a * lo_bf16(raw[v]);
            acc[2 * v + 1] += a * hi_bf16(raw[v]);
          }
        } else {
          const f32x4_t raw = *reinterpret_cast<const f32x4_t*>(src);
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[v] += a * raw[v];
        }
      }
#pragma unroll
      for (int v = 0; v < VEC; ++v) part[grp * H + c + v] = acc[v];
    }
    __syncthreads();
    for (int cc = tid; cc < H; cc += kStepThreads) {
      float acc = 0.f;
      for (int g = 0; g < G; ++g) acc += part[g * H + cc];
      st_elem<TE>(ctx, (int64_t)b * H + cc, acc);
      if (ctx_lo) st_elem<TE>(ctx_lo, (int64_t)b * H + cc, acc - round_elem<TE>(acc));
    }
  } else {
    for (int c = tid; c < H; c += kStepThreads) {
      float acc = 0.f;
      for (int s = 0; s < L; ++s) acc += sc[s] * ld_elem<TE>(h_enc, ((int64_t)s * B + b) * H + c);
      st_elem<TE>(ctx, (int64_t)b * H + c, acc);
      if (ctx_lo) st_elem<TE>(ctx_lo, (int64_t)b * H + c, acc - round_elem<TE>(acc));
    }
  }
}

hipError_t launch_attn_step(const void* h_t, const float* kprime, const void* h_enc, const int32_t* src_len, int B,
                            int S, int H, float* alpha, void* ctx, void* ctx_lo, bool e_bf16, uint8_t* attn_mask,
                            hipStream_t st) {
  // h_t, scores, partial contexts: G groups x H floats with G <= 8 and G * H <= threads * 8
  const size_t part = (size_t)8 * H < (size_t)kStepThreads * 8 ? (size_t)8 * H : (size_t)kStepThreads * 8;
  const size_t smem = ((size_t)H + S + part) * sizeof(float);
  if (smem > 150 * 1024) return hipErrorInvalidValue;
  if (e_bf16) {
    auto k = attn_step_kernel<uint16_t>;
    if (smem > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)smem);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k, dim3(B), dim3(kStepThreads), smem, st, reinterpret_cast<const uint16_t*>(h_t), kprime,
                       reinterpret_cast<const uint16_t*>(h_enc), src_len, B, S, H, alpha,
                       reinterpret_cast<uint16_t*>(ctx), reinterpret_cast<uint16_t*>(ctx_lo), attn_mask);
  } else {
    auto k = attn_step_kernel<float>;
    if (smem > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)smem);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k, dim3(B), dim3(kStepThreads), smem, st, reinterpret_cast<const float*>(h_t), kprime,
                       reinterpret_cast<const float*>(h_enc), src_len, B, S, H, alpha, reinterpret_cast<float*>(ctx),
                       reinterpret_cast<float*>(ctx_lo), attn_mask);
  }
  return hipGetLastError();
}

}  // namespace asx
