// Fused attention for the batched path, bf16 storage (section 3.2, Eq. 1-3): one workgroup per
// (sentence b, block of 32 decoder steps) computes
//   score[t,s] = (q_hi + q_lo)[t,b,:] . h_enc[s,b,:]      (Eq. 2; q = h_dec W_a as value + rounding remainder)
//   alpha[t,:] = softmax over s < src_len[b], exactly 0 elsewhere   (Eq. 1)
//   ctx[t,b,:] = sum_s alpha[t,s] h_enc[s,b,:]             (Eq. 3; alpha enters as value + remainder)
// without the scores ever leaving the compute unit.  It replaces three launches (batched score product,
// softmax rows, batched context product) whose 128x128 tiles were mostly padding at T, S <= 80.
// The same kernel with BWD = true is the first half of the attention backward pass, which has the same shape:
//   dalpha[t,s] = (dC_hi + dC_lo)[t,b,:] . h_enc[s,b,:]
//   dscore[t,:] = alpha[t,:] * (dalpha[t,:] - sum_s alpha[t,s] dalpha[t,s])      (softmax Jacobian)
//   dQ[t,b,:]   = sum_s dscore[t,s] h_enc[s,b,:]
// (dscore also leaves as bf16 value / remainder for the product that forms d_h_enc).
//
// The four waves of a workgroup run as private pipelines, with no workgroup barrier inside a phase: LDS operations
// of one wave complete in order, so a wave can fill its own LDS slice and read fragments back without one.
// Phase 1 (scores): the reduction over H is cut into tiles of 32; wave w takes tiles w, w+4, ...  For each it
//   brings q_hi, q_lo (32 rows each) and the S encoder rows through its own LDS slice (rows of 32 reduction
//   elements = 64 bytes, 16-byte chunks swizzled with (row >> 2) & 3), loaded into registers one tile ahead, and
//   accumulates all score tiles (32 x 32 MFMA tiles, up to four) over its share of H.  The four partial sums
//   meet in LDS in a fixed order.
// Phase 2 (softmax): one wavefront per row, shuffle reductions; alpha goes to global memory (float, and the bf16
//   value / remainder copies the backward pass reads) and to LDS as the row operand of phase 3.
// Phase 3 (context): the reduction runs over source positions, so h_enc_b is the strided operand.  Wave w takes
//   the 64-column chunks w, w+4, ... of H: [s][64 columns] as stored (rows padded to 160 bytes so that the four
//   rows a transposing read touches fall on different banks), read with ds_read_b64_tr_b16.  Results are staged
//   through the wave's LDS slice so that ctx / ctx_lo leave as 8-byte row vectors.
#include "common.h"
#include "kernels.h"

namespace asx {

namespace {

constexpr int AF_ROWS = 32;      // decoder steps per workgroup
constexpr int AF_THREADS = 256;  // 4 waves

typedef uint32_t af_u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t af_u32x2_t __attribute__((ext_vector_type(2)));
typedef short af_s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) af_s16x4_t af_lds_s16x4_t;
typedef __attribute__((address_space(3))) void af_lds_void_t;

// alpha operand blocks: rows of 64 elements (128 bytes), chunk c of row r at chunk c ^ (r & 7) ^ ((r >> 3) & 1)
__device__ __forceinline__ uint32_t kc_off(int row, int chunk) {
  return (uint32_t)(row * 128 + ((chunk ^ (row & 7) ^ ((row >> 3) & 1)) << 4));
}
__device__ __forceinline__ bf16x8_t kc_frag(const unsigned char* tile, int row, int chunk) {
  return *reinterpret_cast<const bf16x8_t*>(tile + kc_off(row, chunk));
}
// phase-1 slices: rows of 32 elements (64 bytes), chunk c (0..3) of row r at chunk c ^ ((r >> 2) & 3)
__device__ __forceinline__ uint32_t k32_off(int row, int chunk) {
  return (uint32_t)(row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4));
}
__device__ __forceinline__ bf16x8_t k32_frag(const unsigned char* tile, int row, int chunk) {
  return *reinterpret_cast<const bf16x8_t*>(tile + k32_off(row, chunk));
}
// phase-3 slices [k][64 columns], k-rows AF_RS bytes apart.  Transposing read: a 16-lane group presents four k-rows x
// 16 columns, each lane receives four consecutive k of its own column (two reads, 4 k-rows apart, give 8).
constexpr int AF_RS = 160;
__device__ __forceinline__ uint32_t st_frag_base(int col0, int lane) {
  const int col = col0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  const int k0 = (lane >> 5) * 8 + ((lane & 15) >> 2);
  return (uint32_t)(k0 * AF_RS + col * 2);
}
__device__ __forceinline__ bf16x8_t st_frag(const unsigned char* tile, uint32_t base, int kk) {
  union { af_s16x4_t h[2]; bf16x8_t v; } u;
#pragma unroll
  for (int q = 0; q < 2; ++q)
    u.h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (af_lds_s16x4_t*)(af_lds_void_t*)(tile + base + kk * 16 * AF_RS + q * 4 * AF_RS));
  return u.v;
}

struct AttnFwdArgs {
  const uint16_t *q_hi, *q_lo, *h_enc;   // row operand of phase 1 as value / remainder (q, or dC for BWD), encoder states
  const int32_t* src_len;
  float* alpha32;                        // forward: written; BWD: read
  uint16_t *alphaE, *alphaE_lo;          // [B,T,ldS] copies of the row result (alpha, or dscore for BWD)
  uint16_t *ctx, *ctx_lo;                // phase-3 result (ctx + remainder, or dQ with ctx_lo = null for BWD)
  uint8_t* attn_mask;
  int T, S, B, H;
  int64_t ldS;
  int SP;         // S rounded up to 32: score columns computed
  int KS;         // S rounded up to 16: reduction length of the context product
  int p1_bytes, p3_bytes;   // bytes of one wave's LDS slice in phase 1 / phase 3 (both live in region 0)
  int off_x, off_a;         // LDS byte offsets of the score / staging region and of the alpha operand blocks
};

template <bool BWD>
__global__ __launch_bounds__(AF_THREADS) void attn_fwd_fused_kernel(AttnFwdArgs p) {
  extern __shared__ __align__(1024) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.x, t0 = blockIdx.y * AF_ROWS;
  const int T = p.T, S = p.S, B = p.B, H = p.H, SP = p.SP;
  const int64_t BH = (int64_t)B * H;
  int L = p.src_len[b];
  L = L < 0 ? 0 : (L > S ? S : L);
  const int SS = SP / 32;                           // score tiles of 32 columns (<= 4)

  // ---------------- phase 1: scores, each wave over its share of H -------------------------------
  {
    unsigned char* slice = smem + wave * p.p1_bytes;
    const int nl = (64 + SP) / 16;                  // wave-wide 16-byte loads per tile (16 rows of 64 bytes each)
    const int nkt = (H + 31) / 32;
    af_u32x4_t regs[12];                            // nl <= 12 (S <= 128)
    auto load_tile = [&](int kt) {
#pragma unroll
      for (int i = 0; i < 12; ++i) {
        regs[i] = af_u32x4_t{0, 0, 0, 0};
        if (i < nl) {
          const int row = i * 16 + (lane >> 2), k = kt * 32 + (lane & 3) * 8;
          const uint16_t* src = nullptr;
          if (row < 32) {
            if (t0 + row < T) src = p.q_hi + (int64_t)(t0 + row) * BH + (int64_t)b * H;
          } else if (row < 64) {
            if (t0 + row - 32 < T) src = p.q_lo + (int64_t)(t0 + row - 32) * BH + (int64_t)b * H;
          } else if (row - 64 < S) {
            src = p.h_enc + (int64_t)(row - 64) * BH + (int64_t)b * H;
          }
          if (src && k < H) regs[i] = *reinterpret_cast<const af_u32x4_t*>(src + k);
        }
      }
    };
    f32x16_t sacc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[j][r] = 0.f;
    if (wave < nkt) load_tile(wave);
    for (int kt = wave; kt < nkt; kt += 4) {
#pragma unroll
      for (int i = 0; i < 12; ++i)
        if (i < nl)
          *reinterpret_cast<af_u32x4_t*>(slice + k32_off(i * 16 + (lane >> 2), lane & 3)) = regs[i];
      if (kt + 4 < nkt) load_tile(kt + 4);          // in flight while this tile is multiplied
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const int chunk = kk * 2 + (lane >> 5);
        const bf16x8_t a_hi = k32_frag(slice, lane & 31, chunk);
        const bf16x8_t a_lo = k32_frag(slice, 32 + (lane & 31), chunk);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (j < SS) {
            const bf16x8_t bf = k32_frag(slice, 64 + j * 32 + (lane & 31), chunk);
            sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, bf, sacc[j], 0, 0, 0);
            sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, bf, sacc[j], 0, 0, 0);
          }
      }
    }
    // the four partial sums meet in two LDS buffers: waves 0, 1 store, then waves 2, 3 add (fixed order)
    const int sld = SP + 8;                         // row stride: the two half-waves of a store hit different banks
    float* buf = reinterpret_cast<float*>(smem + p.off_x) + (wave & 1) * (AF_ROWS * sld);
    if (wave < 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < SS)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            buf[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * sld + j * 32 + (lane & 31)] = sacc[j][r];
    }
    __syncthreads();
    if (wave >= 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < SS)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            buf[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * sld + j * 32 + (lane & 31)] += sacc[j][r];
    }
    __syncthreads();
  }

  // ---------------- phase 2: masked softmax rows --------------------------------------------------
  const int KB = (p.KS + 63) / 64;                                  // 64-wide reduction blocks of the alpha operand
  unsigned char* a_hi_blk = smem + p.off_a;                         // [KB][32 rows][64] value
  unsigned char* a_lo_blk = a_hi_blk + KB * 4096;                   // same, rounding remainder
  {
    const int sld = SP + 8;
    const float* sc0 = reinterpret_cast<const float*>(smem + p.off_x);
    const float* sc1 = sc0 + AF_ROWS * sld;
    for (int rr = 0; rr < 8; ++rr) {
      const int row = wave * 8 + rr, t = t0 + row;
      const int s0 = lane, s1 = lane + 64;
      float a0, a1;
      if constexpr (!BWD) {
        const float x0 = s0 < L ? sc0[row * sld + s0] + sc1[row * sld + s0] : -INFINITY;
        const float x1 = s1 < L ? sc0[row * sld + s1] + sc1[row * sld + s1] : -INFINITY;
        const float m = wave_max(fmaxf(x0, x1));
        const float e0 = s0 < L ? expf(x0 - m) : 0.f, e1 = s1 < L ? expf(x1 - m) : 0.f;
        const float sum = wave_sum(e0 + e1);
        const float inv = L > 0 ? 1.f / sum : 0.f;
        a0 = s0 < L ? e0 * inv : 0.f;             // masked positions: exactly 0
        a1 = s1 < L ? e1 * inv : 0.f;
      } else {
        // softmax Jacobian; alpha is 0 at masked positions, so dscore is exactly 0 there
        const bool v0 = s0 < S && t < T, v1 = s1 < S && t < T;
        const float al0 = v0 ? p.alpha32[((int64_t)b * T + t) * S + s0] : 0.f;
        const float al1 = v1 ? p.alpha32[((int64_t)b * T + t) * S + s1] : 0.f;
        const float x0 = v0 ? sc0[row * sld + s0] + sc1[row * sld + s0] : 0.f;
        const float x1 = v1 ? sc0[row * sld + s1] + sc1[row * sld + s1] : 0.f;
        const float r = wave_sum(al0 * x0 + al1 * x1);
        a0 = al0 * (x0 - r);
        a1 = al1 * (x1 - r);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int s = h ? s1 : s0;
        const float a = h ? a1 : a0;
        const uint32_t hb = f32_to_bf16_bits(a);
        const uint32_t lb = f32_to_bf16_bits(a - bf16_bits_to_f32(hb));
        if (s < KB * 64) {                          // operand of phase 3 (zeros beyond the valid positions)
          const uint32_t o = (uint32_t)((s >> 6) * 4096) + kc_off(row, (s & 63) >> 3) + (uint32_t)(s & 7) * 2;
          *reinterpret_cast<uint16_t*>(a_hi_blk + o) = (uint16_t)hb;
          *reinterpret_cast<uint16_t*>(a_lo_blk + o) = (uint16_t)lb;
        }
        if (t < T) {
          if constexpr (!BWD)
            if (s < S) p.alpha32[((int64_t)b * T + t) * S + s] = a;
          if (s < p.ldS) {
            p.alphaE[((int64_t)b * T + t) * p.ldS + s] = (uint16_t)hb;
            p.alphaE_lo[((int64_t)b * T + t) * p.ldS + s] = (uint16_t)lb;
          }
        }
      }
    }
    if (!BWD && p.attn_mask && blockIdx.y == 0)
      for (int s = tid; s < S; s += AF_THREADS) p.attn_mask[(int64_t)b * S + s] = s < L ? 1 : 0;
  }
  __syncthreads();     // alpha blocks complete; score buffers and phase-1 slices are dead from here on

  // ---------------- phase 3: context vectors, each wave over its 64-column chunks of H ---------------
  {
    unsigned char* slice = smem + wave * p.p3_bytes;
    const int KS = p.KS, nks = KS / 16;             // reduction steps of 16 source positions
    const int nch = (H + 63) / 64;
    const int nl = KS / 8;                          // wave-wide 16-byte loads per chunk (8 k-rows of 128 bytes each)
    af_u32x4_t cregs[16];                           // nl <= 16 (S <= 128)
    auto load_chunk = [&](int c) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        cregs[i] = af_u32x4_t{0, 0, 0, 0};
        if (i < nl) {
          const int k = i * 8 + (lane >> 3), col = c * 64 + (lane & 7) * 8;
          if (k < S && col < H)
            cregs[i] = *reinterpret_cast<const af_u32x4_t*>(p.h_enc + (int64_t)k * BH + (int64_t)b * H + col);
        }
      }
    };
    const uint32_t bbase0 = st_frag_base(0, lane), bbase1 = st_frag_base(32, lane);
    float* stage_f = reinterpret_cast<float*>(smem + p.off_x) + wave * 1024;   // this wave's 16 x 64 floats
    const int vcol = (lane & 15) * 4, vrow = lane >> 4;
    if (wave < nch) load_chunk(wave);
    for (int c = wave; c < nch; c += 4) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (i < nl)
          *reinterpret_cast<af_u32x4_t*>(slice + (i * 8 + (lane >> 3)) * AF_RS + (lane & 7) * 16) = cregs[i];
      if (c + 4 < nch) load_chunk(c + 4);           // in flight while this chunk is multiplied and written out
      f32x16_t cacc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) cacc[j][r] = 0.f;
      for (int kk = 0; kk < nks; ++kk) {
        const int chunk = (kk & 3) * 2 + (lane >> 5);
        const bf16x8_t ah = kc_frag(a_hi_blk + (kk >> 2) * 4096, lane & 31, chunk);
        const bf16x8_t al = kc_frag(a_lo_blk + (kk >> 2) * 4096, lane & 31, chunk);
        const bf16x8_t b0 = st_frag(slice, bbase0, kk);
        const bf16x8_t b1 = st_frag(slice, bbase1, kk);
        cacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b0, cacc[0], 0, 0, 0);
        cacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b1, cacc[1], 0, 0, 0);
        cacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b0, cacc[0], 0, 0, 0);
        cacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b1, cacc[1], 0, 0, 0);
      }
      // write-out: 16 rows at a time through this wave's staging slice, 8-byte row vectors to ctx and ctx_lo
      const int col = c * 64 + vcol;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r8 = 0; r8 < 8; ++r8) {
            const int r = half * 8 + r8;
            stage_f[(8 * (r8 >> 2) + 4 * (lane >> 5) + (r8 & 3)) * 64 + j * 32 + (lane & 31)] = cacc[j][r];
          }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int row = it * 4 + vrow;
          const f32x4_t v4 = *reinterpret_cast<const f32x4_t*>(stage_f + row * 64 + vcol);
          const int t = t0 + half * 16 + row;
          if (t < T && col < H) {
            uint32_t hb[4];
            float lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              hb[e] = f32_to_bf16_bits(v4[e]);
              lo[e] = v4[e] - bf16_bits_to_f32(hb[e]);
            }
            const int64_t o = (int64_t)t * BH + (int64_t)b * H + col;
            *reinterpret_cast<af_u32x2_t*>(p.ctx + o) = af_u32x2_t{hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16)};
            if constexpr (!BWD)
              *reinterpret_cast<af_u32x2_t*>(p.ctx_lo + o) = af_u32x2_t{pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3])};
          }
        }
      }
    }
  }
}

}  // namespace

bool attn_fwd_fused_supported(int S, int H) { return S >= 1 && S <= 128 && (H % 8) == 0; }

static hipError_t launch_attn_fused(bool bwd, AttnFwdArgs p, hipStream_t st) {
  if (!attn_fwd_fused_supported(p.S, p.H) || p.B < 1 || p.T < 1 || p.ldS < p.S || p.ldS > 128) return hipErrorInvalidValue;
  p.SP = (p.S + 31) / 32 * 32;
  p.KS = (p.S + 15) / 16 * 16;
  // LDS: region 0 holds the four wave slices of phase 1 ((64 + SP) rows x 64 bytes each) and later those of phase 3
  // (KS k-rows x 160 bytes each); then the two score buffers / the write-out staging; then the alpha operand blocks
  p.p1_bytes = (64 + p.SP) * 64;
  p.p3_bytes = p.KS * AF_RS;
  const int ph1 = 4 * p.p1_bytes, ph3 = 4 * p.p3_bytes;
  const int region0 = ((ph1 > ph3 ? ph1 : ph3) + 1023) / 1024 * 1024;
  const int scores = 2 * AF_ROWS * (p.SP + 8) * 4, staging = 4 * 16 * 64 * 4;
  const int regionx = ((scores > staging ? scores : staging) + 1023) / 1024 * 1024;
  const int KB = (p.KS + 63) / 64;
  p.off_x = region0;
  p.off_a = region0 + regionx;
  const int smem = p.off_a + 2 * KB * 4096;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_fwd_fused_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_fwd_fused_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const dim3 grid(p.B, (p.T + AF_ROWS - 1) / AF_ROWS);
  if (bwd) hipLaunchKernelGGL(attn_fwd_fused_kernel<true>, grid, dim3(AF_THREADS), smem, st, p);
  else hipLaunchKernelGGL(attn_fwd_fused_kernel<false>, grid, dim3(AF_THREADS), smem, st, p);
  return hipGetLastError();
}

hipError_t launch_attn_fwd_fused(const void* q_hi, const void* q_lo, const void* h_enc, const int32_t* src_len, int B,
                                 int T, int S, int H, float* alpha32, void* alphaE, void* alphaE_lo, int64_t ldS,
                                 void* ctx, void* ctx_lo, uint8_t* attn_mask, hipStream_t st) {
  AttnFwdArgs p{};
  p.q_hi = reinterpret_cast<const uint16_t*>(q_hi);
  p.q_lo = reinterpret_cast<const uint16_t*>(q_lo);
  p.h_enc = reinterpret_cast<const uint16_t*>(h_enc);
  p.src_len = src_len;
  p.alpha32 = alpha32;
  p.alphaE = reinterpret_cast<uint16_t*>(alphaE);
  p.alphaE_lo = reinterpret_cast<uint16_t*>(alphaE_lo);
  p.ctx = reinterpret_cast<uint16_t*>(ctx);
  p.ctx_lo = reinterpret_cast<uint16_t*>(ctx_lo);
  p.attn_mask = attn_mask;
  p.T = T; p.S = S; p.B = B; p.H = H;
  p.ldS = ldS;
  return launch_attn_fused(false, p, st);
}

hipError_t launch_attn_bwd_fused(const void* dC_hi, const void* dC_lo, const void* h_enc, const int32_t* src_len,
                                 int B, int T, int S, int H, const float* alpha32, void* dscoreE, void* dscoreE_lo,
                                 int64_t ldS, void* dQ, hipStream_t st) {
  AttnFwdArgs p{};
  p.q_hi = reinterpret_cast<const uint16_t*>(dC_hi);
  p.q_lo = reinterpret_cast<const uint16_t*>(dC_lo);
  p.h_enc = reinterpret_cast<const uint16_t*>(h_enc);
  p.src_len = src_len;
  p.alpha32 = const_cast<float*>(alpha32);
  p.alphaE = reinterpret_cast<uint16_t*>(dscoreE);
  p.alphaE_lo = reinterpret_cast<uint16_t*>(dscoreE_lo);
  p.ctx = reinterpret_cast<uint16_t*>(dQ);
  p.ctx_lo = nullptr;
  p.attn_mask = nullptr;
  p.T = T; p.S = S; p.B = B; p.H = H;
  p.ldS = ldS;
  return launch_attn_fused(true, p, st);
}

}  // namespace asx
