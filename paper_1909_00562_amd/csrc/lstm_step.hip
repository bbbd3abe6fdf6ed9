// One time step of an LSTM layer as ONE kernel on the bf16 matrix cores (gfx950):
// the recurrent product and the cell (forward), or the product da_{t+1} W_hh and the
// cell derivative (backward), cell as stated in include/lstm_stack.h.
//
// A step is a skinny product (B rows, typically 128) that sits on the critical path
// T times per layer, so it is built for latency, not for reuse:
//   * no LDS staging: every wave loads its MFMA fragments (8 consecutive reduction
//     elements per lane, 16 bytes) straight from L2 into registers.  For that to be
//     coalesced both operands are kept FRAGMENT-MAJOR, [K/8][rows][8]: the 32 lanes
//     that hold the 32 rows of a fragment read 512 contiguous bytes (a row-major
//     operand would make every lane touch a cache line of its own: measured 20 us
//     per forward step against 13 with nothing else changed).  The weights are put into that form once per call and
//     layer; the state and the gate gradients are written in it by the step before;
//   * the reduction is split over the waves of a block (interleaved 16-wide steps, so
//     neighbouring waves read neighbouring 32-byte pieces of the same cache lines) and
//     the partial 32x32 tiles are added through LDS in a fixed order;
//   * the matrix operand is the WEIGHT slice (MFMA rows) and the batch is the MFMA
//     column: a lane then holds, for its sentence, four consecutive rows of the
//     output tile.  Forward, the rows of a tile are ordered so that these are the
//     four gates i, f, g, o of one hidden unit, and a lane's sixteen values are the
//     gates of four consecutive units: the whole cell is lane-local and every access
//     to c, h and the saved gates is a 16-byte (fp32) or 8-byte (bf16) vector.
//   * forward, h comes as a (value, rounding remainder) bf16 pair that shares the
//     weight fragment (two MFMAs per weight load): without the remainder bf16 rounding
//     compounds over the steps and the layers.  Backward, the gate gradients enter the
//     recurrent product as plain bf16 (measured: worst element 0.51 of the tolerance
//     instead of 0.40 at 50 steps x 4 layers, for 15 % of the backward time); the large
//     products that follow still take their remainders.
#include "common.h"
#include "kernels.h"

namespace asx {

typedef uint32_t ls_u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t ls_u32x2_t __attribute__((ext_vector_type(2)));

// 8 consecutive bf16 (one MFMA fragment of a lane), or zeros
__device__ __forceinline__ bf16x8_t ls_frag(const uint16_t* p, bool ok) {
  ls_u32x4_t q = {0u, 0u, 0u, 0u};
  if (ok) q = *reinterpret_cast<const ls_u32x4_t*>(p);
  return __builtin_bit_cast(bf16x8_t, q);
}
__device__ __forceinline__ float ls_sigmoid(float a) { return 1.f / (1.f + expf(-a)); }
__device__ __forceinline__ ls_u32x2_t ls_pack4(const float (&v)[4]) {
  ls_u32x2_t r = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
  return r;
}
__device__ __forceinline__ void ls_split4(const float (&v)[4], ls_u32x2_t& hi, ls_u32x2_t& lo) {
  float l[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) l[e] = v[e] - bf16_bits_to_f32(f32_to_bf16_bits(v[e]));
  hi = ls_pack4(v);
  lo = ls_pack4(l);
}
__device__ __forceinline__ int ls_len(const int32_t* lengths, int b, int T) {
  const int n = lengths[b];
  return n < 0 ? 0 : (n > T ? T : n);
}

// ---- forward ---------------------------------------------------------------------
// Block: 64 gate rows (16 hidden units x 4 gates) x 32*LSF_NJ sentences, LSF_KS waves splitting the reduction over H.
// MFMA row rho of a 32-row tile that starts at unit u: unit u + 4*((rho >> 2) & 1) + (rho >> 3), gate rho & 3,
// i.e. weight row gate*H + unit; output register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, so the lane
// holds units u + 4*(l/32) + r/4 (r/4 = 0..3), gate r%4.
constexpr int LSF_NJ = 1;    // 32-sentence column tiles per block
constexpr int LSF_KS = 8;    // waves per block = ways the reduction is split
constexpr int LSF_U = 8;     // reduction steps whose loads are in flight together
constexpr int LSF_SMEM = LSF_KS * 2 * LSF_NJ * 16 * 64 * 4;
static_assert(2 * LSF_NJ <= LSF_KS, "one wave per output tile finishes it");

__global__ __launch_bounds__(64 * LSF_KS) void lstm_step_fwd_kernel(LstmStepFwd p) {
  constexpr int NJ = LSF_NJ;
  extern __shared__ float red[];   // [wave][tile*16 + r][lane]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rho = lane & 31, kq = lane >> 5;
  const int u0 = blockIdx.x * 16, b0 = blockIdx.y * 32 * NJ;
  const int H = p.H, B = p.B;

  // element offsets inside one 8-wide reduction chunk of the fragment-major operands
  int64_t woff[2], hoff[NJ];
  bool wok[2], bok[NJ];
#pragma unroll
  for (int i = 0; i < 2; ++i) {   // WF rows are ordered unit*4 + gate: the 32 rows of a tile are contiguous
    wok[i] = u0 + 8 * i < H;      // H % 8 == 0: a tile of 8 units is all inside or all outside
    woff[i] = ((int64_t)(u0 + 8 * i) * 4 + 16 * ((rho >> 2) & 1) + 4 * (rho >> 3) + (rho & 3)) * 8;
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int b = b0 + 32 * j + rho;
    bok[j] = b < B;
    hoff[j] = (int64_t)(bok[j] ? b : 0) * 8;
  }
  const int64_t wchunk = (int64_t)4 * H * 8, hchunk = (int64_t)B * 8;   // elements per chunk of WF / hF
  const int nchunks = H / 8;

  // What the wave that finishes an output tile needs from memory is requested now, ahead of the product:
  // the step is a chain of memory latencies, and this one would otherwise sit at its very end.
  constexpr int NT = 2 * NJ;   // output tiles of the block; wave w < NT finishes tile w = (i, j)
  const int ti = wave / NJ, tj = wave % NJ;
  const int b = b0 + 32 * tj + rho;
  const int unit0 = u0 + 8 * ti + 4 * kq;   // this lane: units unit0 .. unit0 + 3 (H % 4 == 0: all in or all out)
  const bool fin = wave < NT && b < B && unit0 < H;
  const int64_t idx = (int64_t)(fin ? b : 0) * H + (fin ? unit0 : 0);
  float* Gp = p.G + (int64_t)(fin ? b : 0) * 4 * H + (fin ? unit0 : 0);
  f32x4_t gx[4], cp;
  if (fin) {
#pragma unroll
    for (int g = 0; g < 4; ++g) gx[g] = *reinterpret_cast<const f32x4_t*>(Gp + (int64_t)g * H);
    cp = *reinterpret_cast<const f32x4_t*>(p.c_prev + idx);
  }
  f32x16_t acc[2][NJ];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // The step is bound by the latency of its loads (one wave per SIMD, everything comes from L2 or beyond):
  // the fragments of LSF_U reduction steps are requested before the first of them is used.
  const int nks = (H + 15) / 16;
  for (int ks0 = wave; ks0 < nks; ks0 += LSF_KS * LSF_U) {
    bf16x8_t wf[LSF_U][2], hf[LSF_U][NJ], lf[LSF_U][NJ];
#pragma unroll
    for (int u = 0; u < LSF_U; ++u) {
      const int kc = (ks0 + u * LSF_KS) * 2 + kq;   // this lane's chunk of the 16-wide step
      const bool kin = kc < nchunks;
#pragma unroll
      for (int i = 0; i < 2; ++i) wf[u][i] = ls_frag(p.WF + kc * wchunk + woff[i], kin && wok[i]);
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        hf[u][j] = ls_frag(p.hF_hi + kc * hchunk + hoff[j], kin && bok[j]);
        lf[u][j] = ls_frag(p.hF_lo + kc * hchunk + hoff[j], kin && bok[j]);
      }
    }
#pragma unroll
    for (int u = 0; u < LSF_U; ++u)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u][i], hf[u][j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u][i], lf[u][j], acc[i][j], 0, 0, 0);
        }
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[((wave * NT + i * NJ + j) * 16 + r) * 64 + lane] = acc[i][j][r];
  __syncthreads();
  if (!fin) return;

  // partial sums added in wave order
  float v[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < LSF_KS; ++w) s += red[((w * NT + wave) * 16 + r) * 64 + lane];
    v[r] = s;
  }
  const bool valid = p.t < ls_len(p.lengths, b, p.T);
  f32x4_t gi, gf, gg, go, cn;
  float hn[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    gi[q] = ls_sigmoid(v[4 * q + 0] + gx[0][q]);
    gf[q] = ls_sigmoid(v[4 * q + 1] + gx[1][q]);
    gg[q] = tanhf(v[4 * q + 2] + gx[2][q]);
    go[q] = ls_sigmoid(v[4 * q + 3] + gx[3][q]);
    cn[q] = gf[q] * cp[q] + gi[q] * gg[q];
    hn[q] = go[q] * tanhf(cn[q]);
  }
  *reinterpret_cast<f32x4_t*>(Gp) = gi;
  *reinterpret_cast<f32x4_t*>(Gp + (int64_t)H) = gf;
  *reinterpret_cast<f32x4_t*>(Gp + 2 * (int64_t)H) = gg;
  *reinterpret_cast<f32x4_t*>(Gp + 3 * (int64_t)H) = go;
  const ls_u32x2_t zero2 = {0u, 0u};
  const int64_t fidx = ((int64_t)(unit0 >> 3) * B + b) * 8 + (unit0 & 7);   // the same four units, fragment-major
  if (valid) {
    *reinterpret_cast<f32x4_t*>(p.c_new + idx) = cn;
    const f32x4_t h4 = {hn[0], hn[1], hn[2], hn[3]};
    *reinterpret_cast<f32x4_t*>(p.hf + idx) = h4;
    ls_u32x2_t hi, lo;
    ls_split4(hn, hi, lo);
    *reinterpret_cast<ls_u32x2_t*>(p.hE_new + idx) = hi;
    *reinterpret_cast<ls_u32x2_t*>(p.hFn_hi + fidx) = hi;
    *reinterpret_cast<ls_u32x2_t*>(p.hFn_lo + fidx) = lo;
    if (p.drop_thr) {   // what the next layer reads: the lane's four units are one block of the generator
      uint32_t w[4];
      dropout_words4((p.drop_index0 + (uint64_t)idx) >> 2, p.drop_seed, w);
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = w[e] >= p.drop_thr ? hn[e] * p.drop_scale : 0.f;
      ls_split4(o, hi, lo);
    }
    *reinterpret_cast<ls_u32x2_t*>(p.out + idx) = hi;
    if (p.out_lo) *reinterpret_cast<ls_u32x2_t*>(p.out_lo + idx) = lo;
  } else {   // padded step: the state passes through, the layer's output is 0
    *reinterpret_cast<f32x4_t*>(p.c_new + idx) = cp;
    *reinterpret_cast<ls_u32x2_t*>(p.hE_new + idx) = *reinterpret_cast<const ls_u32x2_t*>(p.hF_hi + fidx);
    *reinterpret_cast<ls_u32x2_t*>(p.hFn_hi + fidx) = *reinterpret_cast<const ls_u32x2_t*>(p.hF_hi + fidx);
    *reinterpret_cast<ls_u32x2_t*>(p.hFn_lo + fidx) = *reinterpret_cast<const ls_u32x2_t*>(p.hF_lo + fidx);
    *reinterpret_cast<ls_u32x2_t*>(p.out + idx) = zero2;
    if (p.out_lo) *reinterpret_cast<ls_u32x2_t*>(p.out_lo + idx) = zero2;
  }
}

// ---- backward --------------------------------------------------------------------
// Block: 32 hidden units x 32 sentences, 8 waves splitting the reduction over the 4H gate rows of step t+1:
// rec[b,u] = sum_n da_{t+1}[b,n] W_hh[n,u] (weights read from the transposed copy WT [H,4H]).  The gradient
// w.r.t. h_t is rec where step t+1 was a word of sentence b, else the gradient that came in for the final
// state (sentences are right-padded, so the steps of a sentence are a prefix).  Then the cell derivative of
// step t.  t = -1: only the product, written out as the gradient of the initial state.
constexpr int LSB_KS = 8;
constexpr int LSB_U = 8;     // reduction steps whose loads are in flight together (2 fragments each)
constexpr int LSB_SMEM = LSB_KS * 16 * 64 * 4;

__global__ __launch_bounds__(64 * LSB_KS) void lstm_step_bwd_kernel(LstmStepBwd p) {
  extern __shared__ float red[];   // [wave][r][lane]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rho = lane & 31, kq = lane >> 5;
  const int u0 = blockIdx.x * 32, b0 = blockIdx.y * 32;
  const int H = p.H, B = p.B, K = 4 * p.H;

  // the inputs of the cell derivative are requested ahead of the product (waves 0..3 finish the tile)
  const int b = b0 + rho;
  const int unit0 = u0 + 8 * (wave & 3) + 4 * kq;
  const bool fin = wave < 4 && b < B && unit0 < H;
  const int64_t idx = (int64_t)(fin ? b : 0) * H + (fin ? unit0 : 0);
  const int len = fin ? ls_len(p.lengths, b, p.T) : 0;
  const bool cell = fin && p.t >= 0 && p.t < len;
  f32x4_t gi, gf, gg, go, cp, cn, dy, dcs, carried = {0.f, 0.f, 0.f, 0.f};
  if (fin && p.dhT) carried = *reinterpret_cast<const f32x4_t*>(p.dhT + idx);
  if (cell) {
    const float* Gp = p.gates + (int64_t)b * K + unit0;
    gi = *reinterpret_cast<const f32x4_t*>(Gp);
    gf = *reinterpret_cast<const f32x4_t*>(Gp + (int64_t)H);
    gg = *reinterpret_cast<const f32x4_t*>(Gp + 2 * (int64_t)H);
    go = *reinterpret_cast<const f32x4_t*>(Gp + 3 * (int64_t)H);
    cp = *reinterpret_cast<const f32x4_t*>(p.c_prev + idx);
    cn = *reinterpret_cast<const f32x4_t*>(p.c_new + idx);
    dy = *reinterpret_cast<const f32x4_t*>(p.dout_t + idx);
    dcs = *reinterpret_cast<const f32x4_t*>(p.dcs + idx);
    if (p.drop_thr) {   // back through the mask the forward step put on this layer's output
      uint32_t w[4];
      dropout_words4((p.drop_index0 + (uint64_t)idx) >> 2, p.drop_seed, w);
#pragma unroll
      for (int e = 0; e < 4; ++e) dy[e] = w[e] >= p.drop_thr ? dy[e] * p.drop_scale : 0.f;
    }
  }

  f32x16_t acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  if (p.dGnF) {
    const int unit = u0 + rho, bb = b0 + rho;
    const bool wok = unit < H, bok = bb < B;
    const int64_t woff = (int64_t)(wok ? unit : 0) * 8, goff = (int64_t)(bok ? bb : 0) * 8;
    const int64_t wchunk = (int64_t)H * 8, gchunk = (int64_t)B * 8;   // elements per 8-wide chunk of WTF / dGF
    const int nchunks = K / 8;
    const int nks = K / 16;   // H % 8 == 0: 4H is a multiple of 32
    for (int ks0 = wave; ks0 < nks; ks0 += LSB_KS * LSB_U) {   // loads of LSB_U steps in flight together
      bf16x8_t wf[LSB_U], gf[LSB_U];
#pragma unroll
      for (int u = 0; u < LSB_U; ++u) {
        const int kc = (ks0 + u * LSB_KS) * 2 + kq;
        const bool kin = kc < nchunks;
        wf[u] = ls_frag(p.WTF + kc * wchunk + woff, kin && wok);
        gf[u] = ls_frag(p.dGnF + kc * gchunk + goff, kin && bok);
      }
#pragma unroll
      for (int u = 0; u < LSB_U; ++u) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u], gf[u], acc, 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) red[(wave * 16 + r) * 64 + lane] = acc[r];
  __syncthreads();
  if (!fin) return;               // waves 0..3 finish four consecutive units each (register group r/4 = wave)
  float rec[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < LSB_KS; ++w) s += red[(w * 16 + 4 * wave + e) * 64 + lane];
    rec[e] = s;
  }
  const bool valid_next = p.t + 1 < len;
  f32x4_t dh;
#pragma unroll
  for (int e = 0; e < 4; ++e) dh[e] = valid_next ? rec[e] : carried[e];
  if (p.t < 0) {
    *reinterpret_cast<f32x4_t*>(p.dh0_out + idx) = dh;
    return;
  }
  uint16_t* dhi = p.dG_hi + (int64_t)b * K + unit0;
  uint16_t* dlo = p.dG_lo + (int64_t)b * K + unit0;
  if (cell) {
    float da[4][4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float d = dy[e] + dh[e];
      const float tc = tanhf(cn[e]);
      const float dc = dcs[e] + d * go[e] * (1.f - tc * tc);
      da[0][e] = dc * gg[e] * gi[e] * (1.f - gi[e]);
      da[1][e] = dc * cp[e] * gf[e] * (1.f - gf[e]);
      da[2][e] = dc * gi[e] * (1.f - gg[e] * gg[e]);
      da[3][e] = d * tc * go[e] * (1.f - go[e]);
      dcs[e] = dc * gf[e];
    }
    *reinterpret_cast<f32x4_t*>(p.dcs + idx) = dcs;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      ls_u32x2_t hi, lo;
      ls_split4(da[g], hi, lo);
      const int n0 = g * H + unit0;   // gate row of the first of the four units
      const int64_t fidx = ((int64_t)(n0 >> 3) * B + b) * 8 + (n0 & 7);
      *reinterpret_cast<ls_u32x2_t*>(dhi + (int64_t)g * H) = hi;
      *reinterpret_cast<ls_u32x2_t*>(dlo + (int64_t)g * H) = lo;
      *reinterpret_cast<ls_u32x2_t*>(p.dGF + fidx) = hi;
    }
  } else {
    const ls_u32x2_t zero2 = {0u, 0u};
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n0 = g * H + unit0;
      const int64_t fidx = ((int64_t)(n0 >> 3) * B + b) * 8 + (n0 & 7);
      *reinterpret_cast<ls_u32x2_t*>(dhi + (int64_t)g * H) = zero2;
      *reinterpret_cast<ls_u32x2_t*>(dlo + (int64_t)g * H) = zero2;
      *reinterpret_cast<ls_u32x2_t*>(p.dGF + fidx) = zero2;
    }
  }
}

// Weights of one layer into fragment-major form, 16 bytes per thread.
// Forward: WF[kc][unit*4 + gate][e] = W_hh[gate*H + unit][8*kc + e]   (a straight copy of 16-byte pieces)
__global__ __launch_bounds__(256) void ls_wfrag_fwd_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ WF,
                                                          int H) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over (kc, row')
  const int64_t n = (int64_t)(H / 8) * 4 * H;
  if (i >= n) return;
  const int kc = (int)(i / (4 * H)), rp = (int)(i - (int64_t)kc * 4 * H);
  const int unit = rp >> 2, gate = rp & 3;
  *reinterpret_cast<ls_u32x4_t*>(WF + i * 8) =
      *reinterpret_cast<const ls_u32x4_t*>(W + ((int64_t)gate * H + unit) * H + 8 * kc);
}
// Backward: WTF[kc][unit][e] = W_hh[8*kc + e][unit]   (8 x 8 blocks transposed in registers)
__global__ __launch_bounds__(256) void ls_wfrag_bwd_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ WTF,
                                                          int H) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over (kc, unit)
  const int64_t n = (int64_t)(4 * H / 8) * H;
  if (i >= n) return;
  const int kc = (int)(i / H), unit = (int)(i - (int64_t)kc * H);
  uint32_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = W[((int64_t)8 * kc + e) * H + unit];   // coalesced over `unit`
  const ls_u32x4_t q = {v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
  *reinterpret_cast<ls_u32x4_t*>(WTF + i * 8) = q;
}

hipError_t launch_lstm_step_fwd(const LstmStepFwd& p, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(lstm_step_fwd_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LSF_SMEM);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if ((p.H & 7) != 0 || p.B < 1) return hipErrorInvalidValue;
  dim3 grid((p.H + 15) / 16, (p.B + 32 * LSF_NJ - 1) / (32 * LSF_NJ));
  hipLaunchKernelGGL(lstm_step_fwd_kernel, grid, dim3(64 * LSF_KS), LSF_SMEM, st, p);
  return hipGetLastError();
}

hipError_t launch_lstm_step_bwd(const LstmStepBwd& p, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(lstm_step_bwd_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LSB_SMEM);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if ((p.H & 7) != 0 || p.B < 1) return hipErrorInvalidValue;   // 4H is then a multiple of 32: whole 16-wide steps
  dim3 grid((p.H + 31) / 32, (p.B + 31) / 32);
  hipLaunchKernelGGL(lstm_step_bwd_kernel, grid, dim3(64 * LSB_KS), LSB_SMEM, st, p);
  return hipGetLastError();
}

hipError_t launch_ls_wfrag(const void* W_hh, void* dst, int H, bool backward, hipStream_t st) {
  if ((H & 7) != 0) return hipErrorInvalidValue;
  const int64_t n = (int64_t)(H / 8) * 4 * H;
  const dim3 grid((unsigned)((n + 255) / 256));
  if (backward)
    hipLaunchKernelGGL(ls_wfrag_bwd_kernel, grid, dim3(256), 0, st, reinterpret_cast<const uint16_t*>(W_hh),
                       reinterpret_cast<uint16_t*>(dst), H);
  else
    hipLaunchKernelGGL(ls_wfrag_fwd_kernel, grid, dim3(256), 0, st, reinterpret_cast<const uint16_t*>(W_hh),
                       reinterpret_cast<uint16_t*>(dst), H);
  return hipGetLastError();
}

}  // namespace asx
