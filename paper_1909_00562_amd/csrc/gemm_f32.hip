// fp32 matrix products for the AS_F32 path (fp32 operands, products summed in
// fp64 so that each output is rounded once; plain FMA arithmetic, LDS tiled),
// the split-K combine kernel shared with the bf16 path, and the tile planner.
#include "common.h"
#include "gemm.h"

namespace asx {

struct GemmDevF {
  const float* A[kMaxSeg];
  const float* B[kMaxSeg];
  int64_t sam[kMaxSeg], sak[kMaxSeg], sbn[kMaxSeg], sbk[kMaxSeg];  // element strides of A(m,k), B(n,k)
  int64_t sA[kMaxSeg], sB[kMaxSeg];
  int K[kMaxSeg];
  int M, N;
  float* C;
  float* C_lo;
  float* C_dact;
  int64_t ldc, sC;
  const float* bias;
  const float* gate;
  int64_t ldg;
  int act_tanh, accumulate;
  uint32_t drop_thr;
  float drop_scale;
  uint64_t drop_seed;
  int splits;
  float* partial;
  int kper;
  int a_kc, b_kc;
  const int32_t* M_dev;   // device-side row count / reduction length (or null), clamped to M / K[0]
  const int32_t* K_dev;
};

__device__ __forceinline__ int dev_bound_f(const int32_t* count, int bound) {
  if (!count) return bound;
  const int v = *count;
  return v < 0 ? 0 : (v < bound ? v : bound);
}

constexpr int FT = 64;   // block tile edge
constexpr int FK = 16;   // reduction slice

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmDevF p) {
  __shared__ float As[FK][FT + 4];
  __shared__ float Bs[FK][FT + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * FT, n0 = blockIdx.x * FT;
  const int Mv = dev_bound_f(p.M_dev, p.M);
  const int K0 = dev_bound_f(p.K_dev, p.K[0]);
  if (m0 >= Mv) return;   // the whole block, before any barrier
  const int kper = p.K_dev ? (((K0 + FK - 1) / FK + p.splits - 1) / p.splits) * FK : p.kper;
  const int z = blockIdx.z;
  const int batch = z / p.splits, split = z - batch * p.splits;

  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

  for (int seg = 0; seg < kMaxSeg; ++seg) {
    if (p.K[seg] <= 0) continue;
    int kbeg = 0, kend = seg == 0 ? K0 : p.K[seg];
    if (p.splits > 1) {
      kbeg = split * kper;
      kend = kbeg + kper < kend ? kbeg + kper : kend;
    }
    const float* A = p.A[seg] + (int64_t)batch * p.sA[seg];
    const float* B = p.B[seg] + (int64_t)batch * p.sB[seg];
    for (int k0 = kbeg; k0 < kend; k0 += FK) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int idx = tid + 256 * j;
        int m, k;
        if (p.a_kc) { k = idx & 15; m = idx >> 4; } else { m = idx & 63; k = idx >> 6; }
        const int gm = m0 + m, gk = k0 + k;
        As[k][m] = (gm < Mv && gk < kend) ? A[(int64_t)gm * p.sam[seg] + (int64_t)gk * p.sak[seg]] : 0.f;
        int n;
        if (p.b_kc) { k = idx & 15; n = idx >> 4; } else { n = idx & 63; k = idx >> 6; }
        const int gn = n0 + n;
        const int gk2 = k0 + k;
        Bs[k][n] = (gn < p.N && gk2 < kend) ? B[(int64_t)gn * p.sbn[seg] + (int64_t)gk2 * p.sbk[seg]] : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < FK; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fma((double)a[i], (double)b[j], acc[i][j]);
      }
      __syncthreads();
    }
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + ty * 4 + i;
    if (row >= Mv) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col >= p.N) continue;
      double v = acc[i][j];
      if (p.splits > 1) {
        p.partial[((int64_t)z * p.M + row) * p.N + col] = (float)v;
        continue;
      }
      if (p.bias) v += (double)p.bias[col];
      if (p.act_tanh) v = tanh(v);
      double dact = 1.0 - v * v;
      if (p.drop_thr) {
        const double s = (double)dropout_mult((uint64_t)row * p.N + col, p.drop_seed, p.drop_thr, p.drop_scale);
        v *= s;
        dact *= s;
      }
      if (p.gate) v *= (double)p.gate[(int64_t)row * p.ldg + col];
      const int64_t ci = (int64_t)batch * p.sC + (int64_t)row * p.ldc + col;
      if (p.accumulate) v += (double)p.C[ci];
      const float vf = (float)v;
      p.C[ci] = vf;
      if (p.C_lo) p.C_lo[ci] = (float)(v - (double)vf);
      if (p.C_dact) p.C_dact[ci] = (float)dact;
    }
  }
}

hipError_t launch_gemm_f32(const GemmArgs& g, hipStream_t st) {
  if (g.M < 1 || g.N < 1 || g.batch < 1 || g.splits < 1 || g.c_bf16) return hipErrorInvalidValue;
  if (g.splits > 1 && (g.K[1] != 0 || g.partial == nullptr)) return hipErrorInvalidValue;
  if (g.splits > 1 && (g.C_dact || g.drop_thr)) return hipErrorInvalidValue;
  if (g.drop_thr && g.batch != 1) return hipErrorInvalidValue;
  GemmDevF d;
  for (int s = 0; s < kMaxSeg; ++s) {
    d.A[s] = reinterpret_cast<const float*>(g.A[s]);
    d.B[s] = reinterpret_cast<const float*>(g.B[s]);
    d.sam[s] = g.a_kc ? g.lda[s] : 1;
    d.sak[s] = g.a_kc ? 1 : g.lda[s];
    d.sbn[s] = g.b_kc ? g.ldb[s] : 1;
    d.sbk[s] = g.b_kc ? 1 : g.ldb[s];
    d.sA[s] = g.sA[s];
    d.sB[s] = g.sB[s];
    d.K[s] = g.K[s];
  }
  d.M = g.M;
  d.N = g.N;
  d.C = reinterpret_cast<float*>(g.C);
  d.C_lo = reinterpret_cast<float*>(g.C_lo);
  d.C_dact = g.C_dact;
  d.ldc = g.ldc;
  d.sC = g.sC;
  d.bias = reinterpret_cast<const float*>(g.bias);
  d.gate = g.gate;
  d.ldg = g.ldg;
  d.act_tanh = g.act_tanh;
  d.drop_thr = g.drop_thr;
  d.drop_scale = g.drop_scale;
  d.drop_seed = g.drop_seed;
  d.accumulate = g.accumulate;
  d.splits = g.splits;
  d.partial = g.partial;
  d.a_kc = g.a_kc;
  d.b_kc = g.b_kc;
  if (g.M_dev && g.batch != 1) return hipErrorInvalidValue;
  if (g.K_dev && g.K[1] != 0) return hipErrorInvalidValue;
  d.M_dev = g.M_dev;
  d.K_dev = g.K_dev;
  const int ktiles = (g.K[0] + FK - 1) / FK;
  d.kper = ((ktiles + g.splits - 1) / g.splits) * FK;
  if (g.splits > 1 && (int64_t)d.kper * (g.splits - 1) >= g.K[0]) return hipErrorInvalidValue;
  dim3 grid((g.N + FT - 1) / FT, (g.M + FT - 1) / FT, g.batch * g.splits);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, d);
  return hipGetLastError();
}

// ---- split-K combine: C = epilogue(sum_s partial[b*splits+s]) in fixed order --
template <typename TIn, bool OUT_BF16>
__global__ __launch_bounds__(256) void splitk_combine_kernel(const float* __restrict__ partial, int splits,
                                                            int M, int N, void* C, void* C_lo, int64_t ldc,
                                                            int64_t sC, const TIn* bias, const float* gate,
                                                            int64_t ldg, int act_tanh, int accumulate,
                                                            float* C_dact, uint32_t drop_thr, float drop_scale,
                                                            uint64_t drop_seed, const int32_t* M_dev,
                                                            int dyn_ktiles, int dyn_blocks) {
  const int64_t mn = (int64_t)M * N;      // extent of one partial
  const int Mv = dev_bound_f(M_dev, M);
  const int64_t mn_valid = (int64_t)Mv * N;   // rows the product wrote
  if (dyn_ktiles > 0)   // the product chose its split from the row count: the same choice here
    splits = pp_dyn_splits(((Mv + 255) / 256) * ((N + 255) / 256), dyn_ktiles, splits, dyn_blocks);
  const int batch = blockIdx.y;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < mn_valid; i += (int64_t)gridDim.x * 256) {
    const int row = (int)(i / N), col = (int)(i - (int64_t)row * N);
    const float* P = partial + (int64_t)batch * splits * mn + i;
    float v = 0.f;
    for (int s = 0; s < splits; ++s) v += P[(int64_t)s * mn];
    if (bias) v += ld_elem<TIn>(bias, col);
    if (act_tanh) v = tanhf(v);
    float dact = 1.f - v * v;
    if (drop_thr) {
      const float sc = dropout_mult((uint64_t)i, drop_seed, drop_thr, drop_scale);   // i = row * N + col
      v *= sc;
      dact *= sc;
    }
    if (gate) v *= gate[(int64_t)row * ldg + col];
    const int64_t ci = (int64_t)batch * sC + (int64_t)row * ldc + col;
    if (C_dact) C_dact[ci] = dact;
    if constexpr (OUT_BF16) {
      const uint32_t hi = f32_to_bf16_bits(v);
      reinterpret_cast<uint16_t*>(C)[ci] = (uint16_t)hi;
      if (C_lo) reinterpret_cast<uint16_t*>(C_lo)[ci] = (uint16_t)f32_to_bf16_bits(v - bf16_bits_to_f32(hi));
    } else {
      float* Cf = reinterpret_cast<float*>(C);
      if (accumulate) v += Cf[ci];
      Cf[ci] = v;
      if (C_lo) reinterpret_cast<float*>(C_lo)[ci] = 0.f;   // partial sums were already rounded to fp32
    }
  }
}

hipError_t launch_splitk_combine(const GemmArgs& g, bool in_bf16, hipStream_t st) {
  const int64_t mn = (int64_t)g.M * g.N;
  // a split chosen by the persistent kernel (dyn_split): its reduction tiles and its grid, as that launch had them
  const int dyn_ktiles = g.dyn_split ? (g.K[0] + 63) / 64 : 0;
  const int dyn_blocks = g.dyn_split ? pp_grid_blocks(((g.M + 255) / 256) * ((g.N + 255) / 256) * g.splits) : 0;
  int blocks = (int)((mn + 255) / 256);
  if (blocks > 8192) blocks = 8192;
  dim3 grid(blocks, g.batch);
  if (in_bf16) {
    const uint16_t* bias = reinterpret_cast<const uint16_t*>(g.bias);
    const float* gate = g.gate;
    if (g.c_bf16)
      hipLaunchKernelGGL((splitk_combine_kernel<uint16_t, true>), grid, dim3(256), 0, st, g.partial, g.splits,
                         g.M, g.N, g.C, g.C_lo, g.ldc, g.sC, bias, gate, g.ldg, g.act_tanh, g.accumulate, g.C_dact,
                         g.drop_thr, g.drop_scale, g.drop_seed, g.M_dev, dyn_ktiles, dyn_blocks);
    else
      hipLaunchKernelGGL((splitk_combine_kernel<uint16_t, false>), grid, dim3(256), 0, st, g.partial, g.splits,
                         g.M, g.N, g.C, g.C_lo, g.ldc, g.sC, bias, gate, g.ldg, g.act_tanh, g.accumulate, g.C_dact,
                         g.drop_thr, g.drop_scale, g.drop_seed, g.M_dev, dyn_ktiles, dyn_blocks);
  } else {
    hipLaunchKernelGGL((splitk_combine_kernel<float, false>), grid, dim3(256), 0, st, g.partial, g.splits, g.M,
                       g.N, g.C, g.C_lo, g.ldc, g.sC, reinterpret_cast<const float*>(g.bias),
                       g.gate, g.ldg, g.act_tanh, g.accumulate, g.C_dact, g.drop_thr, g.drop_scale, g.drop_seed,
                       g.M_dev, dyn_ktiles, dyn_blocks);
  }
  return hipGetLastError();
}

// ---- planner ----------------------------------------------------------------
// Cost model (seconds) used to pick the block tile and the reduction split of a bf16
// product on a 256-CU part: blocks run in rounds of `slots` (one 256x256 block or
// two 128x128 blocks per CU); a round costs the block's flops at the per-CU rate
// the kernel sustains plus a fixed prologue/epilogue; a split adds the round trip
// of its fp32 partial sums through HBM and one more launch.
static double plan_cost(int M, int N, int K, int batch, int tile, int splits) {
  const double cus = 256.0;
  const double rate = tile == 256 ? 3.9e12 : 1.35e12;      // flop/s of one resident block
  const double slots = tile == 256 ? cus : 2.0 * cus;
  const double fixed = tile == 256 ? 8e-6 : 5e-6;
  const double blocks = (double)((M + tile - 1) / tile) * ((N + tile - 1) / tile) * batch * splits;
  const double rounds = (double)(int64_t)((blocks + slots - 1) / slots);
  const double kblk = (double)((K + splits - 1) / splits);
  double t = rounds * (2.0 * tile * tile * kblk / rate + fixed);
  if (splits > 1) t += 2.0 * splits * (double)M * N * batch * 4.0 / 4e12 + 8e-6;
  return t;
}

GemmPlan gemm_plan(int M, int N, int K, int batch, bool bf16, bool allow_split, bool multi_segment) {
  GemmPlan pl;
  pl.big_tile = 0;
  pl.splits = 1;
  if (!bf16) {
    if (multi_segment) allow_split = false;
    // fp32 path: plain 64x64 tiles; split only to fill the machine
    const int64_t tiles = (int64_t)((M + FT - 1) / FT) * ((N + FT - 1) / FT) * batch;
    if (allow_split && tiles < 384) {
      const int ktiles = (K + FK - 1) / FK;
      int64_t want = (768 + tiles - 1) / tiles;
      const int64_t cap = ktiles / 16;
      if (want > cap) want = cap;
      if (want > 32) want = 32;
      if (want > 1) {
        const int per = (int)((ktiles + want - 1) / want);
        pl.splits = (ktiles + per - 1) / per;
      }
    }
    return pl;
  }
  const int ktiles = (K + 63) / 64;
  double best = 1e30;
  for (int tile = 128; tile <= 256; tile += 128) {
    if (tile == 256 && (M < 192 || N < 192)) continue;   // most of a 256-row tile would be padding
    const int smax = allow_split ? (ktiles / 4 < 32 ? (ktiles / 4 > 1 ? ktiles / 4 : 1) : 32) : 1;
    for (int want = 1; want <= smax; ++want) {
      const int per = (ktiles + want - 1) / want;
      const int s = (ktiles + per - 1) / per;            // no empty split
      if (s != want) continue;
      if (tile == 256 && s > 1 && multi_segment) continue;
      const double c = plan_cost(M, N, K, batch, tile, s);
      if (c < best) {
        best = c;
        pl.big_tile = tile == 256;
        pl.splits = s;
      }
    }
  }
  return pl;
}

hipError_t launch_gemm(const GemmArgs& g, bool in_bf16, int big_tile, hipStream_t st) {
  hipError_t e = in_bf16 ? launch_gemm_bf16(g, big_tile, st) : launch_gemm_f32(g, st);
  if (e != hipSuccess) return e;
  if (g.splits > 1) e = launch_splitk_combine(g, in_bf16, st);
  return e;
}

}  // namespace asx
