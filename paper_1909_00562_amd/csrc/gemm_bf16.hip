// bf16 x bf16 -> fp32 matrix products on the CDNA4 matrix cores (gfx950).
//
// One kernel template covers the three operand orientations the path needs
// (both operands reduction-contiguous; B stored [K,N]; A and B stored [K,*]).
// Whatever the orientation in memory, a block tile lands in LDS as rows of 64
// reduction elements (128 bytes), 16-byte chunks XOR-swizzled by the row index
// so that both the tile stores and the 16-byte MFMA fragment reads are free of
// bank conflicts.  Operands whose reduction index is the strided one are
// transposed in registers (4 k-rows x 8 columns per lane, v_perm_b32) on their
// way from the global loads to LDS.  The main loop is double buffered in LDS
// with the next tile's global loads in flight during the MFMAs.
//
// Wave tiling: 256 threads = 2 x 2 waves, each wave owns (BM/2) x (BN/2) of the
// block tile as 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16, 8 reduction
// elements per lane per operand).
#include "common.h"
#include "gemm.h"

namespace asx {

struct GemmDev {
  const uint16_t* A[kMaxSeg];
  const uint16_t* B[kMaxSeg];
  int64_t lda[kMaxSeg], ldb[kMaxSeg], sA[kMaxSeg], sB[kMaxSeg];
  int K[kMaxSeg];
  int M, N;
  void* C;
  uint16_t* C_lo;
  float* C_dact;
  int64_t ldc, sC;
  const uint16_t* bias;
  const float* gate;
  int64_t ldg;
  int act_tanh, accumulate;
  int splits;
  float* partial;
  int tiles_m, tiles_n;
  int kper;  // reduction elements per split, multiple of 64
};

constexpr int BK = 64;          // reduction elements per LDS tile row
constexpr int ROWB = BK * 2;    // bytes per LDS tile row

// ---- global -> registers ---------------------------------------------------
template <int ROWS, bool KC>
__device__ __forceinline__ void tile_gload(uint4 (&r)[ROWS / 32], const uint16_t* __restrict__ X,
                                           int64_t ld, int row0, int R, int k0, int kend, int tid) {
  const uint4 zero = make_uint4(0, 0, 0, 0);
  if constexpr (KC) {
    const int c = tid & 7, rr = tid >> 3;
    const int gk = k0 + c * 8;
#pragma unroll
    for (int j = 0; j < ROWS / 32; ++j) {
      const int gr = row0 + rr + 32 * j;
      const bool ok = (gr < R) && (gk < kend);
      r[j] = ok ? *reinterpret_cast<const uint4*>(X + (int64_t)gr * ld + gk) : zero;
    }
  } else {
    const int lane = tid & 63, w = tid >> 6;
    const int kq = lane & 15, rb = w * 4 + (lane >> 4);
#pragma unroll
    for (int j = 0; j < ROWS / 128; ++j) {
      const int gr = row0 + (rb + 16 * j) * 8;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int gk = k0 + kq * 4 + kk;
        const bool ok = (gk < kend) && (gr < R);
        r[j * 4 + kk] = ok ? *reinterpret_cast<const uint4*>(X + (int64_t)gk * ld + gr) : zero;
      }
    }
  }
}

__device__ __forceinline__ uint32_t u4_get(const uint4& v, int i) {
  return i == 0 ? v.x : (i == 1 ? v.y : (i == 2 ? v.z : v.w));
}

// ---- registers -> LDS (swizzled, reduction-contiguous rows) -----------------
template <int ROWS, bool KC>
__device__ __forceinline__ void tile_sstore(const uint4 (&r)[ROWS / 32], unsigned char* base, int tid) {
  if constexpr (KC) {
    const int c = tid & 7, rr = tid >> 3;
#pragma unroll
    for (int j = 0; j < ROWS / 32; ++j) {
      const int row = rr + 32 * j;
      *reinterpret_cast<uint4*>(base + row * ROWB + ((c ^ (row & 7)) << 4)) = r[j];
    }
  } else {
    const int lane = tid & 63, w = tid >> 6;
    const int kq = lane & 15, rb = w * 4 + (lane >> 4);
    const int chunk = kq >> 1, half = kq & 1;
#pragma unroll
    for (int j = 0; j < ROWS / 128; ++j) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = (rb + 16 * j) * 8 + e;
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        const int dw = e >> 1;
        const uint32_t lo = __builtin_amdgcn_perm(u4_get(r[j * 4 + 1], dw), u4_get(r[j * 4 + 0], dw), sel);
        const uint32_t hi = __builtin_amdgcn_perm(u4_get(r[j * 4 + 3], dw), u4_get(r[j * 4 + 2], dw), sel);
        *reinterpret_cast<uint2*>(base + row * ROWB + ((chunk ^ e) << 4) + half * 8) = make_uint2(lo, hi);
      }
    }
  }
}

__device__ __forceinline__ bf16x8_t frag_read(const unsigned char* base, int row, int chunk) {
  return *reinterpret_cast<const bf16x8_t*>(base + row * ROWB + ((chunk ^ (row & 7)) << 4));
}

template <int BM, int BN, bool AKC, bool BKC, bool OUT_BF16>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmDev p) {
  constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
  constexpr int NA = BM / 32, NB = BN / 32;
  constexpr int STAGE = (BM + BN) * ROWB;
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // --- block -> tile: consecutive blocks go round-robin to the 8 XCDs, so give
  // each XCD a contiguous run of tiles, then walk tiles in groups of 8 tile
  // rows so that co-resident blocks share operand panels in their XCD's L2.
  const int nt = p.tiles_m * p.tiles_n;
  int pid = blockIdx.x;
  {
    const int xcd = pid & 7, idx = pid >> 3;
    const int per = nt >> 3, rem = nt & 7;
    pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  constexpr int GROUP = 8;
  const int gsize = GROUP * p.tiles_n;
  const int gid = pid / gsize;
  const int first_m = gid * GROUP;
  const int gm = (p.tiles_m - first_m) < GROUP ? (p.tiles_m - first_m) : GROUP;
  const int in_g = pid - gid * gsize;
  const int tile_m = first_m + in_g % gm, tile_n = in_g / gm;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int z = blockIdx.z;
  const int batch = z / p.splits, split = z - batch * p.splits;

  // reduction range of each segment (a split applies to a single segment only)
  int kbeg0 = 0, kend0 = p.K[0];
  if (p.splits > 1) {
    kbeg0 = split * p.kper;
    kend0 = kbeg0 + p.kper < p.K[0] ? kbeg0 + p.kper : p.K[0];
  }
  int nks[kMaxSeg];
  nks[0] = kend0 > kbeg0 ? (kend0 - kbeg0 + BK - 1) / BK : 0;
  int nk = nks[0];
#pragma unroll
  for (int s = 1; s < kMaxSeg; ++s) {
    nks[s] = (p.K[s] + BK - 1) / BK;
    nk += nks[s];
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[NA], rb[NB];

  auto issue = [&](int kt) {
    int seg = 0;
#pragma unroll
    for (int s = 0; s < kMaxSeg - 1; ++s)
      if (seg == s && kt >= nks[s]) {
        kt -= nks[s];
        seg = s + 1;
      }
    const int k0 = (seg == 0 ? kbeg0 : 0) + kt * BK;
    const int kend = seg == 0 ? kend0 : p.K[seg];
    const uint16_t* A = p.A[seg] + (int64_t)batch * p.sA[seg];
    const uint16_t* B = p.B[seg] + (int64_t)batch * p.sB[seg];
    tile_gload<BM, AKC>(ra, A, p.lda[seg], m0, p.M, k0, kend, tid);
    tile_gload<BN, BKC>(rb, B, p.ldb[seg], n0, p.N, k0, kend, tid);
  };
  auto commit = [&](int stage) {
    unsigned char* as = smem + stage * STAGE;
    tile_sstore<BM, AKC>(ra, as, tid);
    tile_sstore<BN, BKC>(rb, as + BM * ROWB, tid);
  };

  if (nk > 0) {
    issue(0);
    commit(0);
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    if (more) issue(kt + 1);
    const unsigned char* as = smem + (kt & 1) * STAGE;
    const unsigned char* bs = as + BM * ROWB;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8_t af[TM], bfr[TN];
      const int chunk = kk * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = frag_read(as, wm * WM + i * 32 + (lane & 31), chunk);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = frag_read(bs, wn * WN + j * 32 + (lane & 31), chunk);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) commit((kt + 1) & 1);
    __syncthreads();
  }

  // --- epilogue.  MFMA 32x32 output: register r of lane l holds
  // row 8*(r/4) + 4*(l/32) + r%4, column l%32 of the tile.
  const int col_l = lane & 31, row_l = (lane >> 5) * 4;
  if (p.splits > 1) {
    float* P = p.partial + (int64_t)z * p.M * p.N;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * WN + j * 32 + col_l;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm * WM + i * 32 + (r >> 2) * 8 + row_l + (r & 3);
          if (row < p.M && col < p.N) P[(int64_t)row * p.N + col] = acc[i][j][r];
        }
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * WN + j * 32 + col_l;
      if (col >= p.N) continue;
      const float bias = p.bias ? bf16_bits_to_f32(p.bias[col]) : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WM + i * 32 + (r >> 2) * 8 + row_l + (r & 3);
        if (row >= p.M) continue;
        float v = acc[i][j][r] + bias;
        if (p.act_tanh) v = tanhf(v);
        if (p.gate) v *= p.gate[(int64_t)row * p.ldg + col];
        const int64_t ci = (int64_t)batch * p.sC + (int64_t)row * p.ldc + col;
        if constexpr (OUT_BF16) {
          const uint32_t hi = f32_to_bf16_bits(v);
          reinterpret_cast<uint16_t*>(p.C)[ci] = (uint16_t)hi;
          if (p.C_lo) p.C_lo[ci] = (uint16_t)f32_to_bf16_bits(v - bf16_bits_to_f32(hi));
          if (p.C_dact) p.C_dact[ci] = 1.f - v * v;
        } else {
          float* C = reinterpret_cast<float*>(p.C);
          if (p.accumulate) v += C[ci];
          C[ci] = v;
        }
      }
    }
}

template <int BM, int BN, bool AKC, bool BKC, bool OUT_BF16>
static hipError_t launch_one(const GemmDev& d, int batch, hipStream_t st) {
  constexpr int smem = 2 * (BM + BN) * ROWB;
  auto kfn = gemm_bf16_kernel<BM, BN, AKC, BKC, OUT_BF16>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid(d.tiles_m * d.tiles_n, 1, batch * d.splits);
  hipLaunchKernelGGL(kfn, grid, dim3(256), smem, st, d);
  return hipGetLastError();
}

template <int BM, int BN>
static hipError_t launch_tile(const GemmArgs& g, const GemmDev& d, hipStream_t st) {
  const bool obf = g.c_bf16 && g.splits <= 1;
  if (g.a_kc && g.b_kc)
    return obf ? launch_one<BM, BN, true, true, true>(d, g.batch, st)
               : launch_one<BM, BN, true, true, false>(d, g.batch, st);
  if (g.a_kc && !g.b_kc)
    return obf ? launch_one<BM, BN, true, false, true>(d, g.batch, st)
               : launch_one<BM, BN, true, false, false>(d, g.batch, st);
  if (!g.a_kc && !g.b_kc)
    return obf ? launch_one<BM, BN, false, false, true>(d, g.batch, st)
               : launch_one<BM, BN, false, false, false>(d, g.batch, st);
  return hipErrorInvalidValue;  // (A strided, B contiguous) is not used by the path
}

hipError_t launch_gemm_bf16(const GemmArgs& g, int big_tile, hipStream_t st) {
  if (g.M < 1 || g.N < 1 || g.batch < 1 || g.splits < 1) return hipErrorInvalidValue;
  if (g.splits > 1 && (g.K[1] != 0 || g.partial == nullptr || g.C_dact)) return hipErrorInvalidValue;
  if ((g.C_lo || g.C_dact) && !g.c_bf16) return hipErrorInvalidValue;
  GemmDev d;
  for (int s = 0; s < kMaxSeg; ++s) {
    d.A[s] = reinterpret_cast<const uint16_t*>(g.A[s]);
    d.B[s] = reinterpret_cast<const uint16_t*>(g.B[s]);
    d.lda[s] = g.lda[s];
    d.ldb[s] = g.ldb[s];
    d.sA[s] = g.sA[s];
    d.sB[s] = g.sB[s];
    d.K[s] = g.K[s];
    if (g.K[s] > 0) {
      // 16-byte vector loads: leading dimensions and batch strides in units of 8 elements
      if ((g.lda[s] & 7) || (g.ldb[s] & 7) || (g.sA[s] & 7) || (g.sB[s] & 7)) return hipErrorInvalidValue;
      if ((reinterpret_cast<uintptr_t>(g.A[s]) & 15) || (reinterpret_cast<uintptr_t>(g.B[s]) & 15))
        return hipErrorInvalidValue;
    }
  }
  d.M = g.M;
  d.N = g.N;
  d.C = g.C;
  d.C_lo = reinterpret_cast<uint16_t*>(g.C_lo);
  d.C_dact = g.C_dact;
  d.ldc = g.ldc;
  d.sC = g.sC;
  d.bias = reinterpret_cast<const uint16_t*>(g.bias);
  d.gate = g.gate;
  d.ldg = g.ldg;
  d.act_tanh = g.act_tanh;
  d.accumulate = g.accumulate;
  d.splits = g.splits;
  d.partial = g.partial;
  const int bm = big_tile ? 256 : 128;
  d.tiles_m = (g.M + bm - 1) / bm;
  d.tiles_n = (g.N + bm - 1) / bm;
  const int ktiles = (g.K[0] + BK - 1) / BK;
  d.kper = ((ktiles + g.splits - 1) / g.splits) * BK;
  if (g.splits > 1 && (int64_t)d.kper * (g.splits - 1) >= g.K[0]) return hipErrorInvalidValue;
  return big_tile ? launch_tile<256, 256>(g, d, st) : launch_tile<128, 128>(g, d, st);
}

}  // namespace asx
