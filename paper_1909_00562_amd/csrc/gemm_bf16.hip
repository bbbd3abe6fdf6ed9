// bf16 x bf16 -> fp32 matrix products on the CDNA4 matrix cores (gfx950).
//
// Three kernels, one operand description (GemmDev: up to six reduction segments, three
// operand orientations: both reduction-contiguous; B stored [K,N]; A and B stored [K,*]):
//   * gemm_bf16_pp_kernel: 256x256x64 block tile, 8 waves in two staggered groups, two
//     LDS stages, persistent (one block per compute unit walks an XCD-partitioned list
//     of work items as one stream of reduction tiles).  The large products.
//   * gemm_bf16_ring_kernel: the same with 32-wide reduction sub-tiles in a ring of four
//     LDS slots (three in flight).  The weight-gradient products (both operands strided
//     in the reduction index).
//   * gemm_bf16_kernel: 128x128x64 tile, 4 waves, one block per output tile, fragment reads
//     software-pipelined inside a wave, split-K over multi-segment reductions.  Batched
//     T x S attention products and small shapes.
// Every operand goes HBM -> LDS directly (buffer_load_dwordx4 ... lds: no staging
// registers, no ds_write) in the persistent kernels; the 128x128 kernel does the same for
// reduction-contiguous operands and transposes strided ones in registers (v_perm_b32,
// ds_write_b64).  Reduction-contiguous tiles are LDS rows of 64 reduction elements
// (128 bytes) whose 16-byte chunks are XOR-swizzled by the row index
// (chunk ^ (row & 7) ^ ((row >> 3) & 1): 16 consecutive rows of one chunk column land in
// 16 different bank groups of the 64-bank LDS); the swizzle is applied on the global
// side (lane l of a wave-wide load fills LDS slot l and fetches the chunk that belongs
// there).  Strided tiles stay [k][256 columns] as in memory and are read with the
// transposing ds_read_b64_tr_b16.  Out-of-range rows / reduction indices are redirected
// to an offset beyond the buffer resource's range, which reads as zero: no branches.
// Wave tile 128x64 (persistent kernels) or 64x64.  MFMA 32x32x16 bf16, except that the persistent two-stage
// kernel runs 16x16x32 when both operands are reduction-contiguous (the clock this part grants is higher on it).
// The epilogue stages each wave's accumulators through its own slice of LDS so that
// global stores are 8/16-byte vectors along rows.
#include "common.h"
#include "gemm.h"

#include <type_traits>

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
  uint32_t drop_thr;
  float drop_scale;
  uint64_t drop_seed;
  int splits;
  float* partial;
  int tiles_m, tiles_n;
  int group;   // tile rows per group of the persistent kernel's tile walk
  int kper;    // reduction elements per split, multiple of 64
  int vec_ok;  // rows of C (and C_lo, C_dact, gate) allow 8/16-byte vector access
  const int32_t* M_dev;   // device-side row count (or null): min(*M_dev, M) rows are valid
  const int32_t* K_dev;   // device-side reduction length of segment 0 (or null)
  int nz;                 // batch * splits
  int dyn_split;          // splits is the bound of a split chosen in the kernel from the row count (pp kernel)
};

// size made by an earlier kernel of the stream, clamped to the bound the launch was sized for
__device__ __forceinline__ int dev_bound(const int32_t* count, int bound) {
  if (!count) return bound;
  const int v = *count;
  return v < 0 ? 0 : (v < bound ? v : bound);
}

constexpr int BK = 64;                  // reduction elements per LDS tile row
constexpr int ROWB = BK * 2;            // bytes per LDS tile row
constexpr uint32_t kOob = 0x80000000u;  // offset outside every buffer resource below

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void_t;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base) {
  // raw buffer, 2 GiB range: offsets >= 2^31 (kOob) read as zero
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}

// ---- reduction-contiguous operand: HBM -> LDS, no registers ----------------------
// The tile's ROWS rows are split into groups of 8 rows (1 KiB of LDS); one wave-wide
// 16-byte load fills one group.  Per-lane byte offsets relative to element
// (row0, k0) are computed once per kernel; rows beyond the operand get kOob.
template <int ROWS, int NW>
struct DirectLoader {
  static constexpr int NL = ROWS / 8 / NW;   // loads per wave and tile
  uint32_t voff[NL];
  int chunk8;                                // first reduction element of this lane's chunk
  __device__ __forceinline__ void init(int64_t ld, int rows_left, int wave, int lane) {
    static_assert(NW % 2 == 0, "swizzle below assumes the parity of the row group is the wave's");
    const int rl = lane >> 3;                        // row inside the group
    const int chunk = (lane & 7) ^ rl ^ (wave & 1);  // logical 16-byte chunk that belongs in LDS slot `lane`
    chunk8 = chunk * 8;
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int r = (wave + NW * j) * 8 + rl;
      voff[j] = r < rows_left ? (uint32_t)(((int64_t)r * ld + chunk * 8) * 2) : kOob;
    }
  }
  // X points at element (row0, k0); k_left = reduction elements left from k0
  __device__ __forceinline__ void load(int j, const __amdgpu_buffer_rsrc_t& rs, int k_left, unsigned char* lds_tile,
                                       int wave) const {
    const uint32_t off = chunk8 < k_left ? voff[j] : kOob;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_t*)(lds_tile + (wave + NW * j) * 1024), 16, off, 0, 0, 0);
  }
};

// ---- strided-reduction operand: HBM -> registers -> transposed into LDS --------------
// Thread t owns rows (t/16)*8 .. +7 (contiguous index) x reduction rows (t%16)*4 .. +3.
template <int ROWS, int NT>
struct TransposeLoader {
  static constexpr int NB = ROWS * 2 / NT;   // 4x8 blocks per thread
  static constexpr int NL = NB * 4;          // 16-byte loads per thread and tile
  uint32_t voff[NL];
  u32x4_t r[NL];
  int k4;
  __device__ __forceinline__ void init(int64_t ld, int rows_left, int tid) {
    const int kq = tid & 15, rb = tid >> 4;
    k4 = kq * 4;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int row = (rb + (NT / 16) * j) * 8;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        voff[j * 4 + kk] = row < rows_left ? (uint32_t)(((int64_t)(k4 + kk) * ld + row) * 2) : kOob;
    }
  }
  // X points at element (k0, row0) of the operand stored [K, rows]
  __device__ __forceinline__ void load(int l, const __amdgpu_buffer_rsrc_t& rs, int k_left) {
    const uint32_t off = (k4 + (l & 3)) < k_left ? voff[l] : kOob;
    r[l] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
  }
  __device__ __forceinline__ void store(unsigned char* lds_tile, int tid) const {
    static_assert((NT / 16) % 2 == 0, "row-group parity must not depend on j");
    const int kq = tid & 15, rb = tid >> 4;
    const int chunk = (kq >> 1) ^ (rb & 1), half = kq & 1;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = (rb + (NT / 16) * j) * 8 + e;
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        const uint32_t lo = __builtin_amdgcn_perm(r[j * 4 + 1][e >> 1], r[j * 4 + 0][e >> 1], sel);
        const uint32_t hi = __builtin_amdgcn_perm(r[j * 4 + 3][e >> 1], r[j * 4 + 2][e >> 1], sel);
        *reinterpret_cast<uint2*>(lds_tile + row * ROWB + ((chunk ^ e) << 4) + half * 8) = make_uint2(lo, hi);
      }
    }
  }
};

__device__ __forceinline__ bf16x8_t frag_read(const unsigned char* base, int row, int chunk) {
  return *reinterpret_cast<const bf16x8_t*>(base + row * ROWB + ((chunk ^ (row & 7) ^ ((row >> 3) & 1)) << 4));
}

// ---- epilogue --------------------------------------------------------------------
// MFMA 32x32 output: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4,
// column l%32 of its tile.  Each wave stages 32 rows x 64 columns at a time through
// its own slice of LDS (rows padded to 72 floats so that the two half-waves of a
// store hit different banks) and reads them back as 4-column vectors (16 lanes per
// row), so the global accesses are row-contiguous.  row0 / col0: first row / column
// of this wave's tile in C.
// `region` is this wave's private LDS slice: CH rows of EP_LD floats (CH = 32 or 16).
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// Accumulators of one round (CH rows of the wave tile) -> the wave's staging slice.
// MI16 = false: 32x32 MFMA tiles (register r of lane l: row 8*(r/4) + 4*(l/32) + r%4, column l%32).
// MI16 = true: 16x16 tiles (register r of lane l: row 4*(l/16) + r, column l%16), one tile row per round; the four
// lane groups of a store would hit the same 16 banks, so the 16-column block j of row group g is kept at block j ^ g.
template <bool MI16, int TN, int CH, int EP_LD, typename AccT>
__device__ __forceinline__ void stage_round(float* stage_f, AccT& acc, int ic, int lane) {
  if constexpr (MI16) {
    static_assert(CH == 16 && EP_LD == 64 && TN == 4, "one 16-row tile row per round, 64-column wave tile");
    const int g = lane >> 4, c = lane & 15;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) stage_f[(4 * g + r) * 64 + (((j ^ g) & 3) << 4) + c] = acc[ic][j][r];
  } else {
    const int i = ic / (32 / CH), part = ic % (32 / CH);
    const int col_l = lane & 31, row_l = (lane >> 5) * 4;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int trow = (r >> 2) * 8;
        if (trow / CH != part) continue;
        stage_f[(trow % CH + row_l + (r & 3)) * EP_LD + j * 32 + col_l] = acc[i][j][r];
      }
  }
}
// float offset of the 4-column vector (row group it, lane's vrow / vcol) inside the staging slice
template <bool MI16, int EP_LD>
__device__ __forceinline__ int stage_read_off(int it, int vrow, int vcol) {
  return (it * 4 + vrow) * EP_LD + (MI16 ? (vcol ^ (it << 4)) : vcol);
}

// Vector form of the epilogue below for products whose destinations allow 8/16-byte
// row vectors and whose N is a multiple of 4 (chosen on the host, per launch): stores (and the gate / accumulate
// loads) go through buffer resources that start at the wave tile's first element, so
// the row part of an address is a scalar offset, the lane part one register, and rows
// beyond M are dropped by pointing the lane offset outside the resource instead of branching.
template <int TM, int TN, bool OUT_BF16, bool DROP, int CH, int EP_LD, bool MI16, typename AccT>
__device__ __forceinline__ void gemm_epilogue_vec(const GemmDev& p, int Mv, AccT& acc,
                                                  unsigned char* region, int lane, int row0, int col0, int batch,
                                                  int z) {
  constexpr int WAIT_LGKM_ONLY = 0xC07F;
  constexpr int ES = OUT_BF16 ? 2 : 4;
  float* stage_f = reinterpret_cast<float*>(region);
  const int col_l = lane & 31, row_l = (lane >> 5) * 4;
  const int vcol = (lane & 15) * 4, vrow = lane >> 4;
  const bool to_partial = p.splits > 1;
  const int64_t ld = to_partial ? (int64_t)p.N : p.ldc;
  const int64_t origin = to_partial ? ((int64_t)z * p.M + row0) * p.N + col0
                                    : (int64_t)batch * p.sC + (int64_t)row0 * p.ldc + col0;
  unsigned char* cbase = to_partial ? reinterpret_cast<unsigned char*>(p.partial) : reinterpret_cast<unsigned char*>(p.C);
  const __amdgpu_buffer_rsrc_t rs_c = make_rsrc(cbase + origin * ES);
  const __amdgpu_buffer_rsrc_t rs_lo = make_rsrc(p.C_lo ? p.C_lo + origin : nullptr);
  const __amdgpu_buffer_rsrc_t rs_da = make_rsrc(p.C_dact ? p.C_dact + origin : nullptr);
  const float* gate0 = p.gate ? p.gate + (int64_t)row0 * p.ldg + col0 : nullptr;   // gate and old-C reads: plain loads
  const int rows_left = Mv - row0 - vrow;                        // valid rows of C from this lane's first row on
  const bool col_in = col0 + vcol < p.N;                         // N % 4 == 0: a 4-column group is all in or all out
  const uint32_t lane_off = (uint32_t)(vrow * ld + vcol);        // elements, inside the wave tile's window
  const uint32_t lane_off_g = (uint32_t)(vrow * p.ldg + vcol);
  const uint32_t ld32 = (uint32_t)ld, ldg32 = (uint32_t)p.ldg;
  const bool fuse = !to_partial;
  float bias4[4] = {0.f, 0.f, 0.f, 0.f};
  if (p.bias && fuse) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (col_in) bias4[c] = bf16_bits_to_f32(p.bias[col0 + vcol + c]);
  }
  const bool plain = !DROP && !p.act_tanh && !p.gate && !p.C_lo && !p.C_dact && !(fuse && p.accumulate);
  if (plain) {
    // Bias only (no tanh, gate, remainder / derivative outputs, accumulation, dropout), decided once per tile:
    // the general form below tests each of those per row group, and its branches and the arithmetic behind
    // them were most of the write-out time of the vocabulary projection (two waves share a SIMD's vector ALU).
    // The CH/4 reads of a round are in flight together, and the LDS writes of round ic+1 are issued when
    // the last read of round ic has returned, so their latency hides behind that row group's stores.
    constexpr int NR = MI16 ? TM : TM * (32 / CH);
    auto write_round = [&](int ic) { stage_round<MI16, TN, CH, EP_LD>(stage_f, acc, ic, lane); };
    write_round(0);
#pragma unroll
    for (int ic = 0; ic < NR; ++ic) {
      __builtin_amdgcn_s_waitcnt(WAIT_LGKM_ONLY);
      f32x4_t v4s[CH / 4];
#pragma unroll
      for (int it = 0; it < CH / 4; ++it)
        v4s[it] = *reinterpret_cast<const f32x4_t*>(stage_f + stage_read_off<MI16, EP_LD>(it, vrow, vcol));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int it = 0; it < CH / 4; ++it) {
        const int nrow = ic * CH + it * 4;                       // tile row of the lane's row group (compile time)
        const bool in = nrow < rows_left && col_in;
        if (it == CH / 4 - 1) {
          __builtin_amdgcn_s_waitcnt(WAIT_LGKM_ONLY);
          if (ic + 1 < NR) write_round(ic + 1);
          __builtin_amdgcn_sched_barrier(0);
        }
        const f32x4_t v4 = v4s[it];
        const uint32_t row_el = (uint32_t)nrow * ld32;           // wave-uniform: goes into the scalar offset operand
        const float v[4] = {v4[0] + bias4[0], v4[1] + bias4[1], v4[2] + bias4[2], v4[3] + bias4[3]};
        if constexpr (OUT_BF16) {
          const u32x2_t hv = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
          __builtin_amdgcn_raw_buffer_store_b64(hv, rs_c, in ? lane_off * 2u : kOob, row_el * 2u, 0);
        } else {
          const u32x4_t sv = {__builtin_bit_cast(uint32_t, v[0]), __builtin_bit_cast(uint32_t, v[1]),
                              __builtin_bit_cast(uint32_t, v[2]), __builtin_bit_cast(uint32_t, v[3])};
          __builtin_amdgcn_raw_buffer_store_b128(sv, rs_c, in ? lane_off * 4u : kOob, row_el * 4u, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    return;
  }
#pragma unroll
  for (int ic = 0; ic < (MI16 ? TM : TM * (32 / CH)); ++ic) {
    stage_round<MI16, TN, CH, EP_LD>(stage_f, acc, ic, lane);
    __builtin_amdgcn_s_waitcnt(WAIT_LGKM_ONLY);
#pragma unroll
    for (int it = 0; it < CH / 4; ++it) {
      const int nrow = ic * CH + it * 4;                         // tile row of the lane's row group (compile time)
      const bool in = nrow < rows_left && col_in;
      const f32x4_t v4 = *reinterpret_cast<const f32x4_t*>(stage_f + stage_read_off<MI16, EP_LD>(it, vrow, vcol));
      const uint32_t row_el = (uint32_t)nrow * ld32;             // wave-uniform: goes into the scalar offset operand
      float v[4] = {v4[0] + bias4[0], v4[1] + bias4[1], v4[2] + bias4[2], v4[3] + bias4[3]};
      if (fuse && p.act_tanh) {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = tanhf(v[c]);
      }
      float dact[4] = {1.f - v[0] * v[0], 1.f - v[1] * v[1], 1.f - v[2] * v[2], 1.f - v[3] * v[3]};
      if constexpr (DROP) {       // the lane's four columns are one block of the generator (N % 4 == 0)
        uint32_t w[4];
        dropout_words4(((uint64_t)(row0 + vrow + nrow) * p.N + (uint32_t)(col0 + vcol)) >> 2, p.drop_seed, w);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float sc = w[c] >= p.drop_thr ? p.drop_scale : 0.f;
          v[c] *= sc;
          dact[c] *= sc;
        }
      }
      if (fuse && p.gate && in) {
        const f32x4_t g4 = *reinterpret_cast<const f32x4_t*>(gate0 + (uint32_t)nrow * ldg32 + lane_off_g);
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] *= g4[c];
      }
      if constexpr (OUT_BF16) {
        const uint32_t off = in ? lane_off * 2u : kOob;
        uint32_t hb[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) hb[c] = f32_to_bf16_bits(v[c]);
        const u32x2_t hv = {hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16)};
        __builtin_amdgcn_raw_buffer_store_b64(hv, rs_c, off, row_el * 2u, 0);
        if (p.C_lo) {
          const u32x2_t lv = {pack_bf16(v[0] - bf16_bits_to_f32(hb[0]), v[1] - bf16_bits_to_f32(hb[1])),
                              pack_bf16(v[2] - bf16_bits_to_f32(hb[2]), v[3] - bf16_bits_to_f32(hb[3]))};
          __builtin_amdgcn_raw_buffer_store_b64(lv, rs_lo, off, row_el * 2u, 0);
        }
        if (p.C_dact) {
          const u32x4_t dv = {__builtin_bit_cast(uint32_t, dact[0]), __builtin_bit_cast(uint32_t, dact[1]),
                              __builtin_bit_cast(uint32_t, dact[2]), __builtin_bit_cast(uint32_t, dact[3])};
          __builtin_amdgcn_raw_buffer_store_b128(dv, rs_da, in ? lane_off * 4u : kOob, row_el * 4u, 0);
        }
      } else {
        const uint32_t off = in ? lane_off * 4u : kOob;
        if (fuse && p.accumulate && in) {
          const f32x4_t o4 =
              *reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(cbase) + origin + row_el + lane_off);
#pragma unroll
          for (int c = 0; c < 4; ++c) v[c] += o4[c];
        }
        const u32x4_t sv = {__builtin_bit_cast(uint32_t, v[0]), __builtin_bit_cast(uint32_t, v[1]),
                            __builtin_bit_cast(uint32_t, v[2]), __builtin_bit_cast(uint32_t, v[3])};
        __builtin_amdgcn_raw_buffer_store_b128(sv, rs_c, off, row_el * 4u, 0);
      }
      __builtin_amdgcn_sched_barrier(0);           // keeps the live ranges of one row group apart from the next
    }
    __builtin_amdgcn_s_waitcnt(WAIT_LGKM_ONLY);  // LDS reads done before the next rows overwrite the slice
  }
}

template <int TM, int TN, bool OUT_BF16, bool VEC, bool DROP, int CH = 32, int EP_LD = 72, bool MI16 = false,
          typename AccT>
__device__ __forceinline__ void gemm_epilogue(const GemmDev& p, int Mv, AccT& acc,
                                              unsigned char* region, int lane, int row0, int col0, int batch, int z) {
  static_assert(TN == (MI16 ? 4 : 2), "64-column wave tiles");
  static_assert(CH == 32 || CH == 16, "chunk of one or half an MFMA tile");
  if constexpr (VEC) {
    gemm_epilogue_vec<TM, TN, OUT_BF16, DROP, CH, EP_LD, MI16>(p, Mv, acc, region, lane, row0, col0, batch, z);
    return;
  }
  constexpr int WAIT_LGKM_ONLY = 0xC07F;   // leaves global loads in flight
  float* stage_f = reinterpret_cast<float*>(region);
  const int col_l = lane & 31, row_l = (lane >> 5) * 4;
  const int vcol = (lane & 15) * 4, vrow = lane >> 4;
  const int gcol = col0 + vcol;
  float* Pz = p.splits > 1 ? p.partial + (int64_t)z * p.M * p.N : nullptr;
  float bias4[4] = {0.f, 0.f, 0.f, 0.f};
  if (p.bias && p.splits <= 1) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (gcol + c < p.N) bias4[c] = bf16_bits_to_f32(p.bias[gcol + c]);
  }
#pragma unroll
  for (int ic = 0; ic < (MI16 ? TM : TM * (32 / CH)); ++ic) {
    stage_round<MI16, TN, CH, EP_LD>(stage_f, acc, ic, lane);
    __builtin_amdgcn_s_waitcnt(WAIT_LGKM_ONLY);
#pragma unroll 4
    for (int it = 0; it < CH / 4; ++it) {
      const int lr = it * 4 + vrow;
      const int grow = row0 + ic * CH + lr;
      if (grow >= Mv || gcol >= p.N) continue;
      const f32x4_t v4 = *reinterpret_cast<const f32x4_t*>(stage_f + stage_read_off<MI16, EP_LD>(it, vrow, vcol));
      float v[4] = {v4[0], v4[1], v4[2], v4[3]};
      if (Pz) {
        float* dst = Pz + (int64_t)grow * p.N + gcol;
        if (gcol + 3 < p.N && (p.N & 3) == 0) {
          *reinterpret_cast<f32x4_t*>(dst) = v4;
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (gcol + c < p.N) dst[c] = v[c];
        }
        continue;
      }
      const bool vec = p.vec_ok && gcol + 3 < p.N;
      const int64_t ci = (int64_t)batch * p.sC + (int64_t)grow * p.ldc + gcol;
      float gt[4] = {1.f, 1.f, 1.f, 1.f};
      if (p.gate) {
        const float* gp = p.gate + (int64_t)grow * p.ldg + gcol;
        if (vec) {
          const f32x4_t g4 = *reinterpret_cast<const f32x4_t*>(gp);
          gt[0] = g4[0]; gt[1] = g4[1]; gt[2] = g4[2]; gt[3] = g4[3];
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (gcol + c < p.N) gt[c] = gp[c];
        }
      }
      float dact[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float x = v[c] + bias4[c];
        if (p.act_tanh) x = tanhf(x);
        dact[c] = 1.f - x * x;
        if (DROP && gcol + c < p.N) {
          const float sc = dropout_mult((uint64_t)grow * p.N + (gcol + c), p.drop_seed, p.drop_thr, p.drop_scale);
          x *= sc;
          dact[c] *= sc;
        }
        v[c] = x * gt[c];
      }
      if constexpr (OUT_BF16) {
        uint16_t* C = reinterpret_cast<uint16_t*>(p.C) + ci;
        uint32_t hb[4];
        float lo[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          hb[c] = f32_to_bf16_bits(v[c]);
          lo[c] = v[c] - bf16_bits_to_f32(hb[c]);
        }
        if (vec) {
          *reinterpret_cast<uint2*>(C) = make_uint2(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16));
          if (p.C_lo)
            *reinterpret_cast<uint2*>(p.C_lo + ci) = make_uint2(pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]));
          if (p.C_dact) {
            f32x4_t d4 = {dact[0], dact[1], dact[2], dact[3]};
            *reinterpret_cast<f32x4_t*>(p.C_dact + ci) = d4;
          }
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (gcol + c < p.N) {
              C[c] = (uint16_t)hb[c];
              if (p.C_lo) p.C_lo[ci + c] = (uint16_t)f32_to_bf16_bits(lo[c]);
              if (p.C_dact) p.C_dact[ci + c] = dact[c];
            }
        }
      } else {
        float* C = reinterpret_cast<float*>(p.C) + ci;
        if (vec) {
          if (p.accumulate) {
            const f32x4_t o4 = *reinterpret_cast<const f32x4_t*>(C);
            v[0] += o4[0]; v[1] += o4[1]; v[2] += o4[2]; v[3] += o4[3];
          }
          f32x4_t s4 = {v[0], v[1], v[2], v[3]};
          *reinterpret_cast<f32x4_t*>(C) = s4;
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (gcol + c < p.N) C[c] = p.accumulate ? v[c] + C[c] : v[c];
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(WAIT_LGKM_ONLY);  // LDS reads done before the next rows overwrite the slice
  }
}

template <int BM, int BN, int WGM, int WGN, bool AKC, bool BKC, bool OUT_BF16, bool VEC, bool DROP>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_kernel(GemmDev p) {
  constexpr int NW = WGM * WGN, NT = 64 * NW;
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  constexpr int STAGE = (BM + BN) * ROWB;
  static_assert(WN == 64 && (WM == 64 || WM == 128), "epilogue assumes 64-column wave tiles");
  static_assert(2 * STAGE >= NW * 16384, "epilogue needs 16 KiB of LDS per wave");
  extern __shared__ __align__(1024) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS bases of direct loads
  const int wm = wave / WGN, wn = wave % WGN;

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
  const int Mv = dev_bound(p.M_dev, p.M);   // valid rows: the grid was sized for p.M
  const int K0 = dev_bound(p.K_dev, p.K[0]);
  if (m0 >= Mv) return;                     // the whole block, before any barrier

  const int z = blockIdx.z;
  const int batch = z / p.splits, split = z - batch * p.splits;

  // reduction tiles of this block: all of them, or (split-K) tiles [t0, t1) of the sequence that runs
  // through the segments one after the other; the cursor below starts at tile t0
  int nks[kMaxSeg];
  int nk = 0;
#pragma unroll
  for (int s = 0; s < kMaxSeg; ++s) {
    nks[s] = ((s == 0 ? K0 : p.K[s]) + BK - 1) / BK;
    nk += nks[s];
  }
  int seg0 = 0, skip0 = 0;   // first segment of this block and reduction tiles skipped inside it
  if (p.splits > 1) {
    // a reduction length read on the device is split here (a split may then come out empty: it stores zeros)
    const int tper = p.K_dev ? (nk + p.splits - 1) / p.splits : p.kper / BK;
    const int t0 = split * tper;
    const int t1 = t0 + tper < nk ? t0 + tper : nk;
    nk = t1 > t0 ? t1 - t0 : 0;
    skip0 = t0;
    while (seg0 < kMaxSeg - 1 && skip0 >= nks[seg0]) {
      skip0 -= nks[seg0];
      ++seg0;
    }
  }
  const int kbeg0 = skip0 * BK;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // per-lane load offsets, fixed for the whole kernel (all segments share lda / ldb)
  DirectLoader<BM, NW> dla;
  DirectLoader<BN, NW> dlb;
  TransposeLoader<BM, NT> tla;
  TransposeLoader<BN, NT> tlb;
  if constexpr (AKC) dla.init(p.lda[0], Mv - m0, wave, lane); else tla.init(p.lda[0], Mv - m0, tid);
  if constexpr (BKC) dlb.init(p.ldb[0], p.N - n0, wave, lane); else tlb.init(p.ldb[0], p.N - n0, tid);
  constexpr int NLA = AKC ? DirectLoader<BM, NW>::NL : TransposeLoader<BM, NT>::NL;
  constexpr int NLB = BKC ? DirectLoader<BN, NW>::NL : TransposeLoader<BN, NT>::NL;
  constexpr int NLT = NLA + NLB;

  // cursor over the reduction tiles of all segments: operand pointers of the next tile to load
  const int64_t stepA = AKC ? BK : (int64_t)BK * p.lda[0], stepB = BKC ? BK : (int64_t)BK * p.ldb[0];
  const int64_t offA = AKC ? (int64_t)m0 * p.lda[0] : m0, offB = BKC ? (int64_t)n0 * p.ldb[0] : n0;
  int cseg = seg0, ck_left = (seg0 == 0 ? K0 : p.K[seg0]) - kbeg0;
  const uint16_t* cA = p.A[seg0] + (int64_t)batch * p.sA[seg0] + offA + (AKC ? kbeg0 : (int64_t)kbeg0 * p.lda[0]);
  const uint16_t* cB = p.B[seg0] + (int64_t)batch * p.sB[seg0] + offB + (BKC ? kbeg0 : (int64_t)kbeg0 * p.ldb[0]);
  auto advance = [&]() {
    cA += stepA;
    cB += stepB;
    ck_left -= BK;
    if (ck_left <= 0) {
      do { ++cseg; } while (cseg < kMaxSeg && p.K[cseg] <= 0);
      if (cseg < kMaxSeg) {
        cA = p.A[cseg] + (int64_t)batch * p.sA[cseg] + offA;
        cB = p.B[cseg] + (int64_t)batch * p.sB[cseg] + offB;
        ck_left = p.K[cseg];
      }
    }
  };
  // loads [l0, l1) of the tile under the cursor into LDS stage `stage` (or registers)
  auto issue = [&](int stage, int l0, int l1) {
    const __amdgpu_buffer_rsrc_t rsa = make_rsrc(cA), rsb = make_rsrc(cB);
    unsigned char* as = smem + stage * STAGE;
    unsigned char* bs = as + BM * ROWB;
#pragma unroll
    for (int l = 0; l < NLT; ++l) {
      if (l < l0 || l >= l1) continue;
      if (l < NLA) {
        if constexpr (AKC) dla.load(l, rsa, ck_left, as, wave); else tla.load(l, rsa, ck_left);
      } else {
        if constexpr (BKC) dlb.load(l - NLA, rsb, ck_left, bs, wave); else tlb.load(l - NLA, rsb, ck_left);
      }
    }
  };
  // transposed operands: registers -> LDS
  auto commit = [&](int stage) {
    unsigned char* as = smem + stage * STAGE;
    unsigned char* bs = as + BM * ROWB;
    if constexpr (!AKC) tla.store(as, tid);
    if constexpr (!BKC) tlb.store(bs, tid);
  };
  auto read_frags = [&](bf16x8_t (&af)[TM], bf16x8_t (&bfr)[TN], int stage, int kk) {
    const unsigned char* as = smem + stage * STAGE;
    const unsigned char* bs = as + BM * ROWB;
    const int chunk = kk * 2 + (lane >> 5);
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = frag_read(as, wm * WM + i * 32 + (lane & 31), chunk);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = frag_read(bs, wn * WN + j * 32 + (lane & 31), chunk);
  };

  if (nk > 0) {
    issue(0, 0, NLT);
    advance();
    commit(0);
  }
  __builtin_amdgcn_s_waitcnt(0);  // this wave's direct loads have landed in LDS
  __syncthreads();

  // Software pipeline: the fragments of step kk+1 are read from LDS while the MFMAs
  // of step kk run, also across the tile boundary; the next tile's global loads
  // are spread over the first three steps.
  bf16x8_t af[2][TM], bfr[2][TN];
  if (nk > 0) read_frags(af[0], bfr[0], 0, 0);
  constexpr int KSTEPS = BK / 16;
  constexpr int LPART = (NLT + KSTEPS - 2) / (KSTEPS - 1);
  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    const int cur = kt & 1, nxt = cur ^ 1;
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      if (kk < KSTEPS - 1) {
        if (more) issue(nxt, kk * LPART, (kk + 1) * LPART < NLT ? (kk + 1) * LPART : NLT);
        read_frags(af[(kk + 1) & 1], bfr[(kk + 1) & 1], cur, kk + 1);
      } else {
        if (more) {
          commit(nxt);
          advance();
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (more) read_frags(af[(kk + 1) & 1], bfr[(kk + 1) & 1], nxt, 0);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
    }
  }
  // (the last barrier above came after every wave's final fragment reads: LDS is free for the epilogue)

  gemm_epilogue<TM, TN, OUT_BF16, VEC, DROP>(p, Mv, acc, smem + wave * 16384, lane, m0 + wm * WM, n0 + wn * WN, batch,
                                             z);
}


// ---- 256x256 tile, 8 waves, two staggered wave groups ("ping-pong") ---------------
// Reduction tiles of 64 elements, two LDS stages, every operand loaded HBM -> LDS
// directly whatever its orientation:
//   * reduction-contiguous operand: LDS tile [256 rows][64 k] (128-byte rows, chunks
//     swizzled as above), fragments read with ds_read_b128;
//   * strided-reduction operand: LDS tile [64 k][256 columns] exactly as in memory
//     (512-byte rows, 64-byte segments XOR-swizzled with k & 3), fragments read with
//     the transposing ds_read_b64_tr_b16: a 16-lane group presents four k-rows x 16
//     columns and each lane receives four consecutive k of its own column.
// Waves 0-3 (group A) and 4-7 (group B) sit pairwise on the four SIMDs.  Per tile a
// wave alternates memory and compute phases,
//     M0: read the fragments of steps 0,1      C0: 16 MFMAs from registers
//     M1: read the fragments of steps 2,3      C1: 16 MFMAs
// and there is ONE workgroup barrier per tile, which group A takes after its C1 and
// group B after its M1: B therefore runs one phase behind A, so on every SIMD one
// wave issues MFMAs while its partner waits on LDS, issues loads or sits at the
// barrier, and the matrix pipe stays fed.
// Hazards: tile t lives in stage t&1 and is read only between barrier t and barrier
// t+1 (A: M0,M1 of its iteration t; B: likewise, its C1(t) needs registers only).
// The loads of tile t+1 are issued after barrier t (in M0 of iteration t) into the
// stage tile t-1 has left, and every wave waits for its own loads before barrier t+1.
constexpr int PTILE = 256 * BK * 2;   // bytes of one operand tile
constexpr int PSTAGE = 2 * PTILE;

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

// wave-wide direct loads of one operand tile: 32 loads of 1 KiB per tile, NL = 32 / NW per wave
template <bool KC, int NW = 8>
struct PpLoader {
  static constexpr int NL = 32 / NW;
  static_assert(NW % 2 == 0, "the swizzle terms below take the parity of a row group from the wave index");
  uint32_t voff[NL];
  int kpos;   // KC: first reduction element of the lane's chunk; strided: its k-row for load 0
  __device__ __forceinline__ void init(int64_t ld, int rows_left, int wave, int lane) {
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int g = wave + NW * j;
      if constexpr (KC) {
        // group g = rows 8g .. 8g+7; LDS slot `lane` = row lane/8, physical chunk lane%8
        const int row = g * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ (lane >> 3) ^ (wave & 1);   // (row & 7) ^ ((row >> 3) & 1)
        if (j == 0) kpos = chunk * 8;
        voff[j] = row < rows_left ? (uint32_t)(((int64_t)row * ld + chunk * 8) * 2) : kOob;
      } else {
        // group g = k-rows 2g, 2g+1; LDS slot `lane` = k-row lane/32, physical 16-byte chunk lane%32
        const int k = 2 * g + (lane >> 5);
        const int pc = lane & 31;
        const int seg = (pc >> 2) ^ (((wave & 1) << 1) + (lane >> 5));   // physical ^ (k & 3)
        const int col = (seg * 4 + (pc & 3)) * 8;
        if (j == 0) kpos = k;                                      // load j covers k-row kpos + 2 NW j
        voff[j] = col < rows_left ? (uint32_t)(((int64_t)k * ld + col) * 2) : kOob;
      }
    }
  }
  __device__ __forceinline__ void load_one(int j, const __amdgpu_buffer_rsrc_t& rs, int k_left,
                                           unsigned char* lds_tile, int wave) const {
    const bool ok = KC ? kpos < k_left : kpos + 2 * NW * j < k_left;
    const uint32_t off = ok ? voff[j] : kOob;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_t*)(lds_tile + (wave + NW * j) * 1024), 16, off, 0, 0, 0);
  }
  __device__ __forceinline__ void load(const __amdgpu_buffer_rsrc_t& rs, int k_left, unsigned char* lds_tile,
                                       int wave) const {
#pragma unroll
    for (int j = 0; j < NL; ++j) load_one(j, rs, k_left, lds_tile, wave);
  }
};

// MFMA fragments (8 consecutive k of one row / column per lane).  The lane's byte
// offset inside an operand tile is computed once per kernel (pp_frag_base); the
// fragment of reduction step kk is then one XOR away (reduction-contiguous tiles: the
// swizzled chunk index is chunk0 ^ (kk << 1)) or a constant offset away (strided
// tiles: step kk starts 16 k-rows = 8 KiB further, and k & 3 does not depend on kk).
template <bool KC>
__device__ __forceinline__ uint32_t pp_frag_base(int row0, int lane) {
  if constexpr (KC) {
    const int row = row0 + (lane & 31);
    const int chunk0 = (lane >> 5) ^ (row & 7) ^ ((row >> 3) & 1);
    return (uint32_t)(row * ROWB + (chunk0 << 4));
  } else {
    const int col = row0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;   // four columns this lane presents
    const int kq = (lane & 15) >> 2;                                   // k & 3 of every row it reads
    const int k0 = (lane >> 5) * 8 + kq;
    const int cb = col * 2;
    return (uint32_t)(k0 * 512 + (((cb >> 6) ^ kq) << 6) + (cb & 63));
  }
}
template <bool KC>
__device__ __forceinline__ bf16x8_t pp_frag_at(const unsigned char* tile, uint32_t base, int kk) {
  if constexpr (KC) {
    return *reinterpret_cast<const bf16x8_t*>(tile + (base ^ (uint32_t)(kk << 5)));
  } else {
    union { s16x4_t h[2]; bf16x8_t v; } u;
#pragma unroll
    for (int q = 0; q < 2; ++q)
      u.h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_t*)(lds_void_t*)(tile + base + kk * 8192 + q * 2048));
    return u.v;
  }
}

// The same for the 16x16x32 MFMA: a fragment is 16 rows x 32 reduction elements, lane l holds row l % 16 and the 8
// elements 8 * (l / 16) .. + 7.  Reduction-contiguous tiles: logical chunk 4 * ks + l / 16 of the row for reduction
// step ks (0 or 1) of a 64-wide tile, i.e. bit 6 of the byte offset flips with ks.  Strided tiles: the 16-lane group
// g = l / 16 of a transposing read presents k-rows 8g .. 8g+3 (second read: + 4) x the fragment's 16 columns.
template <bool KC>
__device__ __forceinline__ uint32_t pp16_frag_base(int row0, int lane) {
  if constexpr (KC) {
    const int row = row0 + (lane & 15);
    const int chunk0 = (lane >> 4) ^ (row & 7) ^ ((row >> 3) & 1);
    return (uint32_t)(row * ROWB + (chunk0 << 4));
  } else {
    const int col = row0 + (lane & 3) * 4;                             // four columns this lane presents
    const int kq = (lane & 15) >> 2;                                   // k & 3 of every row it reads
    const int k0 = (lane >> 4) * 8 + kq;
    const int cb = col * 2;
    return (uint32_t)(k0 * 512 + (((cb >> 6) ^ kq) << 6) + (cb & 63));
  }
}
template <bool KC>
__device__ __forceinline__ bf16x8_t pp16_frag_at(const unsigned char* tile, uint32_t base, int ks) {
  if constexpr (KC) {
    return *reinterpret_cast<const bf16x8_t*>(tile + (base ^ (uint32_t)(ks << 6)));
  } else {
    union { s16x4_t h[2]; bf16x8_t v; } u;
#pragma unroll
    for (int q = 0; q < 2; ++q)
      u.h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_t*)(lds_void_t*)(tile + base + ks * 16384 + q * 2048));
    return u.v;
  }
}

// The kernel is persistent: the grid is one block per CU, and each block walks its
// list of (output tile, reduction split, batch) work items as ONE stream of
// reduction tiles, so the loads of the next item's first tiles are in flight while
// the current item finishes and is written out (its epilogue stages through a
// separate 32 KiB of LDS): no pipeline fill / drain and no launch gap per output tile.
constexpr int PP_EPI_OFF = 2 * PSTAGE;        // epilogue staging behind the two tile stages
constexpr int PP_SMEM = PP_EPI_OFF + 8 * 4096;

// MI16: the wave tile as 8 x 4 tiles of the 16x16x32 MFMA instead of 4 x 2 tiles of the 32x32x16 one.  Same LDS
// layout, same number of fragment reads, twice as many (half as long) MFMAs.  On this part the 16x16x32 form
// sustains an 11 % higher rate in a register-only loop on random operands (the clock is held by a power budget and
// the smaller tile moves fewer accumulator bytes per flop); in the kernel it gains 4 % with both operands
// reduction-contiguous and loses 2 % when one operand needs the transposing reads, so the launcher picks it for the
// former only.
template <bool AKC, bool BKC, bool OUT_BF16, bool VEC, bool DROP, bool MI16>
__global__ __launch_bounds__(512) void gemm_bf16_pp_kernel(GemmDev p, int work_total) {
  constexpr int BM = 256, BN = 256, WGN = 4;
  constexpr int WM = 128, WN = 64;
  constexpr int TM = MI16 ? 8 : 4, TN = MI16 ? 4 : 2;   // MFMA tiles per wave tile
  constexpr int NF = MI16 ? 1 : 2;                      // reduction steps held in fragment registers at a time
  using acc_t = typename std::conditional<MI16, f32x4_t, f32x16_t>::type;
  extern __shared__ __align__(1024) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const bool groupB = wave >= 4;

  // Work items are numbered z-major (z = batch * splits + split), tile-minor; consecutive
  // blocks go round-robin to the 8 XCDs, so XCD x owns a contiguous run of items and
  // its blocks take them interleaved: co-resident blocks work on neighbouring tiles and
  // share operand panels in their XCD's L2.
  // Sizes read on the device shrink the work list: the grid and work_total were sized for p.M.
  const int Mv = dev_bound(p.M_dev, p.M);
  const int K0 = dev_bound(p.K_dev, p.K[0]);
  const int tiles_m = p.M_dev ? (Mv + BM - 1) / BM : p.tiles_m;
  const int splits = p.dyn_split ? pp_dyn_splits(tiles_m * p.tiles_n, (K0 + BK - 1) / BK, p.splits, gridDim.x) : p.splits;
  if (p.M_dev) work_total = tiles_m * p.tiles_n * (p.dyn_split ? splits : p.nz);
  const int kper = (p.K_dev || p.dyn_split) ? (((K0 + BK - 1) / BK + splits - 1) / splits) * BK : p.kper;
  const int nt = tiles_m * p.tiles_n;
  const int xcd = blockIdx.x & 7, bidx = blockIdx.x >> 3, nbx = gridDim.x >> 3;
  const int wper = work_total >> 3, wrem = work_total & 7;
  const int wbeg = xcd * wper + (xcd < wrem ? xcd : wrem);
  const int wend = wbeg + wper + (xcd < wrem ? 1 : 0);

  struct Item {
    int m0, n0, batch, z, kbeg, kend;
  };
  auto get_item = [&](int w) {   // w in [wbeg, wend)
    Item it;
    it.z = w / nt;
    const int pid = w - it.z * nt;
    const int GROUP = p.group;    // tiles are walked in groups of `group` tile rows
    const int gsize = GROUP * p.tiles_n;
    const int gid = pid / gsize;
    const int first_m = gid * GROUP;
    const int gm = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
    const int in_g = pid - gid * gsize;
    it.m0 = (first_m + in_g % gm) * BM;
    it.n0 = (in_g / gm) * BN;
    it.batch = it.z / splits;
    const int split = it.z - it.batch * splits;
    it.kbeg = 0;
    it.kend = K0;
    if (splits > 1) {
      it.kbeg = split * kper;
      it.kend = it.kbeg + kper < K0 ? it.kbeg + kper : K0;
    }
    return it;
  };
  int nk_rest = 0;   // reduction tiles of all segments but the first
#pragma unroll
  for (int s = 1; s < kMaxSeg; ++s) nk_rest += (p.K[s] + BK - 1) / BK;

  acc_t acc[TM][TN];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < (MI16 ? 4 : 16); ++r) acc[i][j][r] = 0.f;
  };
  zero_acc();

  // ---- load stream: cursor over (item, segment, reduction tile) --------------------
  PpLoader<AKC> la;
  PpLoader<BKC> lb;
  const int64_t stepA = AKC ? BK : (int64_t)BK * p.lda[0], stepB = BKC ? BK : (int64_t)BK * p.ldb[0];
  int lw = wbeg + bidx;        // work item the cursor is in
  bool lvalid = lw < wend;     // false once every tile of this block has been issued
  int cseg = 0, ck_left = 0;
  const uint16_t *cA = nullptr, *cB = nullptr;
  int64_t offA = 0, offB = 0;
  int lbatch = 0;
  auto enter_item = [&]() {    // cursor to the first reduction tile of item lw
    const Item it = get_item(lw);
    la.init(p.lda[0], Mv - it.m0, wave, lane);
    lb.init(p.ldb[0], p.N - it.n0, wave, lane);
    offA = AKC ? (int64_t)it.m0 * p.lda[0] : it.m0;
    offB = BKC ? (int64_t)it.n0 * p.ldb[0] : it.n0;
    lbatch = it.batch;
    cseg = 0;
    ck_left = it.kend - it.kbeg;
    cA = p.A[0] + (int64_t)lbatch * p.sA[0] + offA + (AKC ? it.kbeg : (int64_t)it.kbeg * p.lda[0]);
    cB = p.B[0] + (int64_t)lbatch * p.sB[0] + offB + (BKC ? it.kbeg : (int64_t)it.kbeg * p.ldb[0]);
  };
  auto advance = [&]() {
    cA += stepA;
    cB += stepB;
    ck_left -= BK;
    if (ck_left <= 0) {
      do { ++cseg; } while (cseg < kMaxSeg && p.K[cseg] <= 0);
      if (cseg < kMaxSeg) {
        cA = p.A[cseg] + (int64_t)lbatch * p.sA[cseg] + offA;
        cB = p.B[cseg] + (int64_t)lbatch * p.sB[cseg] + offB;
        ck_left = p.K[cseg];
      } else {
        lw += nbx;
        lvalid = lw < wend;
        if (lvalid) enter_item();
      }
    }
  };
  auto issue = [&](int stage) {   // this wave's eight loads of the tile under the cursor
    unsigned char* as = smem + stage * PSTAGE;
    la.load(make_rsrc(cA), ck_left, as, wave);
    lb.load(make_rsrc(cB), ck_left, as + PTILE, wave);
    advance();
  };
  bf16x8_t af[NF][TM], bfr[NF][TN];
  uint32_t abase[TM], bbase[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
    abase[i] = MI16 ? pp16_frag_base<AKC>(wm * WM + i * 16, lane) : pp_frag_base<AKC>(wm * WM + i * 32, lane);
#pragma unroll
  for (int j = 0; j < TN; ++j)
    bbase[j] = MI16 ? pp16_frag_base<BKC>(wn * WN + j * 16, lane) : pp_frag_base<BKC>(wn * WN + j * 32, lane);
  auto read_pair = [&](int stage, int kk0) {   // fragments of the 16-wide reduction steps kk0, kk0+1
    const unsigned char* as = smem + stage * PSTAGE;
    const unsigned char* bs = as + PTILE;
    if constexpr (MI16) {                       // one 32-wide step; in the order the MFMAs consume them
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[0][j] = pp16_frag_at<BKC>(bs, bbase[j], kk0 >> 1);
#pragma unroll
      for (int i = 0; i < TM; ++i) af[0][i] = pp16_frag_at<AKC>(as, abase[i], kk0 >> 1);
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[h][j] = pp_frag_at<BKC>(bs, bbase[j], kk0 + h);
#pragma unroll
        for (int i = 0; i < TM; ++i) af[h][i] = pp_frag_at<AKC>(as, abase[i], kk0 + h);
      }
    }
  };
  auto mfma_pair = [&]() {   // the MFMAs of two 16-wide reduction steps from the fragment registers
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int h = 0; h < NF; ++h)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if constexpr (MI16)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[h][i], bfr[h][j], acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[h][i], bfr[h][j], acc[i][j], 0, 0, 0);
        }
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto tile_barrier = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr int WAIT_ALL = 0;        // s_waitcnt vmcnt(0) expcnt(0) lgkmcnt(0)

  if (!lvalid) return;               // more blocks than work items: nothing to do (whole block leaves)
  enter_item();
  issue(0);
  __builtin_amdgcn_s_waitcnt(WAIT_ALL);
  tile_barrier();                                   // barrier 0

  // Both groups run the same M0 C0 M1 C1 sequence per reduction tile; only the position
  // of the tile barrier differs, which keeps group B one phase behind group A.  Every
  // wave issues its share of the next tile's loads in M0, behind its fragment reads:
  // both groups are past barrier g there, so the stage tile g-1 has left is free, and
  // the loads have the rest of the iteration to land while the partner wave computes.
  int g = 0;                                        // reduction tiles done: stage parity
  for (int cw = wbeg + bidx; cw < wend; cw += nbx) {
    const Item it = get_item(cw);
    const int nk0 = (it.kend - it.kbeg + BK - 1) / BK;
    const int nk = (nk0 > 0 ? nk0 : 1) + nk_rest;   // an empty reduction range is one tile of zeros, as the cursor issues it
    for (int t = 0; t < nk; ++t, ++g) {
      const int cur = g & 1, nxt = cur ^ 1;
      read_pair(cur, 0);                            // M0
      if (lvalid) issue(nxt);
      mfma_pair();                                  // C0
      read_pair(cur, 2);                            // M1
      if (groupB) {
        __builtin_amdgcn_s_waitcnt(WAIT_ALL);       // fragments in registers, own loads of the next tile landed
        tile_barrier();                             // every wave is done reading stage cur
      }
      mfma_pair();                                  // C1
      if (!groupB) {
        __builtin_amdgcn_s_waitcnt(WAIT_ALL);       // own loads of the next tile landed
        tile_barrier();
      }
    }
    // item done: write it out while the next item's first tile is already in flight
    gemm_epilogue<TM, TN, OUT_BF16, VEC, DROP, 16, 64, MI16>(p, Mv, acc, smem + PP_EPI_OFF + wave * 4096, lane,
                                                       it.m0 + wm * WM, it.n0 + wn * WN, it.batch, it.z);
    zero_acc();
  }
}

// ---- the same kernel with 32-wide reduction sub-tiles in a ring of four LDS slots ----
// Three sub-tiles are in flight instead of one tile, so a load has about 2.5 sub-tile
// periods to land instead of one tile period; the price is a barrier per 16 MFMAs of a
// wave instead of per 32, and 64-byte instead of 128-byte global row segments.
constexpr int RK = 32;                       // reduction elements per sub-tile
constexpr int RTILE = 256 * RK * 2;          // bytes of one operand sub-tile (16 KiB)
constexpr int RSLOT = 2 * RTILE;
constexpr int RING_EPI_OFF = 4 * RSLOT;
constexpr int RING_SMEM = RING_EPI_OFF + 8 * 4096;

// wave-wide direct loads of one operand sub-tile: 16 loads of 1 KiB, two per wave (8 waves)
template <bool KC>
struct RingLoader {
  uint32_t voff[2];
  int kpos;
  __device__ __forceinline__ void init(int64_t ld, int rows_left, int wave, int lane) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int g = wave + 8 * j;
      if constexpr (KC) {
        // group g = rows 16g .. 16g+15 (64-byte rows); LDS slot `lane` = row lane/4, physical chunk lane%4;
        // chunks are swizzled with (row >> 2) & 3 so that 16 consecutive rows of one chunk cover all 64 banks
        const int row = g * 16 + (lane >> 2);
        const int chunk = (lane & 3) ^ ((lane >> 4) & 3);
        if (j == 0) kpos = chunk * 8;
        voff[j] = row < rows_left ? (uint32_t)(((int64_t)row * ld + chunk * 8) * 2) : kOob;
      } else {
        const int k = 2 * g + (lane >> 5);
        const int pc = lane & 31;
        const int seg = (pc >> 2) ^ (((wave & 1) << 1) + (lane >> 5));   // physical ^ (k & 3)
        const int col = (seg * 4 + (pc & 3)) * 8;
        if (j == 0) kpos = k;                                      // load j covers k-row kpos + 16 j
        voff[j] = col < rows_left ? (uint32_t)(((int64_t)k * ld + col) * 2) : kOob;
      }
    }
  }
  __device__ __forceinline__ void load(const __amdgpu_buffer_rsrc_t& rs, int k_left, unsigned char* lds_tile,
                                       int wave) const {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const bool ok = KC ? kpos < k_left : kpos + 16 * j < k_left;
      const uint32_t off = ok ? voff[j] : kOob;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_t*)(lds_tile + (wave + 8 * j) * 1024), 16, off, 0, 0, 0);
    }
  }
};
template <bool KC>
__device__ __forceinline__ uint32_t ring_frag_base(int row0, int lane) {
  if constexpr (KC) {
    const int row = row0 + (lane & 31);
    const int chunk0 = (lane >> 5) ^ ((row >> 2) & 3);
    return (uint32_t)(row * (RK * 2) + (chunk0 << 4));    // step kk: XOR (kk << 5), as in the 64-wide tiles
  } else {
    return pp_frag_base<false>(row0, lane);               // same [k][256 columns] layout, 32 k-rows
  }
}

template <bool AKC, bool BKC, bool OUT_BF16, bool VEC, bool DROP>
__global__ __launch_bounds__(512) void gemm_bf16_ring_kernel(GemmDev p, int work_total) {
  constexpr int BM = 256, BN = 256, WGN = 4;
  constexpr int WM = 128, WN = 64, TM = 4, TN = 2;
  extern __shared__ __align__(1024) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const bool groupB = wave >= 4;

  // Work items are numbered z-major (z = batch * splits + split), tile-minor; consecutive
  // blocks go round-robin to the 8 XCDs, so XCD x owns a contiguous run of items and
  // its blocks take them interleaved: co-resident blocks work on neighbouring tiles and
  // share operand panels in their XCD's L2.
  // Sizes read on the device shrink the work list: the grid and work_total were sized for p.M.
  const int Mv = dev_bound(p.M_dev, p.M);
  const int K0 = dev_bound(p.K_dev, p.K[0]);
  const int tiles_m = p.M_dev ? (Mv + BM - 1) / BM : p.tiles_m;
  if (p.M_dev) work_total = tiles_m * p.tiles_n * p.nz;
  const int kper = p.K_dev ? (((K0 + BK - 1) / BK + p.splits - 1) / p.splits) * BK : p.kper;
  const int nt = tiles_m * p.tiles_n;
  const int xcd = blockIdx.x & 7, bidx = blockIdx.x >> 3, nbx = gridDim.x >> 3;
  const int wper = work_total >> 3, wrem = work_total & 7;
  const int wbeg = xcd * wper + (xcd < wrem ? xcd : wrem);
  const int wend = wbeg + wper + (xcd < wrem ? 1 : 0);

  struct Item {
    int m0, n0, batch, z, kbeg, kend;
  };
  auto get_item = [&](int w) {   // w in [wbeg, wend)
    Item it;
    it.z = w / nt;
    const int pid = w - it.z * nt;
    const int GROUP = p.group;    // tiles are walked in groups of `group` tile rows
    const int gsize = GROUP * p.tiles_n;
    const int gid = pid / gsize;
    const int first_m = gid * GROUP;
    const int gm = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
    const int in_g = pid - gid * gsize;
    it.m0 = (first_m + in_g % gm) * BM;
    it.n0 = (in_g / gm) * BN;
    it.batch = it.z / p.splits;
    const int split = it.z - it.batch * p.splits;
    it.kbeg = 0;
    it.kend = K0;
    if (p.splits > 1) {
      it.kbeg = split * kper;
      it.kend = it.kbeg + kper < K0 ? it.kbeg + kper : K0;
    }
    return it;
  };
  int nk_rest = 0;   // reduction tiles of all segments but the first
#pragma unroll
  for (int s = 1; s < kMaxSeg; ++s) nk_rest += (p.K[s] + RK - 1) / RK;

  f32x16_t acc[TM][TN];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  };
  zero_acc();

  // ---- load stream: cursor over (item, segment, reduction tile) --------------------
  RingLoader<AKC> la;
  RingLoader<BKC> lb;
  const int64_t stepA = AKC ? RK : (int64_t)RK * p.lda[0], stepB = BKC ? RK : (int64_t)RK * p.ldb[0];
  int lw = wbeg + bidx;        // work item the cursor is in
  bool lvalid = lw < wend;     // false once every tile of this block has been issued
  int cseg = 0, ck_left = 0;
  const uint16_t *cA = nullptr, *cB = nullptr;
  int64_t offA = 0, offB = 0;
  int lbatch = 0;
  auto enter_item = [&]() {    // cursor to the first reduction tile of item lw
    const Item it = get_item(lw);
    la.init(p.lda[0], Mv - it.m0, wave, lane);
    lb.init(p.ldb[0], p.N - it.n0, wave, lane);
    offA = AKC ? (int64_t)it.m0 * p.lda[0] : it.m0;
    offB = BKC ? (int64_t)it.n0 * p.ldb[0] : it.n0;
    lbatch = it.batch;
    cseg = 0;
    ck_left = it.kend - it.kbeg;
    cA = p.A[0] + (int64_t)lbatch * p.sA[0] + offA + (AKC ? it.kbeg : (int64_t)it.kbeg * p.lda[0]);
    cB = p.B[0] + (int64_t)lbatch * p.sB[0] + offB + (BKC ? it.kbeg : (int64_t)it.kbeg * p.ldb[0]);
  };
  auto advance = [&]() {
    cA += stepA;
    cB += stepB;
    ck_left -= RK;
    if (ck_left <= 0) {
      do { ++cseg; } while (cseg < kMaxSeg && p.K[cseg] <= 0);
      if (cseg < kMaxSeg) {
        cA = p.A[cseg] + (int64_t)lbatch * p.sA[cseg] + offA;
        cB = p.B[cseg] + (int64_t)lbatch * p.sB[cseg] + offB;
        ck_left = p.K[cseg];
      } else {
        lw += nbx;
        lvalid = lw < wend;
        if (lvalid) enter_item();
      }
    }
  };
  auto issue = [&](int slot) {   // this wave's four loads of the sub-tile under the cursor
    unsigned char* as = smem + slot * RSLOT;
    la.load(make_rsrc(cA), ck_left, as, wave);
    lb.load(make_rsrc(cB), ck_left, as + RTILE, wave);
    advance();
  };
  bf16x8_t af[2][TM], bfr[2][TN];
  uint32_t abase[TM], bbase[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) abase[i] = ring_frag_base<AKC>(wm * WM + i * 32, lane);
#pragma unroll
  for (int j = 0; j < TN; ++j) bbase[j] = ring_frag_base<BKC>(wn * WN + j * 32, lane);
  auto read_pair = [&](int slot) {   // fragments of both reduction steps of a sub-tile
    const unsigned char* as = smem + slot * RSLOT;
    const unsigned char* bs = as + RTILE;
#pragma unroll
    for (int h = 0; h < 2; ++h) {   // in the order the MFMAs consume them
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[h][j] = pp_frag_at<BKC>(bs, bbase[j], h);
#pragma unroll
      for (int i = 0; i < TM; ++i) af[h][i] = pp_frag_at<AKC>(as, abase[i], h);
    }
  };
  auto mfma_pair = [&]() {   // 16 MFMAs from the fragment registers
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[h][i], bfr[h][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto tile_barrier = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr int WAIT_ALL = 0;        // s_waitcnt vmcnt(0) expcnt(0) lgkmcnt(0)

  if (!lvalid) return;               // more blocks than work items: nothing to do (whole block leaves)
  enter_item();
  issue(0);
  if (lvalid) issue(1);
  if (lvalid) issue(2);
  __builtin_amdgcn_s_waitcnt(WAIT_ALL);
  tile_barrier();                                   // barrier 0: sub-tiles 0..2 are in LDS

  // Per sub-tile s (slot s & 3): M(s) = 12 fragment reads + this wave's 4 loads of sub-tile s+3 (into the slot
  // sub-tile s-1 has left: every wave is past barrier s-1 there), C(s) = 16 MFMAs.  Group A takes barrier s after
  // C(s), group B after M(s), so B runs one phase behind A.  Before barrier s a wave has its own loads of sub-tile
  // s+1 in LDS; the eight younger ones (s+2, s+3) stay in flight: a load has about 2.5 sub-tile periods to land.
  constexpr int WAIT_BUT_8 = 0x0078;  // vmcnt(8) lgkmcnt(0)
  int g = 0;                                        // sub-tiles done: slot = g & 3
  for (int cw = wbeg + bidx; cw < wend; cw += nbx) {
    const Item it = get_item(cw);
    const int nk0 = (it.kend - it.kbeg + RK - 1) / RK;
    const int nk = (nk0 > 0 ? nk0 : 1) + nk_rest;   // an empty reduction range is one sub-tile of zeros, as the cursor issues it
    for (int t = 0; t < nk; ++t, ++g) {
      const int slot = g & 3;
      read_pair(slot);                              // M
      const bool more = lvalid;                     // the cursor still has sub-tiles: the in-flight count below holds
      if (lvalid) issue((g + 3) & 3);
      if (groupB) {
        if (more) __builtin_amdgcn_s_waitcnt(WAIT_BUT_8); else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
        tile_barrier();                             // every wave is done reading this slot
      }
      mfma_pair();                                  // C
      if (!groupB) {
        if (more) __builtin_amdgcn_s_waitcnt(WAIT_BUT_8); else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
        tile_barrier();
      }
    }
    // item done: write it out while the next item's first sub-tiles are already in flight
    gemm_epilogue<TM, TN, OUT_BF16, VEC, DROP, 16, 64>(p, Mv, acc, smem + RING_EPI_OFF + wave * 4096, lane,
                                                       it.m0 + wm * WM, it.n0 + wn * WN, it.batch, it.z);
    zero_acc();
  }
}

template <bool AKC, bool BKC, bool OUT_BF16, bool VEC>
static hipError_t launch_ring(const GemmDev& d, int batch, hipStream_t st) {
  constexpr int smem = RING_SMEM;
  auto kfn = gemm_bf16_ring_kernel<AKC, BKC, OUT_BF16, VEC, false>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int work_total = d.tiles_m * d.tiles_n * batch * d.splits;
  const int blocks = pp_grid_blocks(work_total);
  hipLaunchKernelGGL(kfn, dim3(blocks), dim3(512), smem, st, d, work_total);
  return hipGetLastError();
}
template <bool AKC, bool BKC>
static hipError_t launch_ring_oriented(const GemmArgs& g, const GemmDev& d, hipStream_t st) {
  const bool obf = g.c_bf16 && g.splits <= 1;
  const bool vec = d.vec_ok != 0;
  if (obf) return vec ? launch_ring<AKC, BKC, true, true>(d, g.batch, st) : launch_ring<AKC, BKC, true, false>(d, g.batch, st);
  return vec ? launch_ring<AKC, BKC, false, true>(d, g.batch, st) : launch_ring<AKC, BKC, false, false>(d, g.batch, st);
}

template <int BM, int BN, int WGM, int WGN, bool AKC, bool BKC, bool OUT_BF16, bool VEC, bool DROP = false>
static hipError_t launch_one(const GemmDev& d, int batch, hipStream_t st) {
  constexpr int smem = 2 * (BM + BN) * ROWB;
  auto kfn = gemm_bf16_kernel<BM, BN, WGM, WGN, AKC, BKC, OUT_BF16, VEC, DROP>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid(d.tiles_m * d.tiles_n, 1, batch * d.splits);
  hipLaunchKernelGGL(kfn, grid, dim3(64 * WGM * WGN), smem, st, d);
  return hipGetLastError();
}

template <bool AKC, bool BKC, bool OUT_BF16, bool VEC, bool DROP = false>
static hipError_t launch_pp(const GemmDev& d, int batch, hipStream_t st) {
  constexpr int smem = PP_SMEM;
  auto kfn = gemm_bf16_pp_kernel<AKC, BKC, OUT_BF16, VEC, DROP, AKC && BKC>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  // persistent: one block per CU (a multiple of the 8 XCDs), each walking its share of the work items
  const int work_total = d.tiles_m * d.tiles_n * batch * d.splits;
  const int blocks = pp_grid_blocks(work_total);
  hipLaunchKernelGGL(kfn, dim3(blocks), dim3(512), smem, st, d, work_total);
  return hipGetLastError();
}

// operand orientations x output type x epilogue form -> kernel instance
template <bool BIG, bool AKC, bool BKC>
static hipError_t launch_oriented(const GemmArgs& g, const GemmDev& d, hipStream_t st) {
  const bool obf = g.c_bf16 && g.splits <= 1;
  const bool vec = d.vec_ok != 0;
  if (d.drop_thr) {   // dropout variants exist for the one product that uses them (both operands reduction-contiguous)
    if constexpr (AKC && BKC) {
      if constexpr (BIG) {
        if (obf) return vec ? launch_pp<true, true, true, true, true>(d, g.batch, st) : launch_pp<true, true, true, false, true>(d, g.batch, st);
        return vec ? launch_pp<true, true, false, true, true>(d, g.batch, st) : launch_pp<true, true, false, false, true>(d, g.batch, st);
      } else {
        if (obf)
          return vec ? launch_one<128, 128, 2, 2, true, true, true, true, true>(d, g.batch, st)
                     : launch_one<128, 128, 2, 2, true, true, true, false, true>(d, g.batch, st);
        return vec ? launch_one<128, 128, 2, 2, true, true, false, true, true>(d, g.batch, st)
                   : launch_one<128, 128, 2, 2, true, true, false, false, true>(d, g.batch, st);
      }
    } else {
      return hipErrorInvalidValue;
    }
  }
  if constexpr (BIG) {
    if (obf) return vec ? launch_pp<AKC, BKC, true, true>(d, g.batch, st) : launch_pp<AKC, BKC, true, false>(d, g.batch, st);
    return vec ? launch_pp<AKC, BKC, false, true>(d, g.batch, st) : launch_pp<AKC, BKC, false, false>(d, g.batch, st);
  } else {
    if (obf)
      return vec ? launch_one<128, 128, 2, 2, AKC, BKC, true, true>(d, g.batch, st)
                 : launch_one<128, 128, 2, 2, AKC, BKC, true, false>(d, g.batch, st);
    return vec ? launch_one<128, 128, 2, 2, AKC, BKC, false, true>(d, g.batch, st)
               : launch_one<128, 128, 2, 2, AKC, BKC, false, false>(d, g.batch, st);
  }
}

template <bool BIG>
static hipError_t launch_tile(const GemmArgs& g, const GemmDev& d, hipStream_t st) {
  if (g.a_kc && g.b_kc) return launch_oriented<BIG, true, true>(g, d, st);
  if (g.a_kc && !g.b_kc) return launch_oriented<BIG, true, false>(g, d, st);
  if (!g.a_kc && !g.b_kc) return launch_oriented<BIG, false, false>(g, d, st);
  return hipErrorInvalidValue;  // (A strided, B contiguous) is not used by the path
}

static bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

hipError_t launch_gemm_bf16(const GemmArgs& g, int big_tile, hipStream_t st) {
  if (g.M < 1 || g.N < 1 || g.batch < 1 || g.splits < 1) return hipErrorInvalidValue;
  // split-K: the combine step applies the epilogue; the persistent kernel splits a single segment only
  if (g.splits > 1 && (g.partial == nullptr || (big_tile && g.K[1] != 0))) return hipErrorInvalidValue;
  if (g.drop_thr && g.batch != 1) return hipErrorInvalidValue;   // flat element index = m * N + n
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
      // 16-byte vector loads: leading dimensions and batch strides in units of 8 elements;
      // 32-bit byte offsets inside one 256-row (or 64-reduction-row) tile
      if ((g.lda[s] & 7) || (g.ldb[s] & 7) || (g.sA[s] & 7) || (g.sB[s] & 7)) return hipErrorInvalidValue;
      if (g.lda[s] >= (1 << 22) || g.ldb[s] >= (1 << 22)) return hipErrorInvalidValue;
      if (g.lda[s] != g.lda[0] || g.ldb[s] != g.ldb[0]) return hipErrorInvalidValue;  // one set of lane offsets
      if (!al16(g.A[s]) || !al16(g.B[s])) return hipErrorInvalidValue;
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
  d.drop_thr = g.splits > 1 ? 0u : g.drop_thr;   // with split-K the combine step applies the epilogue
  d.drop_scale = g.drop_scale;
  d.drop_seed = g.drop_seed;
  d.accumulate = g.accumulate;
  d.splits = g.splits;
  d.partial = g.partial;
  if (g.M_dev && g.batch != 1) return hipErrorInvalidValue;
  if (g.K_dev && g.K[1] != 0) return hipErrorInvalidValue;
  d.M_dev = g.M_dev;
  d.K_dev = g.K_dev;
  d.nz = g.batch * g.splits;
  // a split chosen in the kernel: persistent two-stage kernel, rows counted on the device, partial sums always
  if (g.dyn_split && (!big_tile || !g.M_dev || g.splits < 2 || (!g.a_kc && !g.b_kc))) return hipErrorInvalidValue;
  d.dyn_split = g.dyn_split ? 1 : 0;
  // vector epilogue: every row of C / C_lo / C_dact / gate starts 16-byte aligned
  // (ldc % 4 == 0 gives 8-byte alignment for bf16 rows, which their 8-byte stores need)
  d.vec_ok = ((g.ldc & 3) == 0) && ((g.sC & 3) == 0) && al16(g.C) && (!g.C_lo || al16(g.C_lo)) &&
             (!g.C_dact || al16(g.C_dact)) && (!g.gate || (al16(g.gate) && (g.ldg & 3) == 0)) &&
             (g.N & 3) == 0 &&                                            // a 4-column group is all in or all out
             g.ldc < (1 << 21) && g.ldg < (1 << 21) && g.N < (1 << 21);   // 32-bit byte offsets inside a 128-row window
  const int bm = big_tile ? 256 : 128;
  d.tiles_m = (g.M + bm - 1) / bm;
  d.tiles_n = (g.N + bm - 1) / bm;
  // many column tiles: 8 rows x 4 columns of co-resident tiles per XCD share 12 operand panels; few column
  // tiles (long-reduction products): whole tile rows, so a row panel is consumed in one go (measured 2-3 % faster)
  d.group = d.tiles_n >= 16 ? 8 : (16 / d.tiles_n < 2 ? 2 : (16 / d.tiles_n > 8 ? 8 : 16 / d.tiles_n));
  int ktiles = 0;   // reduction tiles of all segments (the persistent kernel splits segment 0 alone, checked above)
  for (int s = 0; s < kMaxSeg; ++s) ktiles += (g.K[s] + BK - 1) / BK;
  d.kper = ((ktiles + g.splits - 1) / g.splits) * BK;
  if (g.splits > 1 && !g.dyn_split && (int64_t)(d.kper / BK) * (g.splits - 1) >= ktiles)
    return hipErrorInvalidValue;   // an empty split
  // Both operands strided in the reduction index (the weight-gradient products): their global rows are
  // 512 contiguous bytes whatever the reduction width, so the ring variant's deeper prefetch is free
  // (measured +7 %); with a reduction-contiguous operand its 64-byte row segments cost more than they hide.
  if (big_tile && !g.a_kc && !g.b_kc && !d.drop_thr) return launch_ring_oriented<false, false>(g, d, st);
  return big_tile ? launch_tile<true>(g, d, st) : launch_tile<false>(g, d, st);
}

}  // namespace asx
