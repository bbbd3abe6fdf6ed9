// Host-side description of one (optionally batched, optionally multi-segment)
// matrix product  C[m,n] = epilogue( sum_seg sum_k A_seg(m,k) * B_seg(n,k) ).
// Segments let one launch add several products into the same accumulators:
// the two halves of W_c [c ; h], or the high and low bf16 parts of an operand
// that was produced inside the path and must not lose its fp32 precision.
//
// Operand addressing (elements of the storage type):
//   a_kc : A(m,k) = A[m*lda + k]   (reduction index contiguous)
//   !a_kc: A(m,k) = A[k*lda + m]   (stored transposed: row index = k)
//   b_kc : B(n,k) = B[n*ldb + k]
//   !b_kc: B(n,k) = B[k*ldb + n]
// The bf16 kernels read 16-byte vectors along the contiguous index, so for a
// bf16 operand: base pointers and batch strides are 16-byte aligned, ld % 8 == 0,
// the allocation extends to a multiple of 8 along the contiguous index, and when
// the reduction index is the contiguous one and K % 8 != 0 the padding elements
// up to the next multiple of 8 must be zero.  The fp32 kernel has no such needs.
//
// Epilogue, applied in this order:  v = acc; v += bias[n]; v = tanh(v) if act;
// v *= gate[m,n] if gate; v += C_old[m,n] if accumulate (fp32 C only);
// C[m,n] = v rounded to the output type.  Optional second outputs with C's
// layout:  C_lo[m,n] = v - C[m,n] (type of C), the part of v the rounding lost;
// C_dact[m,n] = 1 - v^2 as float (the tanh derivative, taken before v is rounded).
// Dropout (drop_thr != 0, after the activation): element (m,n) draws the 32-bit word
// philox4x32-10(counter = (m*N + n) >> 2, key = drop_seed)[(m*N + n) & 3]; it is kept iff
// word >= drop_thr.  Kept: v and C_dact are multiplied by drop_scale; dropped: both are 0,
// so that a later product with C_dact as its gate also backpropagates through the mask.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asx {

constexpr int kMaxSeg = 6;

struct GemmArgs {
  const void* A[kMaxSeg] = {};
  const void* B[kMaxSeg] = {};
  int64_t lda[kMaxSeg] = {}, ldb[kMaxSeg] = {};
  int64_t sA[kMaxSeg] = {}, sB[kMaxSeg] = {};  // batch strides
  int K[kMaxSeg] = {};                         // K[s] = 0: segment unused
  int nseg = 0;
  void seg(const void* a, int64_t lda_, int64_t sa_, const void* b, int64_t ldb_, int64_t sb_, int k) {
    A[nseg] = a; lda[nseg] = lda_; sA[nseg] = sa_;
    B[nseg] = b; ldb[nseg] = ldb_; sB[nseg] = sb_;
    K[nseg] = k; ++nseg;
  }
  bool a_kc = true, b_kc = true;
  int M = 0, N = 0;
  void* C = nullptr;
  int64_t ldc = 0, sC = 0;
  bool c_bf16 = false;          // output storage: bf16 bits or float
  void* C_lo = nullptr;         // optional rounding remainder of C
  float* C_dact = nullptr;      // optional 1 - v^2 (float)
  const void* bias = nullptr;   // [N], storage type of the inputs
  const float* gate = nullptr;  // [M,ldg] multiplier (float)
  int64_t ldg = 0;
  int act_tanh = 0;
  int accumulate = 0;
  uint32_t drop_thr = 0;        // 0 = no dropout
  float drop_scale = 1.f;       // 1 / (1 - p)
  uint64_t drop_seed = 0;
  int batch = 1;
  int splits = 1;               // split of the reduction index (single segment only)
  float* partial = nullptr;     // [batch*splits, M, N] floats when splits > 1
  // Sizes known only on the device (a row count made by an earlier kernel of the same stream).  M and K[0]
  // stay the upper bounds every grid, plan and buffer is sized for; a kernel reads the count once and
  // uses min(count, bound) in their place: rows >= *M_dev of A are not read and of C not written, reduction
  // indices >= *K_dev of segment 0 are not read (so neither operand has to be defined there).
  const int32_t* M_dev = nullptr;   // batch == 1 only
  const int32_t* K_dev = nullptr;   // single segment only
  // With M_dev, the 256x256 persistent kernel and a product of few, long work items (fewer output tiles than a
  // few rounds of the grid): `splits` (>= 2) is then only the bound `partial` is sized for; the kernel picks the
  // split of the reduction from the row count it reads (pp_dyn_splits below), so that the shrunken work list
  // still fills whole rounds of the grid, and the combine step, which always runs, picks the same.
  bool dyn_split = false;
};

// Blocks of a persistent launch (one per compute unit, a multiple of the 8 XCDs).
inline int pp_grid_blocks(int work_total) { return work_total < 256 ? (work_total + 7) / 8 * 8 : 256; }

// Reduction split for `tiles` output tiles of `ktiles` reduction tiles each on `blocks` persistent blocks.  Cost in
// sixteenths of one reduction tile of one block: rounds of the grid times (the split's tiles + 6 for an item's
// prologue and epilogue), plus the round trip of each split's fp32 partial through HBM (256x256x8 bytes per
// tile, spread over the chip: about 7/6 sixteenths per tile and split).  Integer arithmetic: the product
// kernel and the combine kernel must arrive at the same number.
__host__ __device__ inline int pp_dyn_splits(int tiles, int ktiles, int smax, int blocks) {
  int best = 1;
  long long best_cost = -1;
  for (int s = 1; s <= smax; ++s) {
    const int per = (ktiles + s - 1) / s;
    if (s > 1 && (long long)per * (s - 1) >= ktiles) continue;   // a split would be empty
    const long long rounds = ((long long)tiles * s + blocks - 1) / blocks;
    const long long cost = rounds * (per + 6) * 16 + (long long)s * tiles * 7 / 6;
    if (best_cost < 0 || cost < best_cost) {
      best_cost = cost;
      best = s;
    }
  }
  return best;
}

// Tile plan shared by workspace sizing and launching.
struct GemmPlan {
  int big_tile;   // bf16: 1 = 256x256 block tile, 0 = 128x128
  int splits;
};
// multi_segment: the reduction runs over several operand segments; only the 128x128 kernel can split those
GemmPlan gemm_plan(int M, int N, int K, int batch, bool bf16, bool allow_split, bool multi_segment = false);
inline size_t gemm_partial_bytes(int M, int N, int batch, int splits) {
  return splits > 1 ? (size_t)splits * batch * M * N * sizeof(float) : 0;
}

// Enqueue; return hipSuccess or the launch error.  `in_bf16` selects the kernel family.
hipError_t launch_gemm(const GemmArgs& g, bool in_bf16, int big_tile, hipStream_t st);
hipError_t launch_gemm_bf16(const GemmArgs& g, int big_tile, hipStream_t st);
hipError_t launch_gemm_f32(const GemmArgs& g, hipStream_t st);
// partial[batch*splits][M][N] -> C with the epilogue of g
hipError_t launch_splitk_combine(const GemmArgs& g, bool in_bf16, hipStream_t st);

}  // namespace asx
