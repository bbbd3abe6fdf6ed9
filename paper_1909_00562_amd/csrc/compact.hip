// Row compaction for the vocabulary part of the path (Eq. 5-6 and its backward).
// A target position that is padding contributes nothing to the loss or to any
// gradient, so the three products over the vocabulary and the two cross-entropy
// passes need only the rows n = t*B + b whose target is a word.  These kernels
// number those rows in increasing n (the list is made on the device: nothing is
// copied to the host and the stream is never synchronised), gather the rows of
// h_c and of the saved tanh derivative into a dense [n_act, H] block, and scatter
// the rows of dz back to their time-major places with zeros at the padding rows.
#include "common.h"
#include "kernels.h"

namespace asx {

// One block walks the N targets in slices of 1024 and counts the non-pad ones before each
// position (ballot + popcount inside a wave, 16 wave totals through LDS): fixed order, no atomics.
__global__ __launch_bounds__(1024) void row_compact_kernel(const int32_t* __restrict__ targets, int N, int V,
                                                          int pad_id, int32_t* __restrict__ row_pos,
                                                          int32_t* __restrict__ rows, int32_t* __restrict__ n_act,
                                                          uint8_t* __restrict__ tgt_mask, float* __restrict__ tok_loss,
                                                          int32_t* __restrict__ argmax) {
  __shared__ int wave_total[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int base = 0;
  for (int n0 = 0; n0 < N; n0 += 1024) {
    const int n = n0 + tid;
    bool live = false;
    if (n < N) {
      const int y = targets[n];
      live = (y != pad_id) && (y >= 0) && (y < V);
    }
    const unsigned long long votes = __ballot(live);
    const int before = __popcll(votes & ((1ull << lane) - 1ull));
    if (lane == 0) wave_total[wave] = __popcll(votes);
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const int c = wave_total[w];
      woff += w < wave ? c : 0;
      total += c;
    }
    if (n < N) {
      const int pos = base + woff + before;
      row_pos[n] = live ? pos : -1;
      if (live) rows[pos] = n;
      if (tgt_mask) tgt_mask[n] = live ? 1 : 0;
      if (!live) {
        if (tok_loss) tok_loss[n] = 0.f;
        if (argmax) argmax[n] = pad_id;
      }
    }
    base += total;
    __syncthreads();   // wave_total is rewritten by the next slice
  }
  if (tid == 0) *n_act = base;
}

// bytes of one row are a multiple of 4; 16-byte vectors when they are a multiple of 16 (row starts are then aligned)
__device__ __forceinline__ void copy_row(const unsigned char* __restrict__ src, unsigned char* __restrict__ dst,
                                         int64_t bytes, int tid, int nthreads) {
  if ((bytes & 15) == 0) {
    for (int64_t i = (int64_t)tid * 16; i < bytes; i += (int64_t)nthreads * 16)
      *reinterpret_cast<uint4*>(dst + i) = *reinterpret_cast<const uint4*>(src + i);
  } else {
    for (int64_t i = (int64_t)tid * 4; i < bytes; i += (int64_t)nthreads * 4)
      *reinterpret_cast<uint32_t*>(dst + i) = *reinterpret_cast<const uint32_t*>(src + i);
  }
}
__device__ __forceinline__ void zero_row(unsigned char* __restrict__ dst, int64_t bytes, int tid, int nthreads) {
  if ((bytes & 15) == 0) {
    for (int64_t i = (int64_t)tid * 16; i < bytes; i += (int64_t)nthreads * 16)
      *reinterpret_cast<uint4*>(dst + i) = make_uint4(0, 0, 0, 0);
  } else {
    for (int64_t i = (int64_t)tid * 4; i < bytes; i += (int64_t)nthreads * 4)
      *reinterpret_cast<uint32_t*>(dst + i) = 0u;
  }
}

// dst_x[r] = src_x[rows[r]] for r < *n_act, two arrays per launch (row sizes in bytes; src1 may be null)
__global__ __launch_bounds__(256) void gather_rows_kernel(const int32_t* __restrict__ rows,
                                                         const int32_t* __restrict__ n_act,
                                                         const unsigned char* __restrict__ src0,
                                                         unsigned char* __restrict__ dst0, int64_t bytes0,
                                                         const unsigned char* __restrict__ src1,
                                                         unsigned char* __restrict__ dst1, int64_t bytes1) {
  const int r = blockIdx.x;
  if (r >= *n_act) return;
  const int64_t n = rows[r];
  copy_row(src0 + n * bytes0, dst0 + (int64_t)r * bytes0, bytes0, threadIdx.x, 256);
  if (src1) copy_row(src1 + n * bytes1, dst1 + (int64_t)r * bytes1, bytes1, threadIdx.x, 256);
}

// dst_x[n] = src_x[row_pos[n]] where row_pos[n] >= 0, else zeros; every row of dst is written
__global__ __launch_bounds__(256) void scatter_rows_kernel(const int32_t* __restrict__ row_pos,
                                                          const unsigned char* __restrict__ src0,
                                                          unsigned char* __restrict__ dst0,
                                                          const unsigned char* __restrict__ src1,
                                                          unsigned char* __restrict__ dst1, int64_t bytes) {
  const int64_t n = blockIdx.x;
  const int64_t r = row_pos[n];
  if (r >= 0) {
    copy_row(src0 + r * bytes, dst0 + n * bytes, bytes, threadIdx.x, 256);
    if (src1) copy_row(src1 + r * bytes, dst1 + n * bytes, bytes, threadIdx.x, 256);
  } else {
    zero_row(dst0 + n * bytes, bytes, threadIdx.x, 256);
    if (src1) zero_row(dst1 + n * bytes, bytes, threadIdx.x, 256);
  }
}

hipError_t launch_row_compact(const int32_t* targets, int N, int V, int pad_id, int32_t* row_pos, int32_t* rows,
                              int32_t* n_act, uint8_t* tgt_mask, float* tok_loss, int32_t* argmax, hipStream_t st) {
  hipLaunchKernelGGL(row_compact_kernel, dim3(1), dim3(1024), 0, st, targets, N, V, pad_id, row_pos, rows, n_act,
                     tgt_mask, tok_loss, argmax);
  return hipGetLastError();
}

hipError_t launch_gather_rows(const int32_t* rows, const int32_t* n_act, int N, const void* src0, void* dst0,
                              int64_t bytes0, const void* src1, void* dst1, int64_t bytes1, hipStream_t st) {
  if ((bytes0 & 3) || (bytes1 & 3)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(N), dim3(256), 0, st, rows, n_act,
                     reinterpret_cast<const unsigned char*>(src0), reinterpret_cast<unsigned char*>(dst0), bytes0,
                     reinterpret_cast<const unsigned char*>(src1), reinterpret_cast<unsigned char*>(dst1), bytes1);
  return hipGetLastError();
}

hipError_t launch_scatter_rows(const int32_t* row_pos, int N, const void* src0, void* dst0, const void* src1,
                               void* dst1, int64_t bytes, hipStream_t st) {
  if (bytes & 3) return hipErrorInvalidValue;
  hipLaunchKernelGGL(scatter_rows_kernel, dim3(N), dim3(256), 0, st, row_pos,
                     reinterpret_cast<const unsigned char*>(src0), reinterpret_cast<unsigned char*>(dst0),
                     reinterpret_cast<const unsigned char*>(src1), reinterpret_cast<unsigned char*>(dst1), bytes);
  return hipGetLastError();
}

}  // namespace asx
