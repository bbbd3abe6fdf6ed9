// Plain streaming kernels with the access patterns of the two cross-entropy kernels and nothing of their
// arithmetic: what this GPU's memory system gives a read-only stream, a copy and an in-place
// read-modify-write over the same bytes.  A measurement aid (attn_softmax_stream_probe); bench.py reports
// the cross-entropy kernels next to these ceilings.
#include "common.h"
#include "kernels.h"

namespace asx {

typedef uint32_t sp_u32x4_t __attribute__((ext_vector_type(4)));

// One 256-thread block per chunk (a logits row), UNR independent 16-byte streaming loads in flight per thread:
// the load pattern of the statistics kernel.  The words are folded with XOR into one value per block.
template <int UNR>
__global__ __launch_bounds__(256) void stream_read_kernel(const unsigned char* __restrict__ src, size_t chunk,
                                                         uint32_t* __restrict__ sink) {
  const unsigned char* x = src + (size_t)blockIdx.x * chunk;
  uint32_t acc = 0;
  for (size_t o = (size_t)threadIdx.x * 16; o < chunk; o += (size_t)256 * 16 * UNR) {
    sp_u32x4_t q[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const size_t a = o + (size_t)u * 256 * 16;
      q[u] = sp_u32x4_t{0, 0, 0, 0};
      if (a < chunk) q[u] = __builtin_nontemporal_load(reinterpret_cast<const sp_u32x4_t*>(x + a));
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) acc ^= q[u][0] ^ q[u][1] ^ q[u][2] ^ q[u][3];
  }
  acc ^= __shfl_xor(acc, 32, 64);
  if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = acc;
}

// Grid of (2048-column strips x row blocks), each thread owns 16 bytes of a row and walks RB rows with RU rows of
// loads in flight: the pattern of the dlogits kernel.  dst == src: in-place read-modify-write; dst != src: copy.
template <int RU>
__global__ __launch_bounds__(256) void stream_rw_kernel(const unsigned char* __restrict__ src,
                                                       unsigned char* __restrict__ dst, size_t row_bytes, int rows,
                                                       int RB, uint32_t flip) {
  const size_t c0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (c0 >= row_bytes) return;
  const int r0 = blockIdx.y * RB;
  const int r1 = r0 + RB < rows ? r0 + RB : rows;
  for (int r = r0; r < r1; r += RU) {
    sp_u32x4_t q[RU];
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      q[u] = sp_u32x4_t{0, 0, 0, 0};
      if (r + u < r1) q[u] = __builtin_nontemporal_load(reinterpret_cast<const sp_u32x4_t*>(src + (size_t)(r + u) * row_bytes + c0));
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      if (r + u >= r1) break;
      const sp_u32x4_t v = {q[u][0] ^ flip, q[u][1] ^ flip, q[u][2] ^ flip, q[u][3] ^ flip};
      __builtin_nontemporal_store(v, reinterpret_cast<sp_u32x4_t*>(dst + (size_t)(r + u) * row_bytes + c0));
    }
  }
}

hipError_t launch_stream_probe(int kind, void* buf, void* buf2, int rows, size_t row_bytes, hipStream_t st) {
  if (kind == 0) {
    hipLaunchKernelGGL(stream_read_kernel<8>, dim3(rows), dim3(256), 0, st, reinterpret_cast<const unsigned char*>(buf),
                       row_bytes, reinterpret_cast<uint32_t*>(buf2));
  } else {
    const int64_t strips = (int64_t)((row_bytes + 4095) / 4096);
    int64_t rb = ((int64_t)rows * strips + 4095) / 4096;   // the row blocking of the dlogits kernel
    rb = rb < 8 ? 8 : (rb > 256 ? 256 : rb);
    const int RB = (int)((rb + 3) / 4 * 4);
    dim3 grid((unsigned)strips, (rows + RB - 1) / RB);
    unsigned char* s = reinterpret_cast<unsigned char*>(buf);
    unsigned char* d = kind == 1 ? reinterpret_cast<unsigned char*>(buf2) : s;
    hipLaunchKernelGGL(stream_rw_kernel<8>, grid, dim3(256), 0, st, s, d, row_bytes, rows, RB, 0x80008000u);
  }
  return hipGetLastError();
}

}  // namespace asx
