// Vocabulary softmax cross-entropy (Eq. 5-6 of section 3.2) without ever
// forming the probability matrix: a streaming statistics pass (online max /
// sum-exp, target logit, argmax) and an in-place pass that turns the stored
// logits into dlogits = g*(p - onehot) while summing the columns for db_out.
// Both passes are pure HBM streams: 16-byte loads/stores, fp32 arithmetic.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace asx {

// 16-byte load of data that is read once (streamed past the caches)
typedef uint32_t xe_u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16_stream(const void* p) {
  const xe_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const xe_u32x4_t*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void st16_stream(void* p, const uint4& q) {
  const xe_u32x4_t v = {q.x, q.y, q.z, q.w};
  __builtin_nontemporal_store(v, reinterpret_cast<xe_u32x4_t*>(p));
}

template <typename TE> struct Vec;
template <> struct Vec<uint16_t> { static constexpr int N = 8; };
template <> struct Vec<float> { static constexpr int N = 4; };

template <typename TE>
__device__ __forceinline__ void unpack(const uint4& q, float (&f)[Vec<TE>::N]) {
  if constexpr (sizeof(TE) == 2) {
    f[0] = lo_bf16(q.x); f[1] = hi_bf16(q.x); f[2] = lo_bf16(q.y); f[3] = hi_bf16(q.y);
    f[4] = lo_bf16(q.z); f[5] = hi_bf16(q.z); f[6] = lo_bf16(q.w); f[7] = hi_bf16(q.w);
  } else {
    f[0] = __builtin_bit_cast(float, q.x); f[1] = __builtin_bit_cast(float, q.y);
    f[2] = __builtin_bit_cast(float, q.z); f[3] = __builtin_bit_cast(float, q.w);
  }
}
template <typename TE>
__device__ __forceinline__ uint4 pack(const float (&f)[Vec<TE>::N]) {
  uint4 q;
  if constexpr (sizeof(TE) == 2) {
    q.x = pack_bf16(f[0], f[1]); q.y = pack_bf16(f[2], f[3]);
    q.z = pack_bf16(f[4], f[5]); q.w = pack_bf16(f[6], f[7]);
  } else {
    q.x = __builtin_bit_cast(uint32_t, f[0]); q.y = __builtin_bit_cast(uint32_t, f[1]);
    q.z = __builtin_bit_cast(uint32_t, f[2]); q.w = __builtin_bit_cast(uint32_t, f[3]);
  }
  return q;
}

// running (max, sum of exp relative to max, lowest index of the max)
struct RowStat {
  float m, s;
  int idx;
};
__device__ __forceinline__ RowStat combine(const RowStat& a, const RowStat& b) {
  RowStat r;
  r.m = fmaxf(a.m, b.m);
  const float sa = a.m == r.m ? 1.f : __expf(a.m - r.m);
  const float sb = b.m == r.m ? 1.f : __expf(b.m - r.m);
  r.s = a.s * sa + b.s * sb;
  r.idx = a.m > b.m ? a.idx : (b.m > a.m ? b.idx : (a.idx < b.idx ? a.idx : b.idx));
  return r;
}

// UNR loads in flight per thread, all streaming (4 to 8 in flight measure the same).  A plain read stream with the
// same grid and loads moves 6.8 TB/s on this part when it runs alone; the first form of this kernel, which updated
// the running maximum and its index per element, reached 5.4 inside the step, this one 5.7: a wave's
// vector instruction occupies its 16-lane SIMD for four cycles, so every operation per element counts.  Per
// element this form spends: one shift / mask to widen bf16, half a v_max3, one fused multiply-add into the base-2
// exponent, one v_exp_f32, one add.  The running maximum is updated once per group of UNR vectors instead of per
// vector, and the arg max is tracked at vector granularity (column of the first vector of the thread that attains
// the maximum); the element inside that vector is found once per row by re-reading 16 bytes.
template <typename TE, int UNR = 8>
__global__ __launch_bounds__(256) void xent_stats_kernel(const TE* __restrict__ logits, int64_t ldV, int V,
                                                        const int32_t* __restrict__ targets, int pad_id,
                                                        float* __restrict__ lse, float* __restrict__ tok_loss_ws,
                                                        float* __restrict__ tok_loss, int32_t* __restrict__ argmax,
                                                        uint8_t* __restrict__ tgt_mask,
                                                        const int32_t* __restrict__ rows,
                                                        const int32_t* __restrict__ n_act) {
  constexpr int VEC = Vec<TE>::N;
  constexpr float L2E = 1.4426950408889634f;
  constexpr uint32_t NEG_INF_WORD = sizeof(TE) == 2 ? 0xff80ff80u : 0xff800000u;   // -inf in every element
  // compacted rows (rows != null): logits row r belongs to position rows[r]; lse and the workspace loss are
  // indexed by r, the caller's per-position outputs by the position
  const int n = blockIdx.x, tid = threadIdx.x;
  if (rows && n >= *n_act) return;
  const int pos = rows ? rows[n] : n;
  const TE* x = logits + (int64_t)n * ldV;
  RowStat st{-INFINITY, 0.f, 0x7fffffff};   // idx: column of the first element of the vector holding the first maximum
  // one group = UNR vectors of this thread, 256 * VEC columns apart; GUARD: the group may reach past the row
  auto group = [&](int v0, auto guard) {
    constexpr bool GUARD = decltype(guard)::value;
    // UNR independent 16-byte loads per thread are issued before any of them is used: a row is read once, so
    // the only way to cover the memory latency is to have enough bytes in flight per compute unit
    uint4 q[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int v = v0 + u * 256 * VEC;
      if constexpr (GUARD) {
        q[u] = make_uint4(NEG_INF_WORD, NEG_INF_WORD, NEG_INF_WORD, NEG_INF_WORD);   // a vector past the row: all -inf
        if (v < V) q[u] = ld16_stream(x + v);
      } else {
        q[u] = ld16_stream(x + v);
      }
    }
    float f[UNR][VEC], vm[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int v = v0 + u * 256 * VEC;
      unpack<TE>(q[u], f[u]);
      if constexpr (GUARD) {
        if (v < V && v + VEC > V) {           // the one ragged vector of a row whose length is not a multiple of VEC
#pragma unroll
          for (int i = 0; i < VEC; ++i)
            if (v + i >= V) f[u][i] = -INFINITY;
        }
      }
      float a = f[u][0];
#pragma unroll
      for (int i = 1; i + 1 < VEC; i += 2) a = fmaxf(fmaxf(a, f[u][i]), f[u][i + 1]);   // v_max3_f32
      if constexpr (VEC % 2 == 0) a = fmaxf(a, f[u][VEC - 1]);
      vm[u] = a;
    }
    float gm = fmaxf(fmaxf(vm[0], vm[1]), vm[2]);
#pragma unroll
    for (int u = 3; u + 1 < UNR; u += 2) gm = fmaxf(fmaxf(gm, vm[u]), vm[u + 1]);
    if constexpr (UNR % 2 == 0) gm = fmaxf(gm, vm[UNR - 1]);
    if (gm > st.m) {                          // strict: an equal maximum further right does not move the arg max
      st.s *= __builtin_amdgcn_exp2f((st.m - gm) * L2E);   // exp2(-inf) = 0 the first time
      st.m = gm;
      int first = 0;
#pragma unroll
      for (int u = UNR - 1; u >= 0; --u)      // lowest u (= lowest column of this thread) attaining gm
        if (vm[u] == gm) first = u;
      st.idx = v0 + first * 256 * VEC;
    }
    const float mb = -st.m * L2E;
    float e0 = 0.f, e1 = 0.f;                 // two chains: the adds do not wait on each other
#pragma unroll
    for (int u = 0; u < UNR; ++u)
#pragma unroll
      for (int i = 0; i < VEC; i += 2) {
        e0 += __builtin_amdgcn_exp2f(__builtin_fmaf(f[u][i], L2E, mb));
        e1 += __builtin_amdgcn_exp2f(__builtin_fmaf(f[u][i + 1], L2E, mb));
      }
    st.s += e0 + e1;
  };
  static_assert(UNR >= 3, "group maximum is taken with v_max3");
  constexpr int STEP = 256 * VEC * UNR;
  int v0 = tid * VEC;
  for (; v0 + (UNR - 1) * 256 * VEC + VEC <= V; v0 += STEP) group(v0, std::false_type{});
  if (v0 < V) group(v0, std::true_type{});
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    RowStat other;
    other.m = __shfl_xor(st.m, o, 64);
    other.s = __shfl_xor(st.s, o, 64);
    other.idx = __shfl_xor(st.idx, o, 64);
    st = combine(st, other);
  }
  __shared__ RowStat ws[4];
  if ((tid & 63) == 0) ws[tid >> 6] = st;
  __syncthreads();
  if (tid == 0) {
    RowStat r = combine(combine(ws[0], ws[1]), combine(ws[2], ws[3]));
    // the vectors of a row are disjoint column ranges, so the lowest vector column among equal maxima holds the
    // lowest arg max; find the element inside it
    int amax = 0;
    if (r.idx < V) {
      float f[VEC];
      unpack<TE>(*reinterpret_cast<const uint4*>(x + r.idx), f);
      int k = VEC - 1;
#pragma unroll
      for (int i = VEC - 1; i >= 0; --i)
        if (r.idx + i < V && f[i] == r.m) k = i;
      amax = r.idx + k;
    }
    const float l = r.m + logf(r.s);
    const int y = targets[pos];
    const bool nonpad = (y != pad_id) && (y >= 0) && (y < V);
    const float loss = nonpad ? l - ld_elem<TE>(x, y) : 0.f;
    lse[n] = l;
    tok_loss_ws[n] = loss;
    if (tok_loss) tok_loss[pos] = loss;
    if (argmax) argmax[pos] = amax;
    if (tgt_mask) tgt_mask[pos] = nonpad ? 1 : 0;
  }
}

__global__ __launch_bounds__(1024) void loss_reduce_kernel(const float* __restrict__ tok_loss_ws,
                                                          const int32_t* __restrict__ targets, int N, int V,
                                                          int pad_id, float* loss_sum, int32_t* n_tok,
                                                          const int32_t* __restrict__ n_act) {
  __shared__ double sd[1024];
  __shared__ int sc[1024];
  const int tid = threadIdx.x;
  double acc = 0.0;
  int cnt = 0;
  if (n_act) {   // compacted rows: the first *n_act entries are the non-pad positions
    const int na = *n_act;
    for (int i = tid; i < na; i += 1024) acc += (double)tok_loss_ws[i];
    cnt = tid == 0 ? na : 0;
  } else {
    for (int i = tid; i < N; i += 1024) {
      acc += (double)tok_loss_ws[i];
      const int y = targets[i];
      cnt += ((y != pad_id) && (y >= 0) && (y < V)) ? 1 : 0;
    }
  }
  sd[tid] = acc;
  sc[tid] = cnt;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (tid < o) { sd[tid] += sd[tid + o]; sc[tid] += sc[tid + o]; }
    __syncthreads();
  }
  if (tid == 0) { *loss_sum = (float)sd[0]; *n_tok = sc[0]; }
}

// RU rows in flight per thread; NT: 1 = streaming loads, 2 = streaming stores, 3 = both.  Measured on
// 12288 x 128000 bf16: (4, 0) 4.93 TB/s, (4, 3) 5.02, (8, 3) 5.09; a plain device copy moves 4.7-5.3.
template <typename TE, int RU = 8, int NT = 3>
__global__ __launch_bounds__(256) void xent_dlogits_kernel(TE* __restrict__ logits, int64_t ldV, int N, int V,
                                                          const int32_t* __restrict__ targets, int pad_id,
                                                          const float* __restrict__ lse, float g, int RB,
                                                          float* __restrict__ db_partial,
                                                          const int32_t* __restrict__ rows,
                                                          const int32_t* __restrict__ n_act) {
  constexpr int VEC = Vec<TE>::N;
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * VEC;
  if (c0 >= ldV) return;
  if (rows) N = *n_act;                 // compacted rows: row r belongs to position rows[r]; blocks past the
  const int r0 = blockIdx.y * RB;       // last row still store their (zero) column sums
  const int r1 = r0 + RB < N ? r0 + RB : N;
  float cs[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) cs[i] = 0.f;
  for (int r = r0; r < r1; r += RU) {   // RU rows of loads in flight per thread
    uint4 q[RU];
    bool live[RU];
    int y[RU];
    float l[RU];
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      const int rr = r + u;
      live[u] = false;
      y[u] = -1;
      l[u] = 0.f;
      q[u] = make_uint4(0, 0, 0, 0);
      if (rr < r1) {
        y[u] = targets[rows ? rows[rr] : rr];
        live[u] = (y[u] != pad_id) && (y[u] >= 0) && (y[u] < V);
        if (live[u]) {                      // pad rows are not read, only zeroed
          l[u] = lse[rr];
          q[u] = (NT & 1) ? ld16_stream(logits + (int64_t)rr * ldV + c0)
                          : *reinterpret_cast<const uint4*>(logits + (int64_t)rr * ldV + c0);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      const int rr = r + u;
      if (rr >= r1) break;
      float f[VEC], d[VEC];
      unpack<TE>(q[u], f);
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        float v = 0.f;
        if (live[u] && c0 + i < V) v = g * (__expf(f[i] - l[u]) - (c0 + i == y[u] ? 1.f : 0.f));
        d[i] = v;
        cs[i] += v;
      }
      if (NT & 2) st16_stream(logits + (int64_t)rr * ldV + c0, pack<TE>(d));
      else *reinterpret_cast<uint4*>(logits + (int64_t)rr * ldV + c0) = pack<TE>(d);
    }
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i)
    if (c0 + i < V) db_partial[(int64_t)blockIdx.y * V + c0 + i] = cs[i];
}

// 64 columns x 4 phases per block: phase p adds the row blocks p, p+4, ... of its column, the four sums meet
// in LDS; the order of the additions is fixed
__global__ __launch_bounds__(256) void db_reduce_kernel(const float* __restrict__ db_partial, int nrb, int V,
                                                       float* __restrict__ db_out) {
  __shared__ float red[4][64];
  const int c = threadIdx.x & 63, phase = threadIdx.x >> 6;
  const int v = blockIdx.x * 64 + c;
  float s = 0.f;
  if (v < V)
    for (int r = phase; r < nrb; r += 4) s += db_partial[(int64_t)r * V + v];
  red[phase][c] = s;
  __syncthreads();
  if (phase == 0 && v < V) db_out[v] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
}

// ---- launchers ----------------------------------------------------------------
hipError_t launch_xent_stats(const void* logits, int64_t ldV, bool e_bf16, int N, int V,
                             const int32_t* targets, int pad_id, float* lse, float* tok_loss_ws,
                             float* tok_loss, int32_t* argmax, uint8_t* tgt_mask, const int32_t* rows,
                             const int32_t* n_act, hipStream_t st) {
  if (e_bf16)
    hipLaunchKernelGGL(xent_stats_kernel<uint16_t>, dim3(N), dim3(256), 0, st,
                       reinterpret_cast<const uint16_t*>(logits), ldV, V, targets, pad_id, lse, tok_loss_ws,
                       tok_loss, argmax, tgt_mask, rows, n_act);
  else
    hipLaunchKernelGGL(xent_stats_kernel<float>, dim3(N), dim3(256), 0, st,
                       reinterpret_cast<const float*>(logits), ldV, V, targets, pad_id, lse, tok_loss_ws, tok_loss,
                       argmax, tgt_mask, rows, n_act);
  return hipGetLastError();
}

hipError_t launch_loss_reduce(const float* tok_loss_ws, const int32_t* targets, int N, int V, int pad_id,
                              float* loss_sum, int32_t* n_tok, const int32_t* n_act, hipStream_t st) {
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, st, tok_loss_ws, targets, N, V, pad_id, loss_sum,
                     n_tok, n_act);
  return hipGetLastError();
}

int xent_rows_per_block(int N, int V, bool e_bf16) {
  const int vec = e_bf16 ? 8 : 4;
  const int64_t ldV = ((int64_t)V + 7) / 8 * 8;
  const int64_t strips = (ldV + 256 * vec - 1) / (256 * vec);
  int64_t rb = ((int64_t)N * strips + 4095) / 4096;
  if (rb < 8) rb = 8;
  if (rb > 256) rb = 256;
  return (int)((rb + 3) / 4 * 4);
}

hipError_t launch_xent_dlogits(void* logits, int64_t ldV, bool e_bf16, int N, int V, const int32_t* targets,
                               int pad_id, const float* lse, float g, float* db_partial, const int32_t* rows,
                               const int32_t* n_act, hipStream_t st) {
  const int vec = e_bf16 ? 8 : 4;
  const int RB = xent_rows_per_block(N, V, e_bf16);
  dim3 grid((unsigned)((ldV + 256 * vec - 1) / (256 * vec)), (N + RB - 1) / RB);
  if (e_bf16)
    hipLaunchKernelGGL(xent_dlogits_kernel<uint16_t>, grid, dim3(256), 0, st, reinterpret_cast<uint16_t*>(logits),
                       ldV, N, V, targets, pad_id, lse, g, RB, db_partial, rows, n_act);
  else
    hipLaunchKernelGGL(xent_dlogits_kernel<float>, grid, dim3(256), 0, st, reinterpret_cast<float*>(logits), ldV, N,
                       V, targets, pad_id, lse, g, RB, db_partial, rows, n_act);
  return hipGetLastError();
}

hipError_t launch_db_reduce(const float* db_partial, int nrb, int V, float* db_out, hipStream_t st) {
  hipLaunchKernelGGL(db_reduce_kernel, dim3((V + 63) / 64), dim3(256), 0, st, db_partial, nrb, V, db_out);
  return hipGetLastError();
}

}  // namespace asx
