// Stacked LSTM without input feeding (section 3.2, Fig. 3; cell as stated in
// include/lstm_stack.h): forward and backward over all steps of one side.
//
// Per layer, forward: the input half of the gate pre-activations of ALL steps is
// one large product (X W_ih^T + b, [T*B, 4H]); then one step after the other adds
// the recurrent half (h_{t-1} W_hh^T) and applies the cell.  Backward walks the
// steps in reverse (cell derivative, then dh_{t-1} = da_t W_hh), after which the
// weight gradients and the gradient of the layer's input are again large
// products over all steps at once.  Right-padded sentences keep their state at
// steps t >= lengths[b]; their gate gradients are zero rows, so the large
// products need no masking.
#include "../../include/lstm_stack.h"

#include <vector>

#include "common.h"
#include "gemm.h"
#include "kernels.h"
#include "status.h"

namespace asx {

__device__ __forceinline__ float sigmoid_f(float a) { return 1.f / (1.f + expf(-a)); }

// State before the first step: h as float, c, and h in the storage type (hE0, row-major: the operand of dW_hh).
// bf16 storage also gets h as (value, rounding remainder) in the fragment-major form [H/8][B][8] the fused
// step kernel reads (hF_hi / hF_lo, else null).
template <typename TE>
__global__ __launch_bounds__(256) void lstm_init_kernel(const float* __restrict__ h0, const float* __restrict__ c0,
                                                       int B, int H, float* __restrict__ hf,
                                                       float* __restrict__ cs0, TE* __restrict__ hE0,
                                                       TE* __restrict__ hF_hi, TE* __restrict__ hF_lo) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= B * H) return;
  const float h = h0 ? h0[i] : 0.f;
  hf[i] = h;
  st_elem<TE>(hE0, i, h);
  cs0[i] = c0 ? c0[i] : 0.f;
  if (hF_hi) {
    const int b = i / H, j = i - b * H;
    const int64_t f = ((int64_t)(j >> 3) * B + b) * 8 + (j & 7);
    st_elem<TE>(hF_hi, f, h);
    st_elem<TE>(hF_lo, f, h - round_elem<TE>(h));
  }
}

// fp32 storage: the cell after the recurrent product has been added by a separate launch.
// G [B,4H]: in = gate pre-activations of step t, out = i, f, g, o (kept for the backward pass).
// hf: running h; h_prev / h_new: h before / after the step (operand of the next step's product and of
// dW_hh); out: the layer's output of step t (0 at padded steps).
__global__ __launch_bounds__(256) void lstm_cell_fwd_kernel(float* __restrict__ G, const float* __restrict__ c_prev,
                                                           float* __restrict__ c_new, float* __restrict__ hf,
                                                           const float* __restrict__ h_prev, float* __restrict__ h_new,
                                                           float* __restrict__ out, const int32_t* __restrict__ lengths,
                                                           int t, int T, int B, int H, uint32_t drop_thr,
                                                           float drop_scale, uint64_t drop_seed,
                                                           uint64_t drop_index0) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * H) return;
  const int b = idx / H, j = idx - b * H;
  int len = lengths[b];
  len = len < 0 ? 0 : (len > T ? T : len);
  float* g4 = G + (int64_t)b * 4 * H + j;
  const float i = sigmoid_f(g4[0]), f = sigmoid_f(g4[H]), g = tanhf(g4[2 * H]), o = sigmoid_f(g4[3 * H]);
  g4[0] = i; g4[H] = f; g4[2 * H] = g; g4[3 * H] = o;
  const float cp = c_prev[idx];
  if (t < len) {
    const float cn = f * cp + i * g;
    const float hn = o * tanhf(cn);
    c_new[idx] = cn;
    hf[idx] = hn;
    h_new[idx] = hn;
    // dropout on what the next layer reads (drop_thr = 0: none)
    out[idx] = drop_thr ? hn * dropout_mult(drop_index0 + (uint64_t)idx, drop_seed, drop_thr, drop_scale) : hn;
  } else {
    c_new[idx] = cp;
    h_new[idx] = h_prev[idx];
    out[idx] = 0.f;
  }
}

// fp32 storage.  dhs / dcs: gradient w.r.t. the state after step t (in) and, for dcs, after step t-1 (out).
// Valid rows write their gate gradients da_t and clear dhs, which the product da_t W_hh then fills; padded
// rows write zero gate gradients and pass dhs, dcs through.
__global__ __launch_bounds__(256) void lstm_cell_bwd_kernel(const float* __restrict__ gates,
                                                           const float* __restrict__ c_prev,
                                                           const float* __restrict__ c_new,
                                                           const float* __restrict__ dout_t, float* __restrict__ dhs,
                                                           float* __restrict__ dcs, float* __restrict__ dG_t,
                                                           const int32_t* __restrict__ lengths, int t, int T, int B,
                                                           int H, uint32_t drop_thr, float drop_scale,
                                                           uint64_t drop_seed, uint64_t drop_index0) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * H) return;
  const int b = idx / H, j = idx - b * H;
  int len = lengths[b];
  len = len < 0 ? 0 : (len > T ? T : len);
  float* d4 = dG_t + (int64_t)b * 4 * H + j;
  if (t < len) {
    const float* g4 = gates + (int64_t)b * 4 * H + j;
    const float i = g4[0], f = g4[H], g = g4[2 * H], o = g4[3 * H];
    float dy = dout_t[idx];   // back through the mask the forward pass put on this layer's output
    if (drop_thr) dy *= dropout_mult(drop_index0 + (uint64_t)idx, drop_seed, drop_thr, drop_scale);
    const float dh = dy + dhs[idx];
    const float tc = tanhf(c_new[idx]);
    const float dc = dcs[idx] + dh * o * (1.f - tc * tc);
    d4[0] = dc * g * i * (1.f - i);
    d4[H] = dc * c_prev[idx] * f * (1.f - f);
    d4[2 * (int64_t)H] = dc * i * (1.f - g * g);
    d4[3 * (int64_t)H] = dh * tc * o * (1.f - o);
    dcs[idx] = dc * f;
    dhs[idx] = 0.f;
  } else {
    d4[0] = 0.f; d4[H] = 0.f; d4[2 * (int64_t)H] = 0.f; d4[3 * (int64_t)H] = 0.f;
  }
}

// dst = src, or zeros when src is null
__global__ __launch_bounds__(256) void lstm_copy_or_zero_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                               int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src ? src[i] : 0.f;
}

// Column sums of da [rows, cols] (+ its rounding remainders, bf16 storage) over blocks of 64 rows:
// part[rb][col], summed by db_reduce in a fixed order.  A thread owns 16 bytes of a row (8 bf16 or 4 float
// columns; cols is a multiple of that: 4H with H % 8 == 0 for bf16, 4H for fp32); the block's 256 threads are
// 64 column groups x 4 row phases (rows r0 + phase, + 4, ...), whose sums meet in LDS in a fixed order.
template <typename TE>
__global__ __launch_bounds__(256) void lstm_bias_partial_kernel(const TE* __restrict__ dG,
                                                               const TE* __restrict__ dGlo, int rows, int cols,
                                                               float* __restrict__ part) {
  constexpr int VEC = 16 / sizeof(TE);
  __shared__ float red[4][64][VEC];
  const int cg = threadIdx.x & 63, phase = threadIdx.x >> 6;
  const int col = (blockIdx.x * 64 + cg) * VEC;
  const int r0 = blockIdx.y * 64;
  const int r1 = r0 + 64 < rows ? r0 + 64 : rows;
  float s[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) s[i] = 0.f;
  auto add = [&](const TE* base, int r) {
    const uint4 q = *reinterpret_cast<const uint4*>(base + (int64_t)r * cols + col);
    if constexpr (sizeof(TE) == 2) {
      s[0] += lo_bf16(q.x); s[1] += hi_bf16(q.x); s[2] += lo_bf16(q.y); s[3] += hi_bf16(q.y);
      s[4] += lo_bf16(q.z); s[5] += hi_bf16(q.z); s[6] += lo_bf16(q.w); s[7] += hi_bf16(q.w);
    } else {
      s[0] += __builtin_bit_cast(float, q.x); s[1] += __builtin_bit_cast(float, q.y);
      s[2] += __builtin_bit_cast(float, q.z); s[3] += __builtin_bit_cast(float, q.w);
    }
  };
  if (col < cols) {
#pragma unroll 4
    for (int r = r0 + phase; r < r1; r += 4) {
      add(dG, r);
      if (dGlo) add(dGlo, r);
    }
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) red[phase][cg][i] = s[i];
  __syncthreads();
  if (phase == 0 && col < cols) {
#pragma unroll
    for (int i = 0; i < VEC; ++i)
      part[(int64_t)blockIdx.y * cols + col + i] = ((red[0][cg][i] + red[1][cg][i]) + red[2][cg][i]) + red[3][cg][i];
  }
}

namespace {

constexpr size_t kAlignL = 256;
size_t upl(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct LsLayout {
  size_t e;
  int64_t TB, BH;
  std::vector<size_t> gates, cs, hE, out, out_lo;   // per layer; out_lo: bf16 storage only
  size_t hf, dGE, dGlo, dhs, dcs, dio[2], dbpart, partial, total;
  // bf16 storage: fragment-major operands of the fused step kernels
  size_t Wfrag;            // W_hh (forward) or its transpose (backward) of the layer being processed
  size_t hF[2][2];         // h of the previous / next step, [slot][value, remainder]
  size_t dGF[2];           // gate gradients (bf16 values) of the next / this step
  int nrb;
  std::vector<GemmPlan> p_gx, p_dwi, p_dx;
  GemmPlan p_rec, p_drec, p_dwh;
};

bool ls_shape_ok(const ls_shape* s) {
  if (!s) return false;
  if (s->T < 1 || s->B < 1 || s->I < 1 || s->H < 1 || s->L < 1 || s->L > 16) return false;
  if (s->dtype != AS_F32 && s->dtype != AS_BF16) return false;
  if (!(s->dropout_p >= 0.f && s->dropout_p < 1.f)) return false;
  if (s->dtype == AS_BF16 && ((s->I % 8) != 0 || (s->H % 8) != 0)) return false;
  if ((int64_t)s->T * s->B > (1 << 24) || s->H > (1 << 16) || s->I > (1 << 16)) return false;
  if ((int64_t)s->T * s->B * 4 * s->H > ((int64_t)1 << 34)) return false;
  return true;
}

LsLayout make_ls_layout(const ls_shape* s) {
  LsLayout L;
  const bool bf = s->dtype == AS_BF16;
  const int T = s->T, B = s->B, I = s->I, H = s->H, NL = s->L;
  L.e = bf ? 2 : 4;
  L.TB = (int64_t)T * B;
  L.BH = (int64_t)B * H;
  const int TB = (int)L.TB;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += upl(bytes, kAlignL);
    return o;
  };
  size_t pb = 0;
  auto mx = [&](size_t v) { if (v > pb) pb = v; };
  for (int l = 0; l < NL; ++l) {
    const int Il = l == 0 ? I : H;
    L.gates.push_back(take((size_t)TB * 4 * H * 4));
    L.cs.push_back(take((size_t)(T + 1) * L.BH * 4));
    L.hE.push_back(take((size_t)(T + 1) * L.BH * L.e));
    L.out.push_back(l + 1 < NL ? take((size_t)TB * H * L.e) : 0);
    L.out_lo.push_back(bf && l + 1 < NL ? take((size_t)TB * H * L.e) : 0);
    // bf16: the output of the layer below and the gate gradients are (value, remainder) pairs: two segments
    L.p_gx.push_back(gemm_plan(TB, 4 * H, (bf && l > 0) ? 2 * Il : Il, 1, bf, false));
    L.p_dwi.push_back(gemm_plan(4 * H, Il, TB, 1, bf, true));
    {
      // The reduction split of this product is a function of the layer's widths alone: with a split chosen
      // from the row count, a sentence's gradients would depend (in the last fp32 bit, then through bf16
      // roundings below) on how many sentences share its batch.
      GemmPlan px = gemm_plan(TB, Il, 4 * H, 1, bf, false);
      if (bf) {
        const int ktiles = (4 * H + 63) / 64, want = Il >= 1024 ? 2 : 4;
        px.splits = ktiles / 8 < 1 ? 1 : (ktiles / 8 < want ? ktiles / 8 : want);
        px.big_tile = 1;
      }
      L.p_dx.push_back(px);
      mx(gemm_partial_bytes(TB, Il, 1, px.splits));
    }
    mx(gemm_partial_bytes(4 * H, Il, 1, L.p_dwi.back().splits));
  }
  L.p_rec = gemm_plan(B, 4 * H, H, 1, false, true);      // the per-step products as launches of their own: fp32 only
  L.p_drec = gemm_plan(B, H, 4 * H, 1, false, true);
  L.p_dwh = gemm_plan(4 * H, H, TB, 1, bf, true);
  if (!bf) {
    mx(gemm_partial_bytes(B, 4 * H, 1, L.p_rec.splits));
    mx(gemm_partial_bytes(B, H, 1, L.p_drec.splits));
  }
  mx(gemm_partial_bytes(4 * H, H, 1, L.p_dwh.splits));
  L.hf = take((size_t)L.BH * 4);
  L.dGE = take((size_t)TB * 4 * H * L.e);
  L.dGlo = bf ? take((size_t)TB * 4 * H * L.e) : 0;
  L.dhs = take((size_t)L.BH * 4);
  L.dcs = take((size_t)L.BH * 4);
  const size_t wmax = (size_t)(I > H ? I : H);
  L.dio[0] = take((size_t)TB * wmax * 4);
  L.dio[1] = take((size_t)TB * wmax * 4);
  L.nrb = (TB + 63) / 64;
  L.dbpart = take((size_t)L.nrb * 4 * H * 4);
  L.partial = take(pb);
  L.Wfrag = bf ? take((size_t)4 * H * H * L.e) : 0;
  for (int sl = 0; sl < 2; ++sl) {
    for (int k = 0; k < 2; ++k) L.hF[sl][k] = bf ? take((size_t)L.BH * L.e) : 0;
    L.dGF[sl] = bf ? take((size_t)4 * L.BH * L.e) : 0;
  }
  L.total = off;
  return L;
}

bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

as_status check_ptr_array(const void* const* arr, int n, const char* name) {
  if (!arr) return set_error(AS_ERR_NULL, "%s is NULL", name);
  for (int l = 0; l < n; ++l) {
    if (!arr[l]) return set_error(AS_ERR_NULL, "%s[%d] is NULL", name, l);
    if (!al16(arr[l])) return set_error(AS_ERR_ALIGN, "%s[%d] = %p is not 16-byte aligned", name, l, arr[l]);
  }
  return AS_OK;
}

as_status check_ls(const ls_shape* s, void* ws, size_t ws_bytes, LsLayout* L) {
  if (!s) return set_error(AS_ERR_NULL, "shape is NULL");
  if (s->dtype != AS_F32 && s->dtype != AS_BF16) return set_error(AS_ERR_DTYPE, "unknown dtype %d", s->dtype);
  if (s->dtype == AS_BF16 && s->T >= 1 && s->B >= 1 && s->I >= 1 && s->H >= 1 && ((s->I % 8) != 0 || (s->H % 8) != 0))
    return set_error(AS_ERR_ALIGN, "AS_BF16 needs I %% 8 == 0 and H %% 8 == 0 (I=%d H=%d)", s->I, s->H);
  if (!ls_shape_ok(s))
    return set_error(AS_ERR_SHAPE, "bad shape T=%d B=%d I=%d H=%d L=%d dropout_p=%g", s->T, s->B, s->I, s->H, s->L,
                     (double)s->dropout_p);
  if (!ws) return set_error(AS_ERR_NULL, "workspace is NULL");
  if (!al16(ws)) return set_error(AS_ERR_ALIGN, "workspace %p is not 16-byte aligned", ws);
  *L = make_ls_layout(s);
  if (ws_bytes < L->total) return set_error(AS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L->total);
  return AS_OK;
}

#define LS_TRY(expr)                                                                            \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess) return set_error(AS_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

template <typename TE>
as_status ls_fwd(const ls_shape* s, const LsLayout& L, const char* x, const int32_t* lengths,
                 const void* const* W_ih, const void* const* W_hh, const void* const* b, const float* h0,
                 const float* c0, char* y, float* hT, float* cT, char* w, hipStream_t st) {
  constexpr bool bf = sizeof(TE) == 2;
  const int T = s->T, B = s->B, I = s->I, H = s->H, NL = s->L;
  const int TB = (int)L.TB, BH = (int)L.BH;
  const int nb = (BH + 255) / 256;
  float* hf = reinterpret_cast<float*>(w + L.hf);
  const char* xin = x;
  const char* xin_lo = nullptr;   // the caller's x is exact in the storage type
  for (int l = 0; l < NL; ++l) {
    const int Il = l == 0 ? I : H;
    float* gates = reinterpret_cast<float*>(w + L.gates[l]);
    float* cs = reinterpret_cast<float*>(w + L.cs[l]);
    TE* hE = reinterpret_cast<TE*>(w + L.hE[l]);
    TE* out = reinterpret_cast<TE*>(l + 1 < NL ? w + L.out[l] : y);
    TE* out_lo = (bf && l + 1 < NL) ? reinterpret_cast<TE*>(w + L.out_lo[l]) : nullptr;
    // dropout sits between the layers: on what layer l+1 reads, never on the top layer's output
    const uint32_t drop_thr = (l + 1 < NL && s->dropout_p > 0.f) ? (uint32_t)((double)s->dropout_p * 4294967296.0) : 0u;
    const float drop_scale = 1.f / (1.f - s->dropout_p);
    TE* hF[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};
    if (bf)
      for (int sl = 0; sl < 2; ++sl)
        for (int k = 0; k < 2; ++k) hF[sl][k] = reinterpret_cast<TE*>(w + L.hF[sl][k]);
    hipLaunchKernelGGL(lstm_init_kernel<TE>, dim3(nb), dim3(256), 0, st, h0 ? h0 + (size_t)l * BH : nullptr,
                       c0 ? c0 + (size_t)l * BH : nullptr, B, H, hf, cs, hE, hF[0][0], hF[0][1]);
    LS_TRY(hipGetLastError());
    {  // input half of the pre-activations of all steps: X W_ih^T + b
      GemmArgs g;
      g.seg(xin, Il, 0, W_ih[l], Il, 0, Il);
      if (xin_lo) g.seg(xin_lo, Il, 0, W_ih[l], Il, 0, Il);
      g.a_kc = true; g.b_kc = true;
      g.M = TB; g.N = 4 * H; g.bias = b[l];
      g.C = gates; g.ldc = 4 * H; g.c_bf16 = false;
      LS_TRY(launch_gemm(g, bf, L.p_gx[l].big_tile, st));
    }
    if constexpr (bf) {   // one kernel per step: recurrent product and cell
      uint16_t* WF = reinterpret_cast<uint16_t*>(w + L.Wfrag);
      LS_TRY(launch_ls_wfrag(W_hh[l], WF, H, false, st));
      for (int t = 0; t < T; ++t) {
        LstmStepFwd f;
        f.WF = WF;
        f.hF_hi = hF[t & 1][0]; f.hF_lo = hF[t & 1][1];
        f.hFn_hi = hF[(t + 1) & 1][0]; f.hFn_lo = hF[(t + 1) & 1][1];
        f.G = gates + (size_t)t * B * 4 * H;
        f.c_prev = cs + (size_t)t * BH; f.c_new = cs + (size_t)(t + 1) * BH; f.hf = hf;
        f.hE_new = hE + (size_t)(t + 1) * BH;
        f.out = out + (size_t)t * BH; f.out_lo = out_lo ? out_lo + (size_t)t * BH : nullptr;
        f.lengths = lengths; f.t = t; f.T = T; f.B = B; f.H = H;
        f.drop_thr = drop_thr; f.drop_scale = drop_scale; f.drop_seed = s->dropout_seed;
        f.drop_index0 = ((uint64_t)l * T + t) * (uint64_t)BH;
        LS_TRY(launch_lstm_step_fwd(f, st));
      }
    } else {              // fp32: the recurrent product and the cell as two launches per step
      float* partial = reinterpret_cast<float*>(w + L.partial);
      for (int t = 0; t < T; ++t) {
        float* Gt = gates + (size_t)t * B * 4 * H;
        GemmArgs g;       // + h_{t-1} W_hh^T
        g.seg(hE + (size_t)t * BH, H, 0, W_hh[l], H, 0, H);
        g.a_kc = true; g.b_kc = true;
        g.M = B; g.N = 4 * H;
        g.C = Gt; g.ldc = 4 * H; g.c_bf16 = false; g.accumulate = 1;
        g.splits = L.p_rec.splits; g.partial = partial;
        LS_TRY(launch_gemm(g, false, L.p_rec.big_tile, st));
        hipLaunchKernelGGL(lstm_cell_fwd_kernel, dim3(nb), dim3(256), 0, st, Gt, cs + (size_t)t * BH,
                           cs + (size_t)(t + 1) * BH, hf, hE + (size_t)t * BH, hE + (size_t)(t + 1) * BH,
                           out + (size_t)t * BH, lengths, t, T, B, H, drop_thr, drop_scale, s->dropout_seed,
                           ((uint64_t)l * T + t) * (uint64_t)BH);
        LS_TRY(hipGetLastError());
      }
    }
    if (hT) LS_TRY(hipMemcpyAsync(hT + (size_t)l * BH, hf, (size_t)BH * 4, hipMemcpyDeviceToDevice, st));
    if (cT) LS_TRY(hipMemcpyAsync(cT + (size_t)l * BH, cs + (size_t)T * BH, (size_t)BH * 4, hipMemcpyDeviceToDevice, st));
    xin = reinterpret_cast<const char*>(out);
    xin_lo = reinterpret_cast<const char*>(out_lo);
  }
  return AS_OK;
}

template <typename TE>
as_status ls_bwd(const ls_shape* s, const LsLayout& L, const char* x, const int32_t* lengths,
                 const void* const* W_ih, const void* const* W_hh, const float* dy, const float* dhT,
                 const float* dcT, char* w, float* dx, float* const* dW_ih, float* const* dW_hh, float* const* db,
                 float* dh0, float* dc0, hipStream_t st) {
  constexpr bool bf = sizeof(TE) == 2;
  const int T = s->T, B = s->B, I = s->I, H = s->H, NL = s->L;
  const int TB = (int)L.TB, BH = (int)L.BH;
  const int nb = (BH + 255) / 256;
  float* partial = reinterpret_cast<float*>(w + L.partial);
  TE* dGE = reinterpret_cast<TE*>(w + L.dGE);
  TE* dGlo = bf ? reinterpret_cast<TE*>(w + L.dGlo) : nullptr;
  float* dhs = reinterpret_cast<float*>(w + L.dhs);
  float* dcs = reinterpret_cast<float*>(w + L.dcs);
  float* dbpart = reinterpret_cast<float*>(w + L.dbpart);
  const float* dout = dy;
  for (int l = NL - 1; l >= 0; --l) {
    const int Il = l == 0 ? I : H;
    const float* gates = reinterpret_cast<const float*>(w + L.gates[l]);
    const float* cs = reinterpret_cast<const float*>(w + L.cs[l]);
    const TE* hE = reinterpret_cast<const TE*>(w + L.hE[l]);
    const char* xin = l == 0 ? x : w + L.out[l - 1];
    const float* dhT_l = dhT ? dhT + (size_t)l * BH : nullptr;
    const uint32_t drop_thr = (l + 1 < NL && s->dropout_p > 0.f) ? (uint32_t)((double)s->dropout_p * 4294967296.0) : 0u;
    const float drop_scale = 1.f / (1.f - s->dropout_p);
    hipLaunchKernelGGL(lstm_copy_or_zero_kernel, dim3(nb), dim3(256), 0, st, dcT ? dcT + (size_t)l * BH : nullptr, dcs, BH);
    LS_TRY(hipGetLastError());
    if constexpr (bf) {   // one kernel per step: da_{t+1} W_hh and the cell derivative of step t
      uint16_t* WTF = reinterpret_cast<uint16_t*>(w + L.Wfrag);
      LS_TRY(launch_ls_wfrag(W_hh[l], WTF, H, true, st));
      uint16_t* dGF[2];
      for (int sl = 0; sl < 2; ++sl) dGF[sl] = reinterpret_cast<uint16_t*>(w + L.dGF[sl]);
      for (int t = T - 1; t >= -1; --t) {   // t = -1: the product alone, for the gradient of the initial h
        LstmStepBwd q;
        q.WTF = WTF;
        q.dGnF = t + 1 < T ? dGF[(t + 1) & 1] : nullptr;
        q.dhT = dhT_l;
        q.dcs = dcs;
        q.lengths = lengths; q.t = t; q.T = T; q.B = B; q.H = H;
        q.drop_thr = drop_thr; q.drop_scale = drop_scale; q.drop_seed = s->dropout_seed;
        q.drop_index0 = ((uint64_t)l * T + (t < 0 ? 0 : t)) * (uint64_t)BH;
        q.gates = nullptr; q.c_prev = q.c_new = q.dout_t = nullptr;
        q.dG_hi = q.dG_lo = q.dGF = nullptr;
        q.dh0_out = dhs;
        if (t >= 0) {
          q.gates = gates + (size_t)t * B * 4 * H;
          q.c_prev = cs + (size_t)t * BH; q.c_new = cs + (size_t)(t + 1) * BH;
          q.dout_t = dout + (size_t)t * BH;
          q.dG_hi = dGE + (size_t)t * B * 4 * H; q.dG_lo = dGlo + (size_t)t * B * 4 * H;
          q.dGF = dGF[t & 1];
        }
        LS_TRY(launch_lstm_step_bwd(q, st));
      }
    } else {              // fp32: cell derivative and product as two launches per step
      hipLaunchKernelGGL(lstm_copy_or_zero_kernel, dim3(nb), dim3(256), 0, st, dhT_l, dhs, BH);
      LS_TRY(hipGetLastError());
      for (int t = T - 1; t >= 0; --t) {
        float* dGt = dGE + (size_t)t * B * 4 * H;
        hipLaunchKernelGGL(lstm_cell_bwd_kernel, dim3(nb), dim3(256), 0, st, gates + (size_t)t * B * 4 * H,
                           cs + (size_t)t * BH, cs + (size_t)(t + 1) * BH, dout + (size_t)t * BH, dhs, dcs, dGt, lengths,
                           t, T, B, H, drop_thr, drop_scale, s->dropout_seed, ((uint64_t)l * T + t) * (uint64_t)BH);
        LS_TRY(hipGetLastError());
        GemmArgs g;       // dh_{t-1} (+)= da_t W_hh: valid rows were cleared, padded rows have da_t = 0 and keep theirs
        g.seg(dGt, 4 * H, 0, W_hh[l], H, 0, 4 * H);
        g.a_kc = true; g.b_kc = false;
        g.M = B; g.N = H;
        g.C = dhs; g.ldc = H; g.c_bf16 = false; g.accumulate = 1;
        g.splits = L.p_drec.splits; g.partial = partial;
        LS_TRY(launch_gemm(g, false, L.p_drec.big_tile, st));
      }
    }
    {  // dW_hh = sum_t da_t^T h_{t-1}
      GemmArgs g;
      g.seg(dGE, 4 * H, 0, hE, H, 0, TB);
      g.a_kc = false; g.b_kc = false;
      g.M = 4 * H; g.N = H;
      g.C = dW_hh[l]; g.ldc = H; g.c_bf16 = false;
      g.splits = L.p_dwh.splits; g.partial = partial;
      LS_TRY(launch_gemm(g, bf, L.p_dwh.big_tile, st));
    }
    {  // dW_ih = sum_t da_t^T x_t
      GemmArgs g;
      g.seg(dGE, 4 * H, 0, xin, Il, 0, TB);
      g.a_kc = false; g.b_kc = false;
      g.M = 4 * H; g.N = Il;
      g.C = dW_ih[l]; g.ldc = Il; g.c_bf16 = false;
      g.splits = L.p_dwi[l].splits; g.partial = partial;
      LS_TRY(launch_gemm(g, bf, L.p_dwi[l].big_tile, st));
    }
    {
      constexpr int per_block = 64 * (16 / (int)sizeof(TE));    // columns one block covers
      hipLaunchKernelGGL(lstm_bias_partial_kernel<TE>, dim3((4 * H + per_block - 1) / per_block, L.nrb), dim3(256), 0,
                         st, dGE, dGlo, TB, 4 * H, dbpart);
    }
    LS_TRY(hipGetLastError());
    LS_TRY(launch_db_reduce(dbpart, L.nrb, 4 * H, db[l], st));
    float* dinp = l == 0 ? dx : reinterpret_cast<float*>(w + L.dio[l & 1]);
    {  // gradient of the layer's input, all steps: da W_ih
      GemmArgs g;
      g.seg(dGE, 4 * H, 0, W_ih[l], Il, 0, 4 * H);   // (bf16: the gate gradients as rounded, like the recurrent product)
      g.a_kc = true; g.b_kc = false;
      g.M = TB; g.N = Il;
      g.C = dinp; g.ldc = Il; g.c_bf16 = false;
      g.splits = L.p_dx[l].splits; g.partial = partial;
      LS_TRY(launch_gemm(g, bf, L.p_dx[l].big_tile, st));
    }
    if (dh0) LS_TRY(hipMemcpyAsync(dh0 + (size_t)l * BH, dhs, (size_t)BH * 4, hipMemcpyDeviceToDevice, st));
    if (dc0) LS_TRY(hipMemcpyAsync(dc0 + (size_t)l * BH, dcs, (size_t)BH * 4, hipMemcpyDeviceToDevice, st));
    dout = dinp;
  }
  return AS_OK;
}
}  // namespace
}  // namespace asx

using namespace asx;

extern "C" {

size_t lstm_stack_workspace_bytes(const ls_shape* shape) {
  if (!ls_shape_ok(shape)) return 0;
  return make_ls_layout(shape).total;
}

as_status lstm_stack_fwd(const ls_shape* s, const void* x, const int32_t* lengths, const void* const* W_ih,
                         const void* const* W_hh, const void* const* b, const float* h0, const float* c0, void* y,
                         float* hT, float* cT, void* workspace, size_t workspace_bytes, void* hip_stream) {
  LsLayout L;
  as_status rc = check_ls(s, workspace, workspace_bytes, &L);
  if (rc != AS_OK) return rc;
  if (!x || !lengths || !y) return set_error(AS_ERR_NULL, "a required pointer is NULL");
  const void* ptrs[] = {x, lengths, y, h0, c0, hT, cT};
  for (const void* p : ptrs)
    if (p && !al16(p)) return set_error(AS_ERR_ALIGN, "pointer %p is not 16-byte aligned", p);
  if ((rc = check_ptr_array(W_ih, s->L, "W_ih")) != AS_OK) return rc;
  if ((rc = check_ptr_array(W_hh, s->L, "W_hh")) != AS_OK) return rc;
  if ((rc = check_ptr_array(b, s->L, "b")) != AS_OK) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  char* w = reinterpret_cast<char*>(workspace);
  if (s->dtype == AS_BF16)
    return ls_fwd<uint16_t>(s, L, reinterpret_cast<const char*>(x), lengths, W_ih, W_hh, b, h0, c0,
                            reinterpret_cast<char*>(y), hT, cT, w, st);
  return ls_fwd<float>(s, L, reinterpret_cast<const char*>(x), lengths, W_ih, W_hh, b, h0, c0,
                       reinterpret_cast<char*>(y), hT, cT, w, st);
}

as_status lstm_stack_bwd(const ls_shape* s, const void* x, const int32_t* lengths, const void* const* W_ih,
                         const void* const* W_hh, const float* dy, const float* dhT, const float* dcT,
                         void* workspace, size_t workspace_bytes, float* dx, float* const* dW_ih,
                         float* const* dW_hh, float* const* db, float* dh0, float* dc0, void* hip_stream) {
  LsLayout L;
  as_status rc = check_ls(s, workspace, workspace_bytes, &L);
  if (rc != AS_OK) return rc;
  if (!x || !lengths || !dy || !dx) return set_error(AS_ERR_NULL, "a required pointer is NULL");
  const void* ptrs[] = {x, lengths, dy, dhT, dcT, dx, dh0, dc0};
  for (const void* p : ptrs)
    if (p && !al16(p)) return set_error(AS_ERR_ALIGN, "pointer %p is not 16-byte aligned", p);
  if ((rc = check_ptr_array(W_ih, s->L, "W_ih")) != AS_OK) return rc;
  if ((rc = check_ptr_array(W_hh, s->L, "W_hh")) != AS_OK) return rc;
  if ((rc = check_ptr_array(reinterpret_cast<const void* const*>(dW_ih), s->L, "dW_ih")) != AS_OK) return rc;
  if ((rc = check_ptr_array(reinterpret_cast<const void* const*>(dW_hh), s->L, "dW_hh")) != AS_OK) return rc;
  if ((rc = check_ptr_array(reinterpret_cast<const void* const*>(db), s->L, "db")) != AS_OK) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  char* w = reinterpret_cast<char*>(workspace);
  if (s->dtype == AS_BF16)
    return ls_bwd<uint16_t>(s, L, reinterpret_cast<const char*>(x), lengths, W_ih, W_hh, dy, dhT, dcT, w, dx, dW_ih,
                            dW_hh, db, dh0, dc0, st);
  return ls_bwd<float>(s, L, reinterpret_cast<const char*>(x), lengths, W_ih, W_hh, dy, dhT, dcT, w, dx, dW_ih, dW_hh,
                       db, dh0, dc0, st);
}

}  // extern "C"
