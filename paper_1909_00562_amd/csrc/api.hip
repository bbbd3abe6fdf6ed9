// C ABI of the attention-softmax library: argument checks, workspace layout
// and the order in which the kernels of the forward / backward pass are
// enqueued.  No arithmetic of the method lives here.
#include "../../include/attn_softmax.h"

#include <hip/hip_runtime.h>
#include <cmath>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "gemm.h"
#include "kernels.h"
#include "status.h"

namespace {

using namespace asx;

thread_local char g_err[512] = "";

as_status fail(as_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
}  // namespace

namespace asx {
as_status set_error(as_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
}  // namespace asx

namespace {
using namespace asx;

// ---- profiling: HIP events around every launch ---------------------------------
struct Prof {
  bool on = false;
  uint64_t mask = ~0ull;   // stages that are timed while on (bit = as_stage)
  struct Rec {
    int stage;
    hipEvent_t a, b;
  };
  std::vector<Rec> pending;
  std::vector<hipEvent_t> pool;
  double ms[AS_STAGE_COUNT] = {0};
  int64_t launches[AS_STAGE_COUNT] = {0};
  hipEvent_t get() {
    if (!pool.empty()) {
      hipEvent_t e = pool.back();
      pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};
Prof g_prof;

struct StageTimer {
  hipStream_t st;
  Prof::Rec rec{0, nullptr, nullptr};
  bool live = false;
  StageTimer(int stage, hipStream_t s) : st(s) {
    if (!g_prof.on || !((g_prof.mask >> stage) & 1ull)) return;
    rec.stage = stage;
    rec.a = g_prof.get();
    rec.b = g_prof.get();
    if (!rec.a || !rec.b) return;
    live = hipEventRecord(rec.a, st) == hipSuccess;
  }
  ~StageTimer() {
    if (!live) return;
    if (hipEventRecord(rec.b, st) == hipSuccess) g_prof.pending.push_back(rec);
  }
};

// ---- workspace layout ------------------------------------------------------------
constexpr size_t kAlign = 256;
size_t up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
  int64_t N, ldS, ldV;
  size_t e;  // bytes per stored element
  size_t q, scores, alpha32, alphaE, ctx, hc, logits, lse, tokloss;
  size_t dz, dC, dalpha, dscoreE, dQ, dbpart, partial, total;
  // rounding remainders (value - stored(value)) of operands made inside the attention core,
  // and the tanh derivative 1 - h_c^2 taken before h_c is rounded
  size_t q_lo, alphaE_lo, dC_lo, dscoreE_lo, dact, dz_lo, ctx_lo;
  // row compaction (skip_pad_rows): position <-> compacted row, the count, and the gathered / to-be-scattered blocks
  bool compact;
  bool dhc_dyn;   // the product with W_out in the backward pass picks its reduction split on the device
  size_t row_pos, rows, n_act, hc_c, dact_c, dz_c, dz_lo_c;
  int rb, nrb;
  GemmPlan p_q, p_score, p_ctx, p_hc, p_logits, p_dwout, p_dhc, p_dwc, p_dch, p_dalpha, p_dq, p_ds, p_dwa, p_dh;
  size_t partial_bytes;
};

bool shape_ok(const as_shape* s) {
  if (!s) return false;
  if (s->T < 1 || s->S < 1 || s->B < 1 || s->H < 1 || s->V < 1) return false;
  if (s->pad_id < 0 || s->pad_id >= s->V) return false;
  if (!(s->dropout_p >= 0.f && s->dropout_p < 1.f)) return false;
  if (s->skip_pad_rows != 0 && s->skip_pad_rows != 1) return false;
  if (s->dtype != AS_F32 && s->dtype != AS_BF16) return false;
  const int64_t N = (int64_t)s->T * s->B;
  if (N > (1 << 30) || (int64_t)s->S * s->B > (1 << 30)) return false;
  if ((int64_t)s->H > (1 << 20) || (int64_t)s->V > (1 << 28)) return false;
  return true;
}

Layout make_layout(const as_shape* s) {
  Layout L;
  const bool bf = s->dtype == AS_BF16;
  const int T = s->T, S = s->S, B = s->B, H = s->H, V = s->V;
  L.N = (int64_t)T * B;
  const int N = (int)L.N;
  L.e = bf ? 2 : 4;
  L.ldS = up(S, 8);
  L.ldV = up(V, 8);
  L.rb = xent_rows_per_block(N, V, bf);
  L.nrb = (N + L.rb - 1) / L.rb;

  L.p_q = gemm_plan(N, H, H, 1, bf, false);
  L.p_score = gemm_plan(T, S, H, B, bf, false);
  L.p_ctx = gemm_plan(T, H, S, B, bf, false);
  L.p_hc = gemm_plan(N, H, bf ? 3 * H : 2 * H, 1, bf, true, true);   // segments: ctx (+ remainder), h_dec
  L.p_logits = gemm_plan(N, V, H, 1, bf, false);
  L.p_dwout = gemm_plan(V, H, N, 1, bf, true);
  L.p_dhc = gemm_plan(N, H, V, 1, bf, true);
  // Few, long work items (N/256 x H/256 tiles, reduction over V): once the padding rows are gone the item count
  // no longer fills whole rounds of the grid, so the kernel splits the reduction to fit the count it reads.
  L.dhc_dyn = s->skip_pad_rows != 0 && bf && L.p_dhc.big_tile;
  if (L.dhc_dyn && L.p_dhc.splits < 8) L.p_dhc.splits = 8;
  L.p_dwc = gemm_plan(H, H, N, 2, bf, true);          // both halves of dW_c in one launch
  L.p_dch = gemm_plan(N, H, H, 1, bf, false);
  L.p_dalpha = gemm_plan(T, S, H, B, bf, false);
  L.p_dq = gemm_plan(T, H, S, B, bf, false);
  L.p_ds = gemm_plan(S, H, T, B, bf, false);
  L.p_dwa = gemm_plan(H, H, N, 1, bf, true);
  L.p_dh = gemm_plan(N, H, H, 1, bf, false);
  size_t pb = 0;
  auto mx = [&](size_t v) { if (v > pb) pb = v; };
  mx(gemm_partial_bytes(N, H, 1, L.p_hc.splits));
  mx(gemm_partial_bytes(V, H, 1, L.p_dwout.splits));
  mx(gemm_partial_bytes(N, H, 1, L.p_dhc.splits));
  mx(gemm_partial_bytes(H, H, 2, L.p_dwc.splits));
  mx(gemm_partial_bytes(H, H, 1, L.p_dwa.splits));
  L.partial_bytes = pb;

  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += up(bytes, kAlign);
    return o;
  };
  const size_t NH = (size_t)N * H;
  const size_t BTS = (size_t)B * T * S, BTSl = (size_t)B * T * L.ldS;
  L.q = take(NH * L.e);
  L.scores = take(BTS * 4);
  L.alpha32 = take(BTS * 4);
  L.alphaE = take(BTSl * L.e);
  L.ctx = take(NH * L.e);
  L.hc = take(NH * L.e);
  L.logits = take((size_t)N * L.ldV * L.e);
  L.lse = take((size_t)N * 4);
  L.tokloss = take((size_t)N * 4);
  L.dz = take(NH * L.e);
  L.dC = take(NH * L.e);
  L.dalpha = take(BTS * 4);
  L.dscoreE = take(BTSl * L.e);
  L.dQ = take(NH * L.e);
  L.dbpart = take((size_t)L.nrb * V * 4);
  L.partial = take(pb);
  L.q_lo = take(NH * L.e);
  L.alphaE_lo = take(BTSl * L.e);
  L.dC_lo = take(NH * L.e);
  L.dscoreE_lo = take(BTSl * L.e);
  L.dact = take(NH * 4);
  L.ctx_lo = take(NH * L.e);
  L.dz_lo = take(NH * L.e);
  L.compact = s->skip_pad_rows != 0;
  L.row_pos = L.rows = L.n_act = L.hc_c = L.dact_c = L.dz_c = L.dz_lo_c = 0;
  if (L.compact) {
    L.row_pos = take((size_t)N * 4);
    L.rows = take((size_t)N * 4);
    L.n_act = take(16);
    L.hc_c = take(NH * L.e);
    L.dact_c = take(NH * 4);
    L.dz_c = take(NH * L.e);
    L.dz_lo_c = take(NH * L.e);
  }
  L.total = off;
  return L;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

as_status check_common(const as_shape* s, const void* h_dec, const void* h_enc, const int32_t* src_len,
                       const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                       const int32_t* targets, void* ws, size_t ws_bytes, Layout* L) {
  if (!s) return fail(AS_ERR_NULL, "shape is NULL");
  if (s->dtype != AS_F32 && s->dtype != AS_BF16) return fail(AS_ERR_DTYPE, "unknown dtype %d", s->dtype);
  if (!shape_ok(s))
    return fail(AS_ERR_SHAPE, "bad shape T=%d S=%d B=%d H=%d V=%d pad_id=%d dropout_p=%g skip_pad_rows=%d", s->T, s->S,
                s->B, s->H, s->V, s->pad_id, (double)s->dropout_p, s->skip_pad_rows);
  if (!h_dec || !h_enc || !src_len || !W_a || !W_c || !W_out || !b_out || !targets || !ws)
    return fail(AS_ERR_NULL, "a required pointer is NULL");
  if (s->dtype == AS_BF16 && (s->H % 8) != 0) return fail(AS_ERR_ALIGN, "AS_BF16 needs H %% 8 == 0 (H=%d)", s->H);
  const void* ptrs[] = {h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, ws};
  for (const void* p : ptrs)
    if (!aligned16(p)) return fail(AS_ERR_ALIGN, "pointer %p is not 16-byte aligned", p);
  *L = make_layout(s);
  if (ws_bytes < L->total)
    return fail(AS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, L->total);
  return AS_OK;
}

#define AS_TRY(stage, expr)                                                              \
  do {                                                                                   \
    hipError_t e_;                                                                       \
    {                                                                                    \
      StageTimer timer_(stage, st);                                                      \
      e_ = (expr);                                                                       \
    }                                                                                    \
    if (e_ != hipSuccess) return fail(AS_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

}  // namespace

// ---- library-owned scratch (attn_softmax_fwd_static) --------------------------------
// The workspace of callers that cannot allocate: one array in the code object, so every GPU the library runs on
// holds its own copy from module load until the process ends.  Host code never uses the array's name as an
// address: the device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// device address of `scratch` on the calling thread's current device
as_status static_scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(AS_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(AS_ERR_HIP, "device %d is outside the %d the library keeps scratch for", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail(AS_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255)) return fail(AS_ERR_HIP, "static scratch resolved to %p", p);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return AS_OK;
}
}  // namespace

// Eq. 4-6 from the context vectors on: shared by the batched forward pass and the per-step one.
static as_status fwd_from_ctx(const as_shape* s, const Layout& L, char* w, const char* hd, const char* wc,
                              const void* W_out, const void* b_out, const int32_t* targets, float* loss_sum,
                              int32_t* n_tok, float* tok_loss, int32_t* argmax, uint8_t* tgt_mask, hipStream_t st) {
  const bool bf = s->dtype == AS_BF16;
  const int H = s->H, V = s->V, N = (int)L.N;
  {  // h_c = tanh(W_c[:, :H] ctx + W_c[:, H:] h_dec)                       (Eq. 4)
    GemmArgs g;
    g.seg(w + L.ctx, H, 0, wc, 2 * H, 0, H);
    g.seg(w + L.ctx_lo, H, 0, wc, 2 * H, 0, H);
    g.seg(hd, H, 0, wc + (size_t)H * L.e, 2 * H, 0, H);
    g.a_kc = true; g.b_kc = true;
    g.M = N; g.N = H; g.act_tanh = 1;
    g.C = w + L.hc; g.ldc = H; g.c_bf16 = bf;
    g.C_dact = reinterpret_cast<float*>(w + L.dact);
    g.splits = L.p_hc.splits; g.partial = reinterpret_cast<float*>(w + L.partial);
    if (s->dropout_p > 0.f) {   // section 4.2: dropout, here on the attentional state; the mask rides on dact into bwd
      g.drop_thr = (uint32_t)((double)s->dropout_p * 4294967296.0);   // floor: the product is exact in double
      g.drop_scale = 1.f / (1.f - s->dropout_p);
      g.drop_seed = s->dropout_seed;
    }
    AS_TRY(AS_STAGE_GEMM_HC, launch_gemm(g, bf, L.p_hc.big_tile, st));
  }
  // Padding rows drop out of Eq. 5-6 here: the rows of h_c (and of its saved derivative) whose target is a
  // word are gathered into a dense block, and everything over the vocabulary runs on that block alone.
  const int32_t* rows = nullptr;
  const int32_t* n_act = nullptr;
  if (L.compact) {
    rows = reinterpret_cast<const int32_t*>(w + L.rows);
    n_act = reinterpret_cast<const int32_t*>(w + L.n_act);
    AS_TRY(AS_STAGE_COMPACT, launch_row_compact(targets, N, V, s->pad_id, reinterpret_cast<int32_t*>(w + L.row_pos),
                                                reinterpret_cast<int32_t*>(w + L.rows),
                                                reinterpret_cast<int32_t*>(w + L.n_act), tgt_mask, tok_loss, argmax, st));
    AS_TRY(AS_STAGE_COMPACT, launch_gather_rows(rows, n_act, N, w + L.hc, w + L.hc_c, (int64_t)H * L.e, w + L.dact,
                                                w + L.dact_c, (int64_t)H * 4, st));
  }
  {  // logits = h_c W_out^T + b_out                                        (Eq. 5)
    GemmArgs g;
    g.seg(L.compact ? w + L.hc_c : w + L.hc, H, 0, W_out, H, 0, H);
    g.a_kc = true; g.b_kc = true;
    g.M = N; g.N = V; g.bias = b_out;
    g.M_dev = n_act;
    g.C = w + L.logits; g.ldc = L.ldV; g.c_bf16 = bf;
    AS_TRY(AS_STAGE_GEMM_LOGITS, launch_gemm(g, bf, L.p_logits.big_tile, st));
  }
  AS_TRY(AS_STAGE_XENT_STATS,                                          // Eq. 5-6
         launch_xent_stats(w + L.logits, L.ldV, bf, N, V, targets, s->pad_id, reinterpret_cast<float*>(w + L.lse),
                           reinterpret_cast<float*>(w + L.tokloss), tok_loss, argmax, L.compact ? nullptr : tgt_mask,
                           rows, n_act, st));
  AS_TRY(AS_STAGE_MISC, launch_loss_reduce(reinterpret_cast<const float*>(w + L.tokloss), targets, N, V, s->pad_id,
                                           loss_sum, n_tok, n_act, st));
  return AS_OK;
}

// the forward pass proper, on whatever workspace the entry point hands it
static as_status fwd_impl(const as_shape* s, const void* h_dec, const void* h_enc, const int32_t* src_len,
                          const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                          const int32_t* targets, float* loss_sum, int32_t* n_tok, float* tok_loss,
                          int32_t* argmax, uint8_t* attn_mask, uint8_t* tgt_mask, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

extern "C" {

size_t attn_softmax_workspace_bytes(const as_shape* shape) {
  if (!shape_ok(shape)) return 0;
  if (shape->dtype == AS_BF16 && (shape->H % 8) != 0) return 0;
  return make_layout(shape).total;
}

const char* attn_softmax_last_error(void) { return g_err; }

as_status attn_softmax_view(const as_shape* shape, void* workspace, int which, void** ptr, size_t* bytes,
                            int64_t* row_stride) {
  if (!shape || !workspace || !ptr || !bytes) return fail(AS_ERR_NULL, "a required pointer is NULL");
  if (shape->dtype != AS_F32 && shape->dtype != AS_BF16) return fail(AS_ERR_DTYPE, "unknown dtype %d", shape->dtype);
  if (!shape_ok(shape)) return fail(AS_ERR_SHAPE, "bad shape");
  if (shape->dtype == AS_BF16 && (shape->H % 8) != 0) return fail(AS_ERR_ALIGN, "AS_BF16 needs H %% 8 == 0");
  const Layout L = make_layout(shape);
  char* w = reinterpret_cast<char*>(workspace);
  const size_t NH = (size_t)L.N * shape->H;
  int64_t ld = 0;
  switch (which) {
    case AS_VIEW_ALPHA: *ptr = w + L.alpha32; *bytes = (size_t)shape->B * shape->T * shape->S * 4; ld = shape->S; break;
    case AS_VIEW_CTX: *ptr = w + L.ctx; *bytes = NH * L.e; ld = shape->H; break;
    case AS_VIEW_HC: *ptr = w + L.hc; *bytes = NH * L.e; ld = shape->H; break;
    case AS_VIEW_LOGITS: *ptr = w + L.logits; *bytes = (size_t)L.N * L.ldV * L.e; ld = L.ldV; break;
    case AS_VIEW_LSE: *ptr = w + L.lse; *bytes = (size_t)L.N * 4; ld = shape->B; break;
    case AS_VIEW_ROW_POS:
      if (!L.compact) return fail(AS_ERR_SHAPE, "AS_VIEW_ROW_POS exists only with skip_pad_rows = 1");
      *ptr = w + L.row_pos; *bytes = (size_t)L.N * 4; ld = shape->B; break;
    default: return fail(AS_ERR_SHAPE, "unknown view %d", which);
  }
  if (row_stride) *row_stride = ld;
  return AS_OK;
}

as_status attn_softmax_fwd(const as_shape* s, const void* h_dec, const void* h_enc, const int32_t* src_len,
                           const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                           const int32_t* targets, float* loss_sum, int32_t* n_tok, float* tok_loss,
                           int32_t* argmax, uint8_t* attn_mask, uint8_t* tgt_mask, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  return fwd_impl(s, h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, loss_sum, n_tok, tok_loss, argmax,
                  attn_mask, tgt_mask, workspace, workspace_bytes, hip_stream);
}

as_status attn_softmax_fwd_static(const as_shape* s, const void* h_dec, const void* h_enc, const int32_t* src_len,
                                  const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                                  const int32_t* targets, float* loss_sum, int32_t* n_tok, float* tok_loss,
                                  int32_t* argmax, uint8_t* attn_mask, uint8_t* tgt_mask, void* hip_stream) {
  // everything checkable on the host first, with a stand-in workspace address that is never dereferenced
  Layout L;
  as_status rc = check_common(s, h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets,
                              reinterpret_cast<void*>(uintptr_t(256)), ~size_t(0), &L);
  if (rc != AS_OK) return rc;
  if (!loss_sum || !n_tok) return fail(AS_ERR_NULL, "loss_sum / n_tok is NULL");
  if (L.total > kStaticScratchBytes)
    return fail(AS_ERR_WORKSPACE, "this shape needs %zu bytes of workspace, the library's static scratch holds %zu: "
                "use attn_softmax_fwd with a caller-owned workspace", L.total, kStaticScratchBytes);
  void* ws = nullptr;
  rc = static_scratch_ptr(&ws);
  if (rc != AS_OK) return rc;
  return fwd_impl(s, h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, loss_sum, n_tok, tok_loss, argmax,
                  attn_mask, tgt_mask, ws, kStaticScratchBytes, hip_stream);
}

}  // extern "C"

static as_status fwd_impl(const as_shape* s, const void* h_dec, const void* h_enc, const int32_t* src_len,
                          const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                          const int32_t* targets, float* loss_sum, int32_t* n_tok, float* tok_loss,
                          int32_t* argmax, uint8_t* attn_mask, uint8_t* tgt_mask, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  Layout L;
  as_status rc = check_common(s, h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, workspace,
                              workspace_bytes, &L);
  if (rc != AS_OK) return rc;
  if (!loss_sum || !n_tok) return fail(AS_ERR_NULL, "loss_sum / n_tok is NULL");
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const bool bf = s->dtype == AS_BF16;
  const int T = s->T, S = s->S, B = s->B, H = s->H, V = s->V, N = (int)L.N;
  char* w = reinterpret_cast<char*>(workspace);
  const char* hd = reinterpret_cast<const char*>(h_dec);
  const char* he = reinterpret_cast<const char*>(h_enc);
  const char* wc = reinterpret_cast<const char*>(W_c);
  const int64_t BH = (int64_t)B * H;

  {  // Q = h_dec W_a                                                    (Eq. 2)
    GemmArgs g;
    g.seg(hd, H, 0, W_a, H, 0, H);
    g.a_kc = true; g.b_kc = false;
    g.M = N; g.N = H;
    g.C = w + L.q; g.ldc = H; g.c_bf16 = bf;
    g.C_lo = w + L.q_lo;
    AS_TRY(AS_STAGE_GEMM_Q, launch_gemm(g, bf, L.p_q.big_tile, st));
  }
  if (bf && attn_fwd_fused_supported(S, H)) {
    // Eq. 2 (second half), 1 and 3 in one kernel per (sentence, 32 decoder steps): the scores stay on chip
    AS_TRY(AS_STAGE_ATTN_SCORE,
           launch_attn_fwd_fused(w + L.q, w + L.q_lo, he, src_len, B, T, S, H, reinterpret_cast<float*>(w + L.alpha32),
                                 w + L.alphaE, w + L.alphaE_lo, L.ldS, w + L.ctx, w + L.ctx_lo, attn_mask, st));
  } else {
    {  // score[b] = Q_b h_enc_b^T, one product per sentence                  (Eq. 2)
      GemmArgs g;
      g.seg(w + L.q, BH, H, he, BH, H, H);
      g.seg(w + L.q_lo, BH, H, he, BH, H, H);
      g.a_kc = true; g.b_kc = true;
      g.M = T; g.N = S; g.batch = B;
      g.C = w + L.scores; g.ldc = S; g.sC = (int64_t)T * S; g.c_bf16 = false;
      AS_TRY(AS_STAGE_ATTN_SCORE, launch_gemm(g, bf, L.p_score.big_tile, st));
    }
    AS_TRY(AS_STAGE_ATTN_SOFTMAX,                                        // Eq. 1
           launch_attn_softmax_rows(reinterpret_cast<const float*>(w + L.scores), src_len, B, T, S,
                                    reinterpret_cast<float*>(w + L.alpha32), w + L.alphaE,
                                    w + L.alphaE_lo, L.ldS, bf, attn_mask, st));
    {  // ctx_b = alpha_b h_enc_b                                            (Eq. 3)
      GemmArgs g;
      g.seg(w + L.alphaE, L.ldS, (int64_t)T * L.ldS, he, BH, H, S);
      g.seg(w + L.alphaE_lo, L.ldS, (int64_t)T * L.ldS, he, BH, H, S);
      g.a_kc = true; g.b_kc = false;
      g.M = T; g.N = H; g.batch = B;
      g.C = w + L.ctx; g.ldc = BH; g.sC = H; g.c_bf16 = bf;
      g.C_lo = w + L.ctx_lo;
      AS_TRY(AS_STAGE_ATTN_CTX, launch_gemm(g, bf, L.p_ctx.big_tile, st));
    }
  }
  return fwd_from_ctx(s, L, w, hd, wc, W_out, b_out, targets, loss_sum, n_tok, tok_loss, argmax, tgt_mask, st);
}

extern "C" {

as_status attn_softmax_bwd(const as_shape* s, const void* h_dec, const void* h_enc, const int32_t* src_len,
                           const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                           const int32_t* targets, void* workspace, size_t workspace_bytes, float* d_h_dec,
                           float* d_h_enc, float* dW_a, float* dW_c, float* dW_out, float* db_out,
                           void* hip_stream) {
  Layout L;
  as_status rc = check_common(s, h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, workspace,
                              workspace_bytes, &L);
  if (rc != AS_OK) return rc;
  if (!d_h_dec || !d_h_enc || !dW_a || !dW_c || !dW_out || !db_out)
    return fail(AS_ERR_NULL, "a gradient output pointer is NULL");
  const void* outs[] = {d_h_dec, d_h_enc, dW_a, dW_c, dW_out, db_out};
  for (const void* p : outs)
    if (!aligned16(p)) return fail(AS_ERR_ALIGN, "pointer %p is not 16-byte aligned", p);
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const bool bf = s->dtype == AS_BF16;
  const int T = s->T, S = s->S, B = s->B, H = s->H, V = s->V, N = (int)L.N;
  char* w = reinterpret_cast<char*>(workspace);
  const char* hd = reinterpret_cast<const char*>(h_dec);
  const char* he = reinterpret_cast<const char*>(h_enc);
  const char* wc = reinterpret_cast<const char*>(W_c);
  const int64_t BH = (int64_t)B * H;
  float* partial = reinterpret_cast<float*>(w + L.partial);

  // dlogits = g (softmax - onehot) in place; db_out = column sums
  const int32_t* rows = L.compact ? reinterpret_cast<const int32_t*>(w + L.rows) : nullptr;
  const int32_t* n_act = L.compact ? reinterpret_cast<const int32_t*>(w + L.n_act) : nullptr;
  AS_TRY(AS_STAGE_XENT_DLOGITS,
         launch_xent_dlogits(w + L.logits, L.ldV, bf, N, V, targets, s->pad_id,
                             reinterpret_cast<const float*>(w + L.lse), s->grad_scale,
                             reinterpret_cast<float*>(w + L.dbpart), rows, n_act, st));
  AS_TRY(AS_STAGE_MISC, launch_db_reduce(reinterpret_cast<const float*>(w + L.dbpart), L.nrb, V, db_out, st));
  {  // dW_out = dlogits^T h_c
    GemmArgs g;
    g.seg(w + L.logits, L.ldV, 0, L.compact ? w + L.hc_c : w + L.hc, H, 0, N);
    g.a_kc = false; g.b_kc = false;
    g.M = V; g.N = H;
    g.K_dev = n_act;     // compacted: the reduction runs over the non-pad rows only
    g.C = dW_out; g.ldc = H; g.c_bf16 = false;
    g.splits = L.p_dwout.splits; g.partial = partial;
    AS_TRY(AS_STAGE_GEMM_DWOUT, launch_gemm(g, bf, L.p_dwout.big_tile, st));
  }
  {  // dz = (dlogits W_out) * (1 - h_c^2), the factor saved by the forward pass
    GemmArgs g;
    g.seg(w + L.logits, L.ldV, 0, W_out, H, 0, V);
    g.a_kc = true; g.b_kc = false;
    g.M = N; g.N = H;
    g.gate = reinterpret_cast<const float*>(w + (L.compact ? L.dact_c : L.dact)); g.ldg = H;
    g.C = w + (L.compact ? L.dz_c : L.dz); g.ldc = H; g.c_bf16 = bf;
    g.C_lo = w + (L.compact ? L.dz_lo_c : L.dz_lo);
    g.M_dev = n_act;
    g.dyn_split = L.dhc_dyn;
    g.splits = L.p_dhc.splits; g.partial = partial;
    AS_TRY(AS_STAGE_GEMM_DHC, launch_gemm(g, bf, L.p_dhc.big_tile, st));
  }
  if (L.compact)   // dz back to its time-major rows, zeros at the padding rows: the rest of the pass is per sentence
    AS_TRY(AS_STAGE_COMPACT, launch_scatter_rows(reinterpret_cast<const int32_t*>(w + L.row_pos), N, w + L.dz_c,
                                                 w + L.dz, w + L.dz_lo_c, w + L.dz_lo, (int64_t)H * L.e, st));
  {  // dW_c = dz^T [ctx ; h_dec]: the two halves as one launch of two products that share dz; the second operand
     // of half 1 is the caller's h_dec, reached from ctx through a "batch stride" that is just the distance
     // between the two buffers (both 16-byte aligned, so it is a whole number of 8-element vectors)
    GemmArgs g;
    const int64_t h_dec_from_ctx = (hd - (w + L.ctx)) / (int64_t)L.e;
    g.seg(w + L.dz, H, 0, w + L.ctx, H, h_dec_from_ctx, N);
    g.a_kc = false; g.b_kc = false;
    g.M = H; g.N = H; g.batch = 2;
    g.C = dW_c; g.ldc = 2 * H; g.sC = H; g.c_bf16 = false;
    g.splits = L.p_dwc.splits; g.partial = partial;
    AS_TRY(AS_STAGE_GEMM_DWC, launch_gemm(g, bf, L.p_dwc.big_tile, st));
  }
  {  // dC = dz W_c[:, :H]
    GemmArgs g;
    g.seg(w + L.dz, H, 0, wc, 2 * H, 0, H);
    g.seg(w + L.dz_lo, H, 0, wc, 2 * H, 0, H);
    g.a_kc = true; g.b_kc = false;
    g.M = N; g.N = H;
    g.C = w + L.dC; g.ldc = H; g.c_bf16 = bf;
    g.C_lo = w + L.dC_lo;
    AS_TRY(AS_STAGE_GEMM_DCH, launch_gemm(g, bf, L.p_dch.big_tile, st));
  }
  {  // dH1 = dz W_c[:, H:]  -> d_h_dec
    GemmArgs g;
    g.seg(w + L.dz, H, 0, wc + (size_t)H * L.e, 2 * H, 0, H);
    g.a_kc = true; g.b_kc = false;
    g.M = N; g.N = H;
    g.C = d_h_dec; g.ldc = H; g.c_bf16 = false;
    AS_TRY(AS_STAGE_GEMM_DCH, launch_gemm(g, bf, L.p_dch.big_tile, st));
  }
  if (bf && attn_fwd_fused_supported(S, H)) {
    // dalpha, the softmax Jacobian and dQ in one kernel per (sentence, 32 decoder steps): dalpha stays on chip
    AS_TRY(AS_STAGE_ATTN_BWD,
           launch_attn_bwd_fused(w + L.dC, w + L.dC_lo, he, src_len, B, T, S, H,
                                 reinterpret_cast<const float*>(w + L.alpha32), w + L.dscoreE, w + L.dscoreE_lo, L.ldS,
                                 w + L.dQ, st));
  } else {
    {  // dalpha_b = dC_b h_enc_b^T
      GemmArgs g;
      g.seg(w + L.dC, BH, H, he, BH, H, H);
      g.seg(w + L.dC_lo, BH, H, he, BH, H, H);
      g.a_kc = true; g.b_kc = true;
      g.M = T; g.N = S; g.batch = B;
      g.C = w + L.dalpha; g.ldc = S; g.sC = (int64_t)T * S; g.c_bf16 = false;
      AS_TRY(AS_STAGE_ATTN_BWD, launch_gemm(g, bf, L.p_dalpha.big_tile, st));
    }
    AS_TRY(AS_STAGE_ATTN_SOFTMAX_BWD,
           launch_attn_softmax_rows_bwd(reinterpret_cast<const float*>(w + L.alpha32),
                                        reinterpret_cast<const float*>(w + L.dalpha), B, T, S, w + L.dscoreE,
                                        w + L.dscoreE_lo, L.ldS, bf, st));
    {  // dQ_b = dscore_b h_enc_b
      GemmArgs g;
      g.seg(w + L.dscoreE, L.ldS, (int64_t)T * L.ldS, he, BH, H, S);
      g.seg(w + L.dscoreE_lo, L.ldS, (int64_t)T * L.ldS, he, BH, H, S);
      g.a_kc = true; g.b_kc = false;
      g.M = T; g.N = H; g.batch = B;
      g.C = w + L.dQ; g.ldc = BH; g.sC = H; g.c_bf16 = bf;
      AS_TRY(AS_STAGE_ATTN_BWD, launch_gemm(g, bf, L.p_dq.big_tile, st));
    }
  }
  {  // d_h_enc_b = alpha_b^T dC_b + dscore_b^T Q_b  (rows s >= src_len[b]: alpha = dscore = 0)
    GemmArgs g;
    const int64_t sAl = (int64_t)T * L.ldS;
    g.seg(w + L.alphaE, L.ldS, sAl, w + L.dC, BH, H, T);
    g.seg(w + L.dscoreE, L.ldS, sAl, w + L.q, BH, H, T);
    // first-order remainder terms of the two products
    g.seg(w + L.alphaE_lo, L.ldS, sAl, w + L.dC, BH, H, T);
    g.seg(w + L.alphaE, L.ldS, sAl, w + L.dC_lo, BH, H, T);
    g.seg(w + L.dscoreE_lo, L.ldS, sAl, w + L.q, BH, H, T);
    g.seg(w + L.dscoreE, L.ldS, sAl, w + L.q_lo, BH, H, T);
    g.a_kc = false; g.b_kc = false;
    g.M = S; g.N = H; g.batch = B;
    g.C = d_h_enc; g.ldc = BH; g.sC = H; g.c_bf16 = false;
    AS_TRY(AS_STAGE_ATTN_BWD, launch_gemm(g, bf, L.p_ds.big_tile, st));
  }
  {  // dW_a = h_dec^T dQ
    GemmArgs g;
    g.seg(hd, H, 0, w + L.dQ, H, 0, N);
    g.a_kc = false; g.b_kc = false;
    g.M = H; g.N = H;
    g.C = dW_a; g.ldc = H; g.c_bf16 = false;
    g.splits = L.p_dwa.splits; g.partial = partial;
    AS_TRY(AS_STAGE_GEMM_DWA, launch_gemm(g, bf, L.p_dwa.big_tile, st));
  }
  {  // d_h_dec += dQ W_a^T
    GemmArgs g;
    g.seg(w + L.dQ, H, 0, W_a, H, 0, H);
    g.a_kc = true; g.b_kc = true;
    g.M = N; g.N = H;
    g.C = d_h_dec; g.ldc = H; g.c_bf16 = false; g.accumulate = 1;
    AS_TRY(AS_STAGE_GEMM_DH, launch_gemm(g, bf, L.p_dh.big_tile, st));
  }
  return AS_OK;
}

// ---- per-step mode (T = 1) ---------------------------------------------------------
namespace {
struct StepLayout {
  Layout L;          // the batched layout for T = 1 (views work unchanged)
  size_t kprime;     // float [S,B,H]: W_a h_enc
  size_t total;
  GemmPlan p_kp;
};
StepLayout make_step_layout(const as_shape* s) {
  as_shape s1 = *s;
  s1.T = 1;
  StepLayout sl;
  sl.L = make_layout(&s1);
  sl.kprime = sl.L.total;
  sl.total = sl.kprime + up((size_t)s->S * s->B * s->H * sizeof(float), kAlign);
  sl.p_kp = gemm_plan(s->S * s->B, s->H, s->H, 1, s->dtype == AS_BF16, false);
  return sl;
}
bool step_shape_ok(const as_shape* s, as_shape* s1) {
  if (!s) return false;
  *s1 = *s;
  s1->T = 1;
  s1->skip_pad_rows = 0;   // a step is also asked for predictions at padding targets: every row is computed
  return shape_ok(s1) && !(s->dtype == AS_BF16 && (s->H % 8) != 0);
}
}  // namespace

size_t attn_softmax_step_workspace_bytes(const as_shape* shape) {
  as_shape s1;
  if (!step_shape_ok(shape, &s1)) return 0;
  return make_step_layout(&s1).total;
}

as_status attn_softmax_step_prepare(const as_shape* shape, const void* h_enc, const void* W_a, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
  as_shape s1;
  if (!shape) return fail(AS_ERR_NULL, "shape is NULL");
  if (shape->dtype != AS_F32 && shape->dtype != AS_BF16) return fail(AS_ERR_DTYPE, "unknown dtype %d", shape->dtype);
  if (!step_shape_ok(shape, &s1)) return fail(AS_ERR_SHAPE, "bad shape for the per-step mode");
  if (!h_enc || !W_a || !workspace) return fail(AS_ERR_NULL, "a required pointer is NULL");
  if (!aligned16(h_enc) || !aligned16(W_a) || !aligned16(workspace)) return fail(AS_ERR_ALIGN, "pointer not 16-byte aligned");
  const StepLayout sl = make_step_layout(&s1);
  if (workspace_bytes < sl.total)
    return fail(AS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, sl.total);
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const bool bf = s1.dtype == AS_BF16;
  const int H = s1.H;
  char* w = reinterpret_cast<char*>(workspace);
  GemmArgs g;   // K'[(s,b), i] = sum_j h_enc[(s,b), j] W_a[i, j]: the encoder-side half of Eq. 2
  g.seg(h_enc, H, 0, W_a, H, 0, H);
  g.a_kc = true; g.b_kc = true;
  g.M = s1.S * s1.B; g.N = H;
  g.C = w + sl.kprime; g.ldc = H; g.c_bf16 = false;
  AS_TRY(AS_STAGE_GEMM_Q, launch_gemm(g, bf, sl.p_kp.big_tile, st));
  return AS_OK;
}

as_status attn_softmax_step_fwd(const as_shape* shape, const void* h_t, const void* h_enc, const int32_t* src_len,
                                const void* W_c, const void* W_out, const void* b_out, const int32_t* targets,
                                float* loss_sum, int32_t* n_tok, float* tok_loss, int32_t* argmax,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  as_shape s1;
  if (!shape) return fail(AS_ERR_NULL, "shape is NULL");
  if (shape->dtype != AS_F32 && shape->dtype != AS_BF16) return fail(AS_ERR_DTYPE, "unknown dtype %d", shape->dtype);
  if (!step_shape_ok(shape, &s1)) return fail(AS_ERR_SHAPE, "bad shape for the per-step mode");
  if (!h_t || !h_enc || !src_len || !W_c || !W_out || !b_out || !targets || !workspace || !loss_sum || !n_tok)
    return fail(AS_ERR_NULL, "a required pointer is NULL");
  const void* ptrs[] = {h_t, h_enc, src_len, W_c, W_out, b_out, targets, workspace};
  for (const void* p : ptrs)
    if (!aligned16(p)) return fail(AS_ERR_ALIGN, "pointer %p is not 16-byte aligned", p);
  const StepLayout sl = make_step_layout(&s1);
  if (workspace_bytes < sl.total)
    return fail(AS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, sl.total);
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const bool bf = s1.dtype == AS_BF16;
  const Layout& L = sl.L;
  char* w = reinterpret_cast<char*>(workspace);
  AS_TRY(AS_STAGE_ATTN_SCORE,                                           // Eq. 1-3 for one step, fused
         launch_attn_step(h_t, reinterpret_cast<const float*>(w + sl.kprime), h_enc, src_len, s1.B, s1.S, s1.H,
                          reinterpret_cast<float*>(w + L.alpha32), w + L.ctx, w + L.ctx_lo, bf, nullptr, st));
  return fwd_from_ctx(&s1, L, w, reinterpret_cast<const char*>(h_t), reinterpret_cast<const char*>(W_c), W_out, b_out,
                      targets, loss_sum, n_tok, tok_loss, argmax, nullptr, st);
}

as_status attn_softmax_adam_step(const as_adam* hp, size_t n, const float* grad, float* master, float* m, float* v,
                                 void* weights_out, int32_t dtype, void* hip_stream) {
  if (!hp || !grad || !master || !m || !v) return fail(AS_ERR_NULL, "a required pointer is NULL");
  if (n == 0 || hp->step < 1 || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f))
    return fail(AS_ERR_SHAPE, "bad Adam arguments n=%zu step=%d beta1=%g beta2=%g", n, hp->step, (double)hp->beta1,
                (double)hp->beta2);
  if (weights_out && dtype != AS_F32 && dtype != AS_BF16) return fail(AS_ERR_DTYPE, "unknown dtype %d", dtype);
  const void* ptrs[] = {grad, master, m, v, weights_out};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return fail(AS_ERR_ALIGN, "pointer %p is not 16-byte aligned", p);
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  // bias corrections in double on the host: 1 - beta^step loses nothing for small steps that way
  const float inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)hp->beta1, (double)hp->step)));
  const float inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)hp->beta2, (double)hp->step)));
  AS_TRY(AS_STAGE_ADAM, launch_adam_step(n, grad, master, m, v, weights_out, dtype == AS_BF16, hp->lr, hp->beta1,
                                         hp->beta2, hp->eps, inv_bc1, inv_bc2, st));
  return AS_OK;
}

as_status attn_softmax_stream_probe(int kind, void* buf, void* buf2, int32_t rows, size_t row_bytes, void* hip_stream) {
  if (!buf || ((kind == 0 || kind == 1) && !buf2)) return fail(AS_ERR_NULL, "a required pointer is NULL");
  if (kind < 0 || kind > 2 || rows < 1 || row_bytes < 16 || (row_bytes & 15) || row_bytes > ((size_t)1 << 31))
    return fail(AS_ERR_SHAPE, "bad stream probe arguments kind=%d rows=%d row_bytes=%zu", kind, rows, row_bytes);
  if (!aligned16(buf) || (buf2 && !aligned16(buf2))) return fail(AS_ERR_ALIGN, "pointer not 16-byte aligned");
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  AS_TRY(AS_STAGE_MISC, launch_stream_probe(kind, buf, buf2, rows, row_bytes, st));
  return AS_OK;
}

as_status attn_softmax_profile_enable(int enable) {
  // drop whatever is pending
  for (auto& r : g_prof.pending) {
    g_prof.pool.push_back(r.a);
    g_prof.pool.push_back(r.b);
  }
  g_prof.pending.clear();
  for (int i = 0; i < AS_STAGE_COUNT; ++i) {
    g_prof.ms[i] = 0;
    g_prof.launches[i] = 0;
  }
  g_prof.on = enable != 0;
  g_prof.mask = ~0ull;
  return AS_OK;
}

as_status attn_softmax_profile_select(uint64_t stage_mask) {
  g_prof.mask = stage_mask;
  return AS_OK;
}

as_status attn_softmax_profile_read(double* ms_total, int64_t* launches) {
  for (auto& r : g_prof.pending) {
    hipError_t e = hipEventSynchronize(r.b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess) return fail(AS_ERR_HIP, "profile events: %s", hipGetErrorString(e));
    g_prof.ms[r.stage] += ms;
    g_prof.launches[r.stage] += 1;
    g_prof.pool.push_back(r.a);
    g_prof.pool.push_back(r.b);
  }
  g_prof.pending.clear();
  for (int i = 0; i < AS_STAGE_COUNT; ++i) {
    if (ms_total) ms_total[i] = g_prof.ms[i];
    if (launches) launches[i] = g_prof.launches[i];
  }
  return AS_OK;
}

}  // extern "C"
