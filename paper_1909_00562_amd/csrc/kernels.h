// Launchers of the row-wise kernels (masked attention softmax, vocabulary
// softmax cross-entropy).  All enqueue on `st` and return the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace asx {

// Eq. 1: alpha[b,t,:] = softmax(score[b,t,:]) over s < clamp(src_len[b],0,S),
// exactly 0 elsewhere.  Writes alpha32 [B,T,S], a copy in the storage type
// alphaE [B,T,ldS] (columns S..ldS-1 zero), if non-null the rounding remainder
// alphaE_lo = alpha - alphaE in the storage type, and, if non-null, attn_mask [B,S].
hipError_t launch_attn_softmax_rows(const float* score, const int32_t* src_len, int B, int T, int S,
                                    float* alpha32, void* alphaE, void* alphaE_lo, int64_t ldS, bool e_bf16,
                                    uint8_t* attn_mask, hipStream_t st);
// Softmax Jacobian: dscore = alpha * (dalpha - sum_s alpha*dalpha), storage type, [B,T,ldS] zero
// padded; dscoreE_lo (optional) receives the rounding remainder.
hipError_t launch_attn_softmax_rows_bwd(const float* alpha32, const float* dalpha, int B, int T, int S,
                                        void* dscoreE, void* dscoreE_lo, int64_t ldS, bool e_bf16,
                                        hipStream_t st);

// Eq. 1-3 fused for the batched path, bf16 storage, S <= 128 (attn_fwd_fused_supported): q_hi / q_lo [T,B,H] (Q = h_dec
// W_a as value and rounding remainder), h_enc [S,B,H] -> alpha32 [B,T,S], alphaE / alphaE_lo [B,T,ldS] (zero padded),
// ctx / ctx_lo [T,B,H], optional attn_mask [B,S].  One workgroup per (sentence, 32 decoder steps).
bool attn_fwd_fused_supported(int S, int H);
hipError_t launch_attn_fwd_fused(const void* q_hi, const void* q_lo, const void* h_enc, const int32_t* src_len, int B,
                                 int T, int S, int H, float* alpha32, void* alphaE, void* alphaE_lo, int64_t ldS,
                                 void* ctx, void* ctx_lo, uint8_t* attn_mask, hipStream_t st);
// First half of the attention backward pass with the same kernel: dC_hi / dC_lo [T,B,H], alpha32 [B,T,S] (read) ->
// dscoreE / dscoreE_lo [B,T,ldS] (softmax Jacobian, zero padded) and dQ [T,B,H] = dscore . h_enc (value only).
hipError_t launch_attn_bwd_fused(const void* dC_hi, const void* dC_lo, const void* h_enc, const int32_t* src_len,
                                 int B, int T, int S, int H, const float* alpha32, void* dscoreE, void* dscoreE_lo,
                                 int64_t ldS, void* dQ, hipStream_t st);

// Row compaction (rows / n_act below, both null = off): logits, lse and tok_loss_ws hold only the *n_act rows
// whose target is not padding, row r being position rows[r]; N stays the bound the launch is sized for.
// Position n -> row_pos[n] (its compacted row, -1 at padding), the list rows[0 .. *n_act) of positions in
// increasing order, *n_act; optional per-position outputs: tgt_mask everywhere, tok_loss = 0 and
// argmax = pad_id at padding (the statistics kernel fills the other positions).
hipError_t launch_row_compact(const int32_t* targets, int N, int V, int pad_id, int32_t* row_pos, int32_t* rows,
                              int32_t* n_act, uint8_t* tgt_mask, float* tok_loss, int32_t* argmax, hipStream_t st);
// dst_x[r] = src_x[rows[r]], r < *n_act; rows of bytes_x bytes (multiples of 4); the second array is optional
hipError_t launch_gather_rows(const int32_t* rows, const int32_t* n_act, int N, const void* src0, void* dst0,
                              int64_t bytes0, const void* src1, void* dst1, int64_t bytes1, hipStream_t st);
// dst_x[n] = src_x[row_pos[n]], zeros where row_pos[n] < 0; all N rows of dst are written; second array optional
hipError_t launch_scatter_rows(const int32_t* row_pos, int N, const void* src0, void* dst0, const void* src1,
                               void* dst1, int64_t bytes, hipStream_t st);

// Eq. 5-6 per row n of logits [N,ldV]: lse, loss, argmax, target mask.
hipError_t launch_xent_stats(const void* logits, int64_t ldV, bool e_bf16, int N, int V,
                             const int32_t* targets, int pad_id, float* lse, float* tok_loss_ws,
                             float* tok_loss, int32_t* argmax, uint8_t* tgt_mask, const int32_t* rows,
                             const int32_t* n_act, hipStream_t st);
// loss_sum = sum(tok_loss_ws) in double, n_tok = number of non-pad targets (= *n_act when given); fixed order.
hipError_t launch_loss_reduce(const float* tok_loss_ws, const int32_t* targets, int N, int V, int pad_id,
                              float* loss_sum, int32_t* n_tok, const int32_t* n_act, hipStream_t st);

// rows of logits handled by one block of the dlogits kernel (also sizes db_partial)
int xent_rows_per_block(int N, int V, bool e_bf16);
// dlogits = g * (exp(logit - lse) - onehot) on non-pad rows, 0 on pad rows and on
// columns V..ldV-1, in place; db_partial[rb][v] = column sums of row block rb.
hipError_t launch_xent_dlogits(void* logits, int64_t ldV, bool e_bf16, int N, int V, const int32_t* targets,
                               int pad_id, const float* lse, float g, float* db_partial, const int32_t* rows,
                               const int32_t* n_act, hipStream_t st);
// db_out[v] = sum_rb db_partial[rb][v]
hipError_t launch_db_reduce(const float* db_partial, int nrb, int V, float* db_out, hipStream_t st);

// One decoder step of attention, fused (Eq. 1-3 with T = 1): kprime [S,B,H] float = W_a h_enc, h_t [B,H],
// h_enc [S,B,H]; writes alpha [B,S] float, ctx [B,H] (+ optional rounding remainder ctx_lo), optional attn_mask.
hipError_t launch_attn_step(const void* h_t, const float* kprime, const void* h_enc, const int32_t* src_len, int B,
                            int S, int H, float* alpha, void* ctx, void* ctx_lo, bool e_bf16, uint8_t* attn_mask,
                            hipStream_t st);
// One LSTM time step of one layer, bf16 storage, fused (cell as in include/lstm_stack.h; H % 8 == 0).
// "Fragment-major" below: an operand X [rows, K] stored as XF[K/8][rows][8], so that the lanes holding the
// rows of an MFMA fragment read contiguous memory.
// Forward: WF = W_hh fragment-major with rows ordered unit*4 + gate (launch_ls_wfrag); hF_hi / hF_lo: h_{t-1}
// [B,H] fragment-major as bf16 value and rounding remainder; G [B,4H] holds the input half of the gate
// pre-activations (X W_ih^T + b) on entry and the gates i, f, g, o on exit; c_prev -> c_new [B,H] float;
// hf [B,H] running float h (written at valid rows); hFn_hi / hFn_lo: h_t fragment-major (h_{t-1} at padded
// rows); hE_new [B,H] row-major value of the same; out / out_lo (out_lo optional) [B,H] row-major: the layer's
// output of step t, 0 at padded rows.
struct LstmStepFwd {
  const uint16_t* WF;
  const uint16_t *hF_hi, *hF_lo;
  float* G;
  const float* c_prev;
  float* c_new;
  float* hf;
  uint16_t *hFn_hi, *hFn_lo, *hE_new, *out, *out_lo;
  const int32_t* lengths;
  int t, T, B, H;
  // dropout on out / out_lo (drop_thr = 0: none): element (b, j) of this step has flat index drop_index0 + b*H + j
  uint32_t drop_thr;
  float drop_scale;
  uint64_t drop_seed, drop_index0;
};
hipError_t launch_lstm_step_fwd(const LstmStepFwd& p, hipStream_t st);
// Backward of step t: WTF = W_hh^T [H,4H] fragment-major (launch_ls_wfrag, backward); dGnF: gate gradients
// of step t+1 [B,4H] fragment-major, bf16 value only (null for t = T-1); gates [B,4H], c_prev, c_new [B,H] as saved by
// the forward step; dout_t [B,H] gradient w.r.t. the layer's output; dhT [B,H] gradient w.r.t. the final h
// (null = 0); dcs [B,H] running gradient w.r.t. c (in: after step t, out: after step t-1); gate gradients of
// step t: dG_hi / dG_lo [B,4H] row-major (value, remainder) and dGF fragment-major (value).
// t = -1: dh0_out [B,H] = gradient w.r.t. the initial h, nothing else is touched.
struct LstmStepBwd {
  const uint16_t* WTF;
  const uint16_t* dGnF;
  const float *gates, *c_prev, *c_new, *dout_t, *dhT;
  float* dcs;
  uint16_t *dG_hi, *dG_lo, *dGF;
  float* dh0_out;
  const int32_t* lengths;
  int t, T, B, H;
  // the dropout the forward step applied to this layer's output: dout_t goes back through the same mask
  uint32_t drop_thr;
  float drop_scale;
  uint64_t drop_seed, drop_index0;
};
hipError_t launch_lstm_step_bwd(const LstmStepBwd& p, hipStream_t st);
// W_hh [4H,H] of one layer into the fragment-major form the forward (backward = false) or backward step reads
hipError_t launch_ls_wfrag(const void* W_hh, void* dst, int H, bool backward, hipStream_t st);

// Measurement aid: plain streams over `rows` chunks of `row_bytes` bytes (a multiple of 16).  kind 0: read-only with
// the statistics kernel's load pattern, buf2 receives 4 words per row; kind 1: copy buf -> buf2 and kind 2:
// in-place read-modify-write of buf, both with the dlogits kernel's grid and loads in flight.
hipError_t launch_stream_probe(int kind, void* buf, void* buf2, int rows, size_t row_bytes, hipStream_t st);

// Adam, bias corrections passed as inv_bc1 = 1 / (1 - beta1^step), inv_bc2 likewise; wout optional.
hipError_t launch_adam_step(size_t n, const float* grad, float* master, float* m, float* v, void* wout,
                            bool out_bf16, float lr, float beta1, float beta2, float eps, float inv_bc1,
                            float inv_bc2, hipStream_t st);

}  // namespace asx
