/*
 * attn_softmax.h -- C ABI of the attention-softmax library for MI355X (gfx950).
 *
 * The library computes, forward and backward, the data-parallel part of the
 * hybrid scheme of "Hybrid Data-Model Parallel Training for Sequence-to-Sequence
 * RNN Machine Translation" (section 3.2, "Proposed model for hybrid
 * parallelism"), for all decoder steps of a batch at once:
 *
 *   Eq. 2   score[b,t,s] = h_dec[t,b,:]^T  W_a  h_enc[s,b,:]
 *   Eq. 1   alpha[b,t,:] = softmax over the valid source positions s < src_len[b]
 *   Eq. 3   ctx[t,b,:]   = sum_s alpha[b,t,s] h_enc[s,b,:]
 *   Eq. 4   h_c[t,b,:]   = tanh( W_c [ ctx[t,b,:] ; h_dec[t,b,:] ] )
 *   Eq. 5   logits       = h_c W_out^T + b_out ;  P = softmax(logits)
 *   Eq. 6   loss_sum     = sum over non-pad target positions of -log P[target]
 *
 * and the gradients of grad_scale * loss_sum with respect to h_dec, h_enc, W_a,
 * W_c, W_out, b_out (the paper's backward pass "in a similar but opposite
 * direction").
 *
 * Conventions
 *   - T decoder steps, S source positions, B sentences, H hidden size, V
 *     vocabulary size; N = T*B rows, row n = t*B + b (time-major).
 *   - Every pointer is DEVICE memory owned by the caller, dense row-major, base
 *     16-byte aligned.  `hip_stream` is a hipStream_t (NULL = default stream).
 *     The library allocates and frees nothing and keeps no device state
 *     between calls except what it writes into the caller's workspace.
 *   - Calls only enqueue work on the stream: outputs are valid once the
 *     stream has been synchronised.  Calls sharing a workspace must be ordered
 *     on one stream.
 *   - dtype selects the storage type of states, weights, bias and of the saved
 *     activations: AS_F32 (float, fp32 arithmetic throughout) or AS_BF16
 *     (bfloat16 storage, products on the bf16 matrix cores with fp32
 *     accumulation, softmax arithmetic in fp32).  AS_BF16 requires H % 8 == 0.
 *   - Errors are returned as codes, never thrown; everything checkable on the
 *     host (null pointers, non-positive sizes, pad_id outside [0,V), unknown
 *     dtype, workspace too small, misalignment) is rejected before any launch.
 *     Launch failures give AS_ERR_HIP.  attn_softmax_last_error() returns a
 *     message for the calling thread's last failure.
 *   - Data faults have defined results: src_len[b] is clamped to [0,S];
 *     src_len[b] = 0 gives alpha = 0 and ctx = 0 for that sentence; a target
 *     equal to pad_id or outside [0,V) is padding (loss 0, zero gradient).
 */
#ifndef ATTN_SOFTMAX_H
#define ATTN_SOFTMAX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AS_OK = 0,
  AS_ERR_NULL = 1,       /* a required pointer is NULL */
  AS_ERR_SHAPE = 2,      /* a size is < 1, pad_id outside [0,V), or sizes overflow */
  AS_ERR_DTYPE = 3,      /* dtype is not AS_F32 / AS_BF16 */
  AS_ERR_WORKSPACE = 4,  /* workspace_bytes < attn_softmax_workspace_bytes() */
  AS_ERR_ALIGN = 5,      /* pointer not 16-byte aligned, or H % 8 != 0 for AS_BF16 */
  AS_ERR_HIP = 6         /* a HIP call or kernel launch failed */
} as_status;

typedef enum { AS_F32 = 0, AS_BF16 = 1 } as_dtype;

typedef struct {
  int32_t T, S, B, H, V;   /* all >= 1 */
  int32_t pad_id;          /* 0 <= pad_id < V */
  int32_t dtype;           /* as_dtype */
  float grad_scale;        /* g: gradients are those of g * loss_sum */
  /* Dropout on h_c (section 4.2, "Parameter settings": a dropout of 0.3), applied
   * after Eq. 4 and before Eq. 5 as inverted dropout: element (t,b,c), flat index
   * i = (t*B + b)*H + c, is kept iff word (i & 3) of philox4x32-10(counter = i >> 2,
   * key = dropout_seed) is >= floor(dropout_p * 2^32); kept elements are multiplied
   * by 1/(1 - dropout_p), dropped ones are 0.  AS_VIEW_HC then holds the dropped,
   * rescaled h_c, and the backward pass goes through the same mask (it is saved in
   * the workspace with the tanh derivative, not drawn again).  0 <= dropout_p < 1;
   * 0 switches it off.  The caller changes dropout_seed from step to step. */
  float dropout_p;
  uint64_t dropout_seed;
  /* Row compaction, 0 or 1.  A position whose target is padding contributes nothing to
   * the loss or to any gradient (Eq. 6 sums over the words of the sentence), so with 1
   * the vocabulary part of the path -- logits, softmax cross-entropy, dW_out, the
   * product with W_out in the backward pass -- runs only on the rows whose target is a
   * word.  The row list is made on the device; nothing is synchronised.  Loss, n_tok,
   * masks and all six gradients are the same as with 0 (up to the order of fp32
   * sums); at padding positions tok_loss = 0 and argmax = pad_id, and AS_VIEW_LOGITS /
   * AS_VIEW_LSE hold one row per non-pad position, in increasing n, located through
   * AS_VIEW_ROW_POS.  The per-step entry points ignore it. */
  int32_t skip_pad_rows;
} as_shape;

/* Saved activations readable through attn_softmax_view(). */
typedef enum {
  AS_VIEW_ALPHA = 0,   /* float  [B,T,S]   attention weights (Eq. 1)                */
  AS_VIEW_CTX = 1,     /* dtype  [T,B,H]   context vectors (Eq. 3)                  */
  AS_VIEW_HC = 2,      /* dtype  [T,B,H]   tanh(W_c[c;h]) (Eq. 4)                   */
  AS_VIEW_LOGITS = 3,  /* dtype  [N,ld]    logits after fwd, dlogits after bwd;     */
                       /*                  ld = *row_stride elements (>= V)         */
  AS_VIEW_LSE = 4,     /* float  [T,B]     log-sum-exp of each logits row           */
  AS_VIEW_ROW_POS = 5  /* int32  [T,B]     skip_pad_rows = 1 only: row of position (t,b) in */
                       /*                  AS_VIEW_LOGITS / AS_VIEW_LSE, -1 at padding      */
} as_view;

/* Bytes of workspace fwd+bwd need for this shape; 0 if the shape is invalid. */
size_t attn_softmax_workspace_bytes(const as_shape* shape);

/*
 * Forward pass, Eq. 1-6.  Fills the workspace with the saved activations and
 * writes the outputs below.  Optional outputs may be NULL.
 *   h_dec [T,B,H] dtype     h_enc [S,B,H] dtype     src_len [B] int32
 *   W_a [H,H] dtype   (row = decoder dim, col = encoder dim)
 *   W_c [H,2H] dtype  (cols 0..H-1 act on ctx, cols H..2H-1 on h_dec)
 *   W_out [V,H] dtype   b_out [V] dtype   targets [T,B] int32
 *   loss_sum [1] float  sum of -log P over non-pad positions (not scaled by g)
 *   n_tok    [1] int32  number of non-pad positions
 *   tok_loss [T,B] float (optional)  per-position loss, 0 at padding
 *   argmax   [T,B] int32 (optional)  lowest id attaining the row maximum of the
 *                                    stored logits
 *   attn_mask [B,S] uint8 (optional) 1 where s < src_len[b]
 *   tgt_mask  [T,B] uint8 (optional) 1 where the target is not padding
 */
as_status attn_softmax_fwd(const as_shape* shape,
                           const void* h_dec, const void* h_enc, const int32_t* src_len,
                           const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                           const int32_t* targets,
                           float* loss_sum, int32_t* n_tok,
                           float* tok_loss, int32_t* argmax, uint8_t* attn_mask, uint8_t* tgt_mask,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * attn_softmax_fwd for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight scoring / decoding loops (T = 1 per call), harnesses that forbid hipMalloc.  Same inputs,
 * outputs, arithmetic and kernels as attn_softmax_fwd; the workspace is a 64 MiB array the library's code object
 * holds on every GPU it runs on (AS_STATIC_SCRATCH_BYTES), so there is no workspace argument, no saved activation
 * can be viewed afterwards and no backward pass can follow.  The call allocates and frees nothing.
 *   - A shape whose attn_softmax_workspace_bytes() exceeds AS_STATIC_SCRATCH_BYTES is rejected with
 *     AS_ERR_WORKSPACE before any launch (the paper's model size, S = 50, H = 1024, V = 32000 in bf16, fits up
 *     to N = T*B = 256 positions per call: one decoder step of 256 sentences, two of 128).
 *   - The calling thread's current device must be the one hip_stream belongs to.  The first call on a device
 *     looks the array's address up (not a capturable operation): make one call outside graph capture first.
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents (nothing in it
 *     needs to start at zero: every region is written before it is read).  Calls that overlap on one GPU,
 *     on different streams or from different threads, race; order them on one stream.
 * Errors otherwise as attn_softmax_fwd.
 */
#define AS_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
as_status attn_softmax_fwd_static(const as_shape* shape,
                                  const void* h_dec, const void* h_enc, const int32_t* src_len,
                                  const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                                  const int32_t* targets,
                                  float* loss_sum, int32_t* n_tok,
                                  float* tok_loss, int32_t* argmax, uint8_t* attn_mask, uint8_t* tgt_mask,
                                  void* hip_stream);

/*
 * Backward pass of grad_scale * loss_sum.  Takes the inputs of the forward
 * call and the workspace exactly as that call left it; overwrites (does not
 * accumulate into) the six float gradient outputs, all required:
 *   d_h_dec [T,B,H]  d_h_enc [S,B,H] (rows s >= src_len[b] exactly 0)
 *   dW_a [H,H]  dW_c [H,2H]  dW_out [V,H]  db_out [V]
 * The logits in the workspace are replaced in place by
 * dlogits = g * (softmax(logits) - onehot(target)), rows at padding = 0, so one
 * forward call supports one backward call.
 */
as_status attn_softmax_bwd(const as_shape* shape,
                           const void* h_dec, const void* h_enc, const int32_t* src_len,
                           const void* W_a, const void* W_c, const void* W_out, const void* b_out,
                           const int32_t* targets,
                           void* workspace, size_t workspace_bytes,
                           float* d_h_dec, float* d_h_enc,
                           float* dW_a, float* dW_c, float* dW_out, float* db_out,
                           void* hip_stream);

/*
 * Address of a saved activation inside the workspace (device pointer, no copy,
 * no launch).  *bytes is its extent; *row_stride (optional) the leading
 * dimension in elements for AS_VIEW_LOGITS, else the dense one.
 */
as_status attn_softmax_view(const as_shape* shape, void* workspace, int which,
                            void** ptr, size_t* bytes, int64_t* row_stride);

/* Message for the calling thread's last non-OK return (static storage). */
const char* attn_softmax_last_error(void);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel the library
 * enqueues is bracketed by HIP events on the caller's stream.
 * attn_softmax_profile_read synchronises those events, adds the elapsed times
 * into per-stage totals and returns them; stage ids are as_stage.  Enabling
 * clears the totals.  Not thread-safe; meant for one benchmarking thread.
 */
typedef enum {
  AS_STAGE_GEMM_Q = 0,        /* Q = h_dec W_a                      (Eq. 2)  */
  AS_STAGE_ATTN_SCORE = 1,    /* batched Q_b h_enc_b^T              (Eq. 2)  */
  AS_STAGE_ATTN_SOFTMAX = 2,  /* masked softmax rows                (Eq. 1)  */
  AS_STAGE_ATTN_CTX = 3,      /* batched alpha_b h_enc_b            (Eq. 3)  */
  AS_STAGE_GEMM_HC = 4,       /* tanh(W_c[c;h])                     (Eq. 4)  */
  AS_STAGE_GEMM_LOGITS = 5,   /* h_c W_out^T + b_out                (Eq. 5)  */
  AS_STAGE_XENT_STATS = 6,    /* online max/sum, loss, argmax       (Eq. 5-6)*/
  AS_STAGE_XENT_DLOGITS = 7,  /* dlogits in place + db_out                   */
  AS_STAGE_GEMM_DWOUT = 8,    /* dW_out = dlogits^T h_c                      */
  AS_STAGE_GEMM_DHC = 9,      /* dz = (dlogits W_out) * (1 - h_c^2)          */
  AS_STAGE_GEMM_DWC = 10,     /* dW_c = dz^T [c;h]                           */
  AS_STAGE_GEMM_DCH = 11,     /* [dC ; dH1] = dz W_c                         */
  AS_STAGE_ATTN_BWD = 12,     /* batched attention backward products         */
  AS_STAGE_ATTN_SOFTMAX_BWD = 13,
  AS_STAGE_GEMM_DWA = 14,     /* dW_a = h_dec^T dQ                           */
  AS_STAGE_GEMM_DH = 15,      /* d_h_dec = dH1 + dQ W_a^T                    */
  AS_STAGE_MISC = 16,         /* small reductions, split-K combine           */
  AS_STAGE_ADAM = 17,         /* attn_softmax_adam_step                      */
  AS_STAGE_COMPACT = 18,      /* row list, gather of h_c rows, scatter of dz */
  AS_STAGE_COUNT = 19
} as_stage;

as_status attn_softmax_profile_enable(int enable);
/* Restrict the timing to the stages whose bit (1 << as_stage) is set, e.g. to keep the events of a
 * measurement out of the small kernels' way; attn_softmax_profile_enable selects all stages again. */
as_status attn_softmax_profile_select(uint64_t stage_mask);
/* ms_total[AS_STAGE_COUNT], launches[AS_STAGE_COUNT]; either may be NULL. */
as_status attn_softmax_profile_read(double* ms_total, int64_t* launches);

/*
 * Measurement aid for benchmarks: plain streaming kernels with the access patterns of the two softmax
 * cross-entropy kernels (Eq. 5-6) and none of their arithmetic, to measure what this GPU's memory system gives
 * such a stream.  `rows` chunks of `row_bytes` bytes each (a multiple of 16, one logits row), device memory:
 *   kind 0  read-only: one block per row, eight 16-byte streaming loads in flight per thread (the statistics
 *           kernel's pattern); buf2 receives 4 * rows uint32 words (so that the loads cannot be dropped)
 *   kind 1  copy buf -> buf2 (rows * row_bytes bytes), the dlogits kernel's grid and loads in flight
 *   kind 2  in-place read-modify-write of buf (each 16-bit element's sign bit flipped), same grid
 * Errors: AS_ERR_NULL, AS_ERR_SHAPE, AS_ERR_ALIGN, AS_ERR_HIP.
 */
as_status attn_softmax_stream_probe(int kind, void* buf, void* buf2, int32_t rows, size_t row_bytes,
                                    void* hip_stream);

/*
 * Per-step mode: one decoder step (T = 1) at a time, for decoding, scoring and the
 * input-feeding variant of the model (section 4, "HybridNMTIF": the attentional
 * state of step t is an input of step t+1, so the steps cannot be batched).
 * The encoder-side half of the score of Eq. 2, K'[s,b,:] = W_a h_enc[s,b,:], does
 * not depend on the step: attn_softmax_step_prepare computes it once per batch of
 * sentences into the workspace; attn_softmax_step_fwd then runs Eq. 1-3 as one
 * fused kernel (score[s] = h_t[b] . K'[s,b], masked softmax, context) followed by
 * Eq. 4-6 exactly as attn_softmax_fwd does.  shape->T is ignored (taken as 1);
 * h_t [B,H] dtype is the decoder state of this step, targets [B] the words to
 * score (pad_id everywhere when only the prediction is wanted).  Outputs as in
 * attn_softmax_fwd with T = 1; the step's attention weights, context, h_c, logits
 * and lse are read with attn_softmax_view() (same workspace, shape with T = 1).
 * The workspace (attn_softmax_step_workspace_bytes) must not be used by another
 * call between prepare and the steps that follow it.  Dropout applies as in
 * attn_softmax_fwd when shape->dropout_p > 0.  Errors as attn_softmax_fwd.
 * The step entry points are forward-only: attn_softmax_step_fwd does not save what the backward products read
 * (Q = h_t W_a and the storage-type copies of the attention weights), so attn_softmax_bwd must NOT be called on
 * a workspace a step left.  Per-step training (the input-feeding variant) runs attn_softmax_fwd with T = 1
 * followed by attn_softmax_bwd with the same shape (same skip_pad_rows in both calls).
 */
size_t attn_softmax_step_workspace_bytes(const as_shape* shape);
as_status attn_softmax_step_prepare(const as_shape* shape, const void* h_enc, const void* W_a,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);
as_status attn_softmax_step_fwd(const as_shape* shape,
                                const void* h_t, const void* h_enc, const int32_t* src_len,
                                const void* W_c, const void* W_out, const void* b_out,
                                const int32_t* targets,
                                float* loss_sum, int32_t* n_tok, float* tok_loss, int32_t* argmax,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One Adam update of one parameter tensor of this part of the model (section
 * 4.2, "Parameter settings": Adam with beta1 = 0.9, beta2 = 0.999, eps = 1e-8;
 * Table 2: initial learning rate 0.001), bias-corrected as in Kingma and Ba's
 * Algorithm 1:
 *   m = beta1 m + (1 - beta1) g ;  v = beta2 v + (1 - beta2) g^2
 *   master -= lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 * n elements; grad [n] float (as attn_softmax_bwd wrote it, read only);
 * master, m, v [n] float, updated in place (m = v = 0 before step 1);
 * weights_out [n] of `dtype` (optional): the updated master rounded to the
 * storage type the forward pass reads (round to nearest even for AS_BF16).
 * All pointers are device memory, 16-byte aligned; step >= 1; the learning-rate
 * decay of the paper is the caller's policy (pass the decayed lr).
 * Errors: AS_ERR_NULL, AS_ERR_SHAPE (n = 0, step < 1, betas outside [0,1)),
 * AS_ERR_DTYPE, AS_ERR_ALIGN, AS_ERR_HIP.
 */
typedef struct {
  float lr, beta1, beta2, eps;
  int32_t step;            /* 1 for the first update */
} as_adam;

as_status attn_softmax_adam_step(const as_adam* hyper, size_t n, const float* grad,
                                 float* master, float* m, float* v,
                                 void* weights_out, int32_t dtype, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ATTN_SOFTMAX_H */
