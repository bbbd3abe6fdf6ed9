/*
 * lstm_stack.h -- C ABI of the stacked-LSTM part of the model for MI355X (gfx950).
 *
 * The step before the attention-softmax part in the proposed model of "Hybrid
 * Data-Model Parallel Training for Sequence-to-Sequence RNN Machine Translation"
 * (section 3.2, Fig. 3): the hidden states of ALL steps of one side (encoder or
 * decoder) of the stacked LSTM WITHOUT input feeding, forward and backward
 * (Table 2: depth 4, hidden state size 1024, word embedding size 512).  The
 * paper does not print the cell; it is the standard LSTM with forget gate:
 *
 *   [a_i; a_f; a_g; a_o] = W_ih x_t + W_hh h_{t-1} + b         (four blocks of H rows)
 *   i = sigmoid(a_i)  f = sigmoid(a_f)  g = tanh(a_g)  o = sigmoid(a_o)
 *   c_t = f * c_{t-1} + i * g           h_t = o * tanh(c_t)
 *
 * Layer l+1 reads the h_t of layer l.  Sentences are right-padded: at steps
 * t >= lengths[b] (lengths clamped to [0,T]) sentence b keeps its state and the
 * layer's output for that step is 0, so hT / cT are the states after each
 * sentence's last word.  One call handles one side; the caller chains them
 * (decoder h0/c0 = encoder hT/cT; encoder dhT/dcT = decoder dh0/dc0), feeds y to
 * attn_softmax_fwd as h_enc / h_dec and its d_h_enc / d_h_dec back in as dy.
 *
 * Conventions as in attn_softmax.h: every data pointer is DEVICE memory owned by
 * the caller, dense row-major, 16-byte aligned; W_ih / W_hh / b / dW_ih / dW_hh /
 * db are HOST arrays of L device pointers; calls only enqueue on hip_stream; the
 * library allocates nothing; errors are returned as as_status codes
 * (attn_softmax_last_error() has the message), host-checkable faults before any
 * launch.  dtype: AS_F32 (float storage, fp64-accumulated products) or AS_BF16
 * (bfloat16 x, weights, bias and y; products on the matrix cores with fp32
 * accumulation; cell arithmetic and the c / h state in fp32); AS_BF16 requires
 * I % 8 == 0 and H % 8 == 0.
 */
#ifndef LSTM_STACK_H
#define LSTM_STACK_H

#include "attn_softmax.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t T, B;    /* steps, sentences: >= 1 */
  int32_t I;       /* width of x (the word embedding): >= 1 */
  int32_t H;       /* hidden state size: >= 1 */
  int32_t L;       /* layers: 1..16 */
  int32_t dtype;   /* as_dtype */
  /* Dropout on the connections BETWEEN layers (section 4.2 names "a dropout of 0.3" and no
   * placement; the recurrent connections and the top layer's output y are left alone):
   * what layer l+1 reads of layer l's output element (t,b,j), flat index
   * i = ((l*T + t)*B + b)*H + j, is kept iff word (i & 3) of philox4x32-10(counter = i >> 2,
   * key = dropout_seed) is >= floor(dropout_p * 2^32), kept elements are multiplied by
   * 1/(1 - dropout_p); the backward pass draws the same words again.  0 <= dropout_p < 1,
   * 0 switches it off; the caller changes the seed from step to step (and uses different
   * seeds for the encoder and the decoder). */
  float dropout_p;
  uint64_t dropout_seed;
} ls_shape;

/* Bytes of workspace fwd+bwd need; 0 if the shape is invalid. */
size_t lstm_stack_workspace_bytes(const ls_shape* shape);

/*
 * Forward.  x [T,B,I] dtype; lengths [B] int32; W_ih[l] [4H, I_l] dtype with
 * I_0 = I and I_l = H above; W_hh[l] [4H,H] dtype; b[l] [4H] dtype (gate blocks
 * in the order i, f, g, o); h0, c0 [L,B,H] float or NULL (zeros).
 * Outputs: y [T,B,H] dtype, the top layer's h_t (0 at padded steps);
 * hT, cT [L,B,H] float (either may be NULL).  The workspace keeps what the
 * backward pass needs (gates, cell states, layer outputs).
 */
as_status lstm_stack_fwd(const ls_shape* shape, const void* x, const int32_t* lengths,
                         const void* const* W_ih, const void* const* W_hh, const void* const* b,
                         const float* h0, const float* c0,
                         void* y, float* hT, float* cT,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward of a scalar with derivative dy [T,B,H] float w.r.t. y (entries at
 * padded steps are ignored) and dhT, dcT [L,B,H] float (NULL = 0) w.r.t. the
 * final states.  Takes x, lengths, W_ih, W_hh of the forward call and its
 * workspace; overwrites dx [T,B,I] float (0 at padded steps), dW_ih[l] [4H,I_l],
 * dW_hh[l] [4H,H], db[l] [4H] float, and dh0, dc0 [L,B,H] float (may be NULL).
 */
as_status lstm_stack_bwd(const ls_shape* shape, const void* x, const int32_t* lengths,
                         const void* const* W_ih, const void* const* W_hh,
                         const float* dy, const float* dhT, const float* dcT,
                         void* workspace, size_t workspace_bytes,
                         float* dx, float* const* dW_ih, float* const* dW_hh, float* const* db,
                         float* dh0, float* dc0, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LSTM_STACK_H */
