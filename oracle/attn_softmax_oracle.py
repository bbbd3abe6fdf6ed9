"""CPU oracle for the attention-softmax path.  TEST INFRASTRUCTURE ONLY.

Plain float64 numpy, one sentence at a time, no blocking or fusion.  It is the
definition written out and serves only to check the HIP library: nothing in
the product path may import it, and it imports nothing from the product.

What it computes (paper section 3.2, "Proposed model for hybrid parallelism"):
  Eq. 2   attention scores  score[t,s] = h_t^T W_a h_s   (Luong "general" form)
  Eq. 1   alpha = softmax of the scores over source positions, with padded
          source positions (s >= src_len[b]) excluded: their weight is exactly 0
  Eq. 3   context vectors   c_t = sum_s alpha[t,s] h_s
  Eq. 4   "context decoded"  h~_t = tanh(W_c [c_t ; h_t])      (no bias)
  Eq. 5   word probabilities P = softmax(F_c(h~)), F_c linear: W_out h~ + b_out
  Eq. 6   P_i = P(y_i | y_<i, x): the training loss is -log P_i summed over the
          target positions that are not padding
and the gradients of  grad_scale * loss_sum  with respect to every input
tensor (the paper only says the backward pass runs "in a similar but opposite
direction"; the formulas below are derived by hand from Eq. 1-6).

Readings where the paper is silent: the batch is block diagonal (sentence b
attends only to its own source); W_a[i,j] pairs decoder dim i with encoder dim
j; the concatenation order is [c ; h_t] (columns 0..H-1 of W_c act on c);
src_len is clamped to [0,S] and src_len = 0 gives alpha = 0 and c = 0; a target
equal to pad_id, or outside [0,V), is padding: loss 0 and zero gradient
contribution; argmax ties go to the lowest id.

Parity status: pinned (tests/test_oracle_pins.py: invariants, closed forms,
scipy logsumexp, loop-only brute force, central finite differences on every
gradient element).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _as64(x):
    return np.asarray(x, dtype=F64)


def _sentence_forward(Hd, Se_full, L, W_a, W_c, W_out, b_out, y, pad_id, Dm=None):
    """Forward for one sentence.  Hd [T,H], Se_full [S,H], L valid source positions.

    Dm [T,H] (optional): dropout multiplier on h~ (0 or 1/(1-p)); the output
    projection then sees Hu = Dm * h~ while tanh' in the backward pass keeps h~."""
    T, H = Hd.shape
    S = Se_full.shape[0]
    V = W_out.shape[0]
    Se = Se_full[:L]
    Q = Hd @ W_a                                  # q_t = W_a^T h_t           (Eq. 2, first half)
    alpha = np.zeros((T, S), dtype=F64)
    if L > 0:
        score = Q @ Se.T                          # score[t,s] = q_t . h_s     (Eq. 2)
        m = score.max(axis=1, keepdims=True)
        e = np.exp(score - m)
        alpha[:, :L] = e / e.sum(axis=1, keepdims=True)       # Eq. 1 over valid positions
    C = alpha[:, :L] @ Se                         # Eq. 3
    Z = C @ W_c[:, :H].T + Hd @ W_c[:, H:].T      # W_c [c ; h_t]
    Ht = np.tanh(Z)                               # Eq. 4
    Hu = Ht if Dm is None else Ht * Dm            # what the output layer is fed
    logits = Hu @ W_out.T + b_out                 # Eq. 5, F_c
    M = logits.max(axis=1)
    lse = M + np.log(np.exp(logits - M[:, None]).sum(axis=1))
    nonpad = (y != pad_id) & (y >= 0) & (y < V)
    ysafe = np.where(nonpad, y, 0)
    tok_loss = np.where(nonpad, lse - logits[np.arange(T), ysafe], 0.0)   # -log P_i, Eq. 6
    argmax = logits.argmax(axis=1)                # numpy returns the first (lowest) maximiser
    return dict(Q=Q, alpha=alpha, C=C, Ht=Ht, Hu=Hu, logits=logits, lse=lse,
                nonpad=nonpad, ysafe=ysafe, tok_loss=tok_loss, argmax=argmax)


def forward(h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, pad_id,
            keep_logits=True, sentences=None, drop=None):
    """Forward pass for the whole batch (or the listed sentences).

    h_dec [T,B,H], h_enc [S,B,H], src_len [B], W_a [H,H], W_c [H,2H],
    W_out [V,H], b_out [V], targets [T,B].  Returns a dict; per-sentence arrays
    keep the caller's layout ([T,B,...], alpha as [B,T,S]) and hold zeros for
    sentences that were not requested.  drop [T,B,H] (optional) is the dropout
    multiplier on h~; the returned h_c is then the dropped, rescaled h~.
    """
    h_dec, h_enc = _as64(h_dec), _as64(h_enc)
    W_a, W_c, W_out, b_out = _as64(W_a), _as64(W_c), _as64(W_out), _as64(b_out)
    targets = np.asarray(targets)
    T, B, H = h_dec.shape
    S = h_enc.shape[0]
    V = W_out.shape[0]
    todo = range(B) if sentences is None else list(sentences)
    out = dict(
        alpha=np.zeros((B, T, S), F64), ctx=np.zeros((T, B, H), F64), h_c=np.zeros((T, B, H), F64),
        lse=np.zeros((T, B), F64), tok_loss=np.zeros((T, B), F64),
        argmax=np.zeros((T, B), np.int64), attn_mask=np.zeros((B, S), np.uint8),
        tgt_mask=np.zeros((T, B), np.uint8))
    if keep_logits:
        out["logits"] = np.zeros((T, B, V), F64)
    loss_sum = 0.0
    n_tok = 0
    for b in todo:
        L = int(min(max(int(src_len[b]), 0), S))
        r = _sentence_forward(h_dec[:, b], h_enc[:, b], L, W_a, W_c, W_out, b_out,
                              targets[:, b], pad_id, None if drop is None else drop[:, b])
        out["alpha"][b] = r["alpha"]
        out["ctx"][:, b] = r["C"]
        out["h_c"][:, b] = r["Hu"]
        out["lse"][:, b] = r["lse"]
        out["tok_loss"][:, b] = r["tok_loss"]
        out["argmax"][:, b] = r["argmax"]
        out["attn_mask"][b, :L] = 1
        out["tgt_mask"][:, b] = r["nonpad"].astype(np.uint8)
        if keep_logits:
            out["logits"][:, b] = r["logits"]
        loss_sum += float(r["tok_loss"].sum())
        n_tok += int(r["nonpad"].sum())
    out["loss_sum"] = loss_sum
    out["n_tok"] = n_tok
    return out


def backward(h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, pad_id,
             grad_scale=1.0, keep_dlogits=False, sentences=None, drop=None):
    """Gradients of  grad_scale * loss_sum  (loss_sum over the listed sentences).

    Returns d_h_dec [T,B,H], d_h_enc [S,B,H], dW_a, dW_c, dW_out, db_out (and
    dlogits [T,B,V] on request).  The forward quantities are recomputed here
    sentence by sentence so that memory stays bounded by one sentence's logits.
    """
    h_dec, h_enc = _as64(h_dec), _as64(h_enc)
    W_a, W_c, W_out, b_out = _as64(W_a), _as64(W_c), _as64(W_out), _as64(b_out)
    targets = np.asarray(targets)
    T, B, H = h_dec.shape
    S = h_enc.shape[0]
    V = W_out.shape[0]
    g = float(grad_scale)
    todo = range(B) if sentences is None else list(sentences)
    d_h_dec = np.zeros((T, B, H), F64)
    d_h_enc = np.zeros((S, B, H), F64)
    dW_a = np.zeros((H, H), F64)
    dW_c = np.zeros((H, 2 * H), F64)
    dW_out = np.zeros((V, H), F64)
    db_out = np.zeros((V,), F64)
    dlogits_all = np.zeros((T, B, V), F64) if keep_dlogits else None
    for b in todo:
        L = int(min(max(int(src_len[b]), 0), S))
        Hd = h_dec[:, b]
        Se = h_enc[:L, b]
        Dm = None if drop is None else drop[:, b]
        r = _sentence_forward(Hd, h_enc[:, b], L, W_a, W_c, W_out, b_out, targets[:, b], pad_id, Dm)
        # d loss / d logits = softmax - onehot on non-pad rows, 0 on pad rows
        P = np.exp(r["logits"] - r["lse"][:, None])
        dlog = P
        dlog[np.arange(T), r["ysafe"]] -= 1.0
        dlog *= g * r["nonpad"][:, None]
        if keep_dlogits:
            dlogits_all[:, b] = dlog
        db_out += dlog.sum(axis=0)
        dW_out += dlog.T @ r["Hu"]
        dHt = dlog @ W_out                                   # gradient at the output layer's input
        if Dm is not None:
            dHt = dHt * Dm                                   # back through the dropout multiplier
        dZ = dHt * (1.0 - r["Ht"] ** 2)                      # tanh'
        dW_c[:, :H] += dZ.T @ r["C"]
        dW_c[:, H:] += dZ.T @ Hd
        dC = dZ @ W_c[:, :H]
        dH1 = dZ @ W_c[:, H:]
        alpha = r["alpha"][:, :L]
        dalpha = dC @ Se.T                                   # [T,L]
        rowdot = (alpha * dalpha).sum(axis=1, keepdims=True)
        dscore = alpha * (dalpha - rowdot)                   # softmax Jacobian
        d_h_enc[:L, b] += alpha.T @ dC + dscore.T @ r["Q"]
        dQ = dscore @ Se
        dW_a += Hd.T @ dQ
        d_h_dec[:, b] = dH1 + dQ @ W_a.T
    out = dict(d_h_dec=d_h_dec, d_h_enc=d_h_enc, dW_a=dW_a, dW_c=dW_c, dW_out=dW_out, db_out=db_out)
    if keep_dlogits:
        out["dlogits"] = dlogits_all
    return out


def scaled_loss(h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, pad_id, grad_scale=1.0, drop=None):
    """The scalar whose gradient `backward` returns."""
    f = forward(h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, pad_id, keep_logits=False, drop=drop)
    return grad_scale * f["loss_sum"]
