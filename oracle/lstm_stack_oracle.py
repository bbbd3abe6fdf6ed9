"""Float64 CPU oracle of the stacked-LSTM part of the model (TEST INFRASTRUCTURE).

This file is the checker, not the product: only tests/, __graft_entry__.smoke()
and bench.py's cpu_baseline leg may import it.  It shares no code with the HIP
path and imports nothing from the package.

What it computes: the hidden states of all steps of one side (encoder or
decoder) of the proposed model of section 3.2 (Fig. 3): stacked LSTM layers
WITHOUT input feeding, so that the input of the first layer is the word
embedding alone and all steps of a layer depend only on the layer below and on
the previous step (Table 2: depth 4, hidden state size 1024, word embedding size
512).  The paper does not print the cell ("straightforward"); the cell is the
standard LSTM with forget gate, as in the cited attention model:

    [a_i; a_f; a_g; a_o] = W_ih x_t + W_hh h_{t-1} + b        (four blocks of H rows)
    i = sigmoid(a_i)  f = sigmoid(a_f)  g = tanh(a_g)  o = sigmoid(a_o)
    c_t = f * c_{t-1} + i * g          h_t = o * tanh(c_t)

no peepholes, no projection, one bias vector per layer.  Layer l+1 reads the
h_t of layer l.  Sentences are right-padded: at steps t >= lengths[b] sentence b
keeps its state (h_t = h_{t-1}, c_t = c_{t-1}) and the layer's output for that
step is 0, so the final state is the state after the sentence's last word.

Dropout (section 4.2 names "a dropout of 0.3" and no placement): the usual placement for
stacked LSTMs, on the connections BETWEEN layers only, never on the recurrent ones and
not on the top layer's output (the attentional state has its own).  `drop` is the
array of multipliers [L-1, T, B, H] (0 where dropped, 1/(1-p) where kept) that layer
l+1 sees on the output of layer l; the random decisions are made by the caller
(train_extras_oracle.dropout_multiplier over (L-1)*T "steps", i.e. element (l,t,b,j) has
flat index ((l*T + t)*B + b)*H + j) and passed in.

Everything is plain numpy float64, one time step after the other, no blocking.
"""
from __future__ import annotations

import numpy as np


def _sigmoid(a):
    return 0.5 * (1.0 + np.tanh(0.5 * a))      # = 1 / (1 + exp(-a)), without overflow for large |a|


def forward(x, lengths, W_ih, W_hh, b, h0=None, c0=None, drop=None):
    """x [T,B,I0]; lengths [B] (clamped to [0,T]); per layer l: W_ih[l] [4H,I_l] (I_0 = I0, I_l = H),
    W_hh[l] [4H,H], b[l] [4H]; h0, c0 [L,B,H] or None (zeros).
    Returns y [T,B,H] (top layer, 0 at padded steps), hT, cT [L,B,H], and `saved` for backward()."""
    x = np.asarray(x, dtype=np.float64)
    T, B, _ = x.shape
    L = len(W_ih)
    H = np.asarray(W_hh[0]).shape[1]
    lengths = np.clip(np.asarray(lengths, dtype=np.int64), 0, T)
    valid = (np.arange(T)[:, None] < lengths[None, :])                 # [T,B]
    hT = np.zeros((L, B, H))
    cT = np.zeros((L, B, H))
    saved = []
    inp = x
    for l in range(L):
        Wi = np.asarray(W_ih[l], dtype=np.float64)
        Wh = np.asarray(W_hh[l], dtype=np.float64)
        bl = np.asarray(b[l], dtype=np.float64)
        h = np.zeros((B, H)) if h0 is None else np.asarray(h0[l], dtype=np.float64).copy()
        c = np.zeros((B, H)) if c0 is None else np.asarray(c0[l], dtype=np.float64).copy()
        hs = np.zeros((T + 1, B, H))       # hs[t] = state before step t, hs[T] = final
        cs = np.zeros((T + 1, B, H))
        gates = np.zeros((T, B, 4, H))     # i, f, g, o after their nonlinearity
        out = np.zeros((T, B, H))
        hs[0], cs[0] = h, c
        for t in range(T):
            a = inp[t] @ Wi.T + h @ Wh.T + bl                          # [B,4H]
            a = a.reshape(B, 4, H)
            i, f, g, o = _sigmoid(a[:, 0]), _sigmoid(a[:, 1]), np.tanh(a[:, 2]), _sigmoid(a[:, 3])
            c_new = f * c + i * g
            h_new = o * np.tanh(c_new)
            m = valid[t][:, None]
            c = np.where(m, c_new, c)
            h = np.where(m, h_new, h)
            out[t] = np.where(m, h_new, 0.0)
            gates[t, :, 0], gates[t, :, 1], gates[t, :, 2], gates[t, :, 3] = i, f, g, o
            hs[t + 1], cs[t + 1] = h, c
        hT[l], cT[l] = h, c
        saved.append(dict(inp=inp, hs=hs, cs=cs, gates=gates, Wi=Wi, Wh=Wh))
        inp = out
        if drop is not None and l + 1 < L:
            inp = out * np.asarray(drop[l], dtype=np.float64)       # what the next layer reads
    return dict(y=inp, hT=hT, cT=cT, saved=saved, valid=valid, drop=drop)


def backward(fwd, dy, dhT=None, dcT=None):
    """Gradients of a scalar whose derivative w.r.t. y is dy [T,B,H] and w.r.t. the final states is
    dhT, dcT [L,B,H] (None = 0).  Returns dx [T,B,I0], dW_ih[l], dW_hh[l], db[l], dh0, dc0 [L,B,H]."""
    saved, valid = fwd["saved"], fwd["valid"]
    L = len(saved)
    T, B = valid.shape
    H = saved[0]["Wh"].shape[1]
    dW_ih, dW_hh, db = [None] * L, [None] * L, [None] * L
    dh0 = np.zeros((L, B, H))
    dc0 = np.zeros((L, B, H))
    dout = np.asarray(dy, dtype=np.float64)
    for l in range(L - 1, -1, -1):
        sv = saved[l]
        Wi, Wh = sv["Wi"], sv["Wh"]
        dh = np.zeros((B, H)) if dhT is None else np.asarray(dhT[l], dtype=np.float64).copy()
        dc = np.zeros((B, H)) if dcT is None else np.asarray(dcT[l], dtype=np.float64).copy()
        dWi = np.zeros_like(Wi)
        dWh = np.zeros_like(Wh)
        dbl = np.zeros(4 * H)
        dinp = np.zeros_like(sv["inp"])
        for t in range(T - 1, -1, -1):
            m = valid[t][:, None]
            i, f, g, o = (sv["gates"][t, :, k] for k in range(4))
            c_prev, c_new = sv["cs"][t], sv["cs"][t + 1]
            h_prev = sv["hs"][t]
            # valid step: h_t = o tanh(c_t) receives the output gradient and the recurrent one
            dh_t = np.where(m, dout[t] + dh, 0.0)
            tc = np.tanh(c_new)
            do = dh_t * tc
            dc_t = np.where(m, dc + dh_t * o * (1.0 - tc * tc), 0.0)
            da = np.stack([dc_t * g * i * (1.0 - i), dc_t * c_prev * f * (1.0 - f),
                           dc_t * i * (1.0 - g * g), do * o * (1.0 - o)], axis=1).reshape(B, 4 * H)
            dWi += da.T @ sv["inp"][t]
            dWh += da.T @ h_prev
            dbl += da.sum(axis=0)
            dinp[t] = da @ Wi
            # padded step: the state passes through unchanged, so do its gradients
            dh = np.where(m, da @ Wh, dh)
            dc = np.where(m, dc_t * f, dc)
        dW_ih[l], dW_hh[l], db[l] = dWi, dWh, dbl
        dh0[l], dc0[l] = dh, dc
        dout = dinp
        if fwd.get("drop") is not None and l > 0:
            dout = dinp * np.asarray(fwd["drop"][l - 1], dtype=np.float64)   # back through the mask on layer l-1's output
    return dict(dx=dout, dW_ih=dW_ih, dW_hh=dW_hh, db=db, dh0=dh0, dc0=dc0)
