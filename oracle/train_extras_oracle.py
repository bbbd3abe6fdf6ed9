"""CPU oracle for the training-step extras of the attention-softmax part.
TEST INFRASTRUCTURE ONLY: nothing in the product path may import it.

What it holds (paper section 4.2, "Parameter settings": a dropout of 0.3 and Adam
with beta1 = 0.9, beta2 = 0.999, eps = 1e-8; Table 2: initial learning rate 0.001):

  philox4x32_10      the counter-based generator of Salmon, Moraes, Dror and Shaw
                     ("Parallel random numbers: as easy as 1, 2, 3", SC'11) that
                     decides which elements are dropped.  The HIP side implements
                     the same published algorithm on its own; the two share no code.
  dropout_multiplier the [T,B,H] array of 0 or 1/(1-p) applied to h~ (Eq. 4)
                     before the output projection (inverted dropout of Srivastava
                     et al.).  Element (t,b,c) has flat index i = (t*B + b)*H + c;
                     its random word is word i & 3 of philox(counter = (i >> 2) as
                     a 128-bit little-endian number, key = seed as 64 bits); it is
                     kept iff word >= floor(p * 2^32), p taken as float32.
  adam_step          Algorithm 1 of Kingma and Ba with bias-corrected moments.

Readings where the paper is silent: the paper names the dropout rate only; it is
applied here to the attentional hidden state h~, the one place inside this part
of the model where the standard recipe for this architecture puts it.  No weight
decay, no gradient clipping (neither is mentioned).

Parity status: pinned (tests/test_train_extras_pins.py: the generator against the
published known-answer vectors of its reference implementation, keep rate and
independence statistics, Adam against closed forms and torch.optim.Adam in
float64, gradients with a fixed mask against central finite differences).
"""
from __future__ import annotations

import numpy as np

M0, M1 = 0xD2511F53, 0xCD9E8D57      # round multipliers
W0, W1 = 0x9E3779B9, 0xBB67AE85      # key increments (golden ratio, sqrt(3) - 1)
MASK32 = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    """ctr: uint64 array [..., 4] of 32-bit words, key: [..., 2].  Returns [..., 4] (uint64 holding 32-bit values)."""
    c = np.array(ctr, dtype=np.uint64) & np.uint64(MASK32)
    k = np.array(key, dtype=np.uint64) & np.uint64(MASK32)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = k[..., 0].copy(), k[..., 1].copy()
    for r in range(10):
        if r > 0:
            k0 = (k0 + np.uint64(W0)) & np.uint64(MASK32)
            k1 = (k1 + np.uint64(W1)) & np.uint64(MASK32)
        p0 = np.uint64(M0) * c0          # 32x32 -> 64 bit products (exact in uint64)
        p1 = np.uint64(M1) * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & np.uint64(MASK32)
        hi1, lo1 = p1 >> np.uint64(32), p1 & np.uint64(MASK32)
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return np.stack([c0, c1, c2, c3], axis=-1)


def dropout_threshold(p):
    """Words below this value drop the element.  p is rounded to float32 first."""
    p32 = float(np.float32(p))
    if not (0.0 <= p32 < 1.0):
        raise ValueError("dropout rate must be in [0, 1)")
    return int(np.floor(p32 * 4294967296.0))


def dropout_words(n_elems, seed):
    """The 32-bit random word of each of the first n_elems flat indices."""
    nq = (n_elems + 3) // 4
    q = np.arange(nq, dtype=np.uint64)
    ctr = np.zeros((nq, 4), np.uint64)
    ctr[:, 0] = q & np.uint64(MASK32)
    ctr[:, 1] = q >> np.uint64(32)
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    key = np.array([seed & MASK32, seed >> 32], np.uint64)
    return philox4x32_10(ctr, np.broadcast_to(key, (nq, 2))).reshape(-1)[:n_elems]


def dropout_multiplier(T, B, H, p, seed):
    """[T,B,H] float64: 0 where dropped, 1/(1-p) where kept (p as float32); all ones for p = 0."""
    p32 = float(np.float32(p))
    if p32 == 0.0:
        return np.ones((T, B, H), np.float64)
    keep = dropout_words(T * B * H, seed) >= np.uint64(dropout_threshold(p))
    return (keep.astype(np.float64) / (1.0 - p32)).reshape(T, B, H)


def adam_step(w, g, m, v, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam update (step = 1 for the first).  Returns new (w, m, v), float64."""
    w, g, m, v = (np.asarray(x, np.float64) for x in (w, g, m, v))
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    return w - lr * m_hat / (np.sqrt(v_hat) + eps), m, v
