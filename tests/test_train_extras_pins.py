"""Pins for the training-step extras of the oracle (no GPU): the dropout
generator, the dropout multiplier on h~ and its gradient, and Adam (paper
section 4.2, "Parameter settings", and Table 2)."""
import os

import numpy as np
import pytest
import torch

from oracle import attn_softmax_oracle as orc
from oracle import train_extras_oracle as tx
from synth_inputs import make_custom


# ------------------------------------------------------------------ generator
def test_philox_known_answers():
    path = os.path.join(os.path.dirname(__file__), "golden", "philox_known_answers.txt")
    n = 0
    with open(path) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if not line:
                continue
            w = [int(x, 16) for x in line]
            out = tx.philox4x32_10(np.array(w[0:4]), np.array(w[4:6]))
            assert [int(x) for x in out] == w[6:10]
            n += 1
    assert n == 3


def test_philox_is_a_bijection_of_the_counter_and_depends_on_every_input_word():
    base_c, base_k = np.array([1, 2, 3, 4]), np.array([5, 6])
    ref = tx.philox4x32_10(base_c, base_k)
    seen = {tuple(int(x) for x in ref)}
    for i in range(4):
        c = base_c.copy(); c[i] ^= 1
        o = tuple(int(x) for x in tx.philox4x32_10(c, base_k))
        assert o not in seen; seen.add(o)
    for i in range(2):
        k = base_k.copy(); k[i] ^= 1
        o = tuple(int(x) for x in tx.philox4x32_10(base_c, k))
        assert o not in seen; seen.add(o)
    # vectorised evaluation == one at a time
    ctr = np.arange(40, dtype=np.uint64).reshape(10, 4)
    key = np.tile(np.array([7, 9], np.uint64), (10, 1))
    allv = tx.philox4x32_10(ctr, key)
    for r in range(10):
        assert np.array_equal(allv[r], tx.philox4x32_10(ctr[r], key[r]))


def test_dropout_words_layout():
    """Element i takes word i & 3 of the block whose counter is i >> 2, key = the 64-bit seed."""
    seed = 0x0123456789ABCDEF
    w = tx.dropout_words(23, seed)
    for i in (0, 1, 5, 22):
        blk = tx.philox4x32_10(np.array([i >> 2, 0, 0, 0]), np.array([seed & 0xFFFFFFFF, seed >> 32]))
        assert int(w[i]) == int(blk[i & 3])
    # a prefix of a longer draw is the shorter draw (the mask of a batch shard does not depend on the batch)
    assert np.array_equal(tx.dropout_words(64, seed)[:23], w)


def test_dropout_multiplier_statistics_and_values():
    p = 0.3
    m = tx.dropout_multiplier(40, 16, 64, p, seed=11)
    vals = np.unique(m)
    assert len(vals) == 2 and vals[0] == 0.0
    assert vals[1] == pytest.approx(1.0 / (1.0 - float(np.float32(p))), rel=1e-15)
    keep = (m != 0).mean()
    n = m.size
    assert abs(keep - 0.7) < 5 * np.sqrt(0.21 / n)              # 5 sigma
    assert m.mean() == pytest.approx(1.0, abs=5 * np.sqrt(0.3 / 0.7 / n))   # inverted dropout keeps the mean
    # neighbouring elements are independent: joint keep rate ~ 0.49
    k = (m != 0).reshape(-1)
    assert abs((k[:-1] & k[1:]).mean() - 0.49) < 0.01
    # another seed gives another mask; p = 0 gives exactly ones; the threshold is floor(p32 * 2^32)
    assert (tx.dropout_multiplier(40, 16, 64, p, seed=12) != m).mean() > 0.3
    assert np.all(tx.dropout_multiplier(3, 2, 8, 0.0, seed=1) == 1.0)
    assert tx.dropout_threshold(0.5) == 1 << 31
    assert tx.dropout_threshold(0.3) == int(np.floor(float(np.float32(0.3)) * 2.0 ** 32))
    with pytest.raises(ValueError):
        tx.dropout_threshold(1.0)


# ------------------------------------------------- dropout inside the oracle
def _args(inp):
    return (inp.h_dec, inp.h_enc, inp.src_len, inp.W_a, inp.W_c, inp.W_out, inp.b_out,
            inp.targets, inp.pad_id)


def test_multiplier_of_ones_changes_nothing_and_zero_rows_see_only_the_bias():
    inp = make_custom(T=4, S=5, B=3, H=8, V=9, seed=21)
    f0 = orc.forward(*_args(inp))
    g0 = orc.backward(*_args(inp))
    ones = np.ones((inp.T, inp.B, inp.H))
    f1 = orc.forward(*_args(inp), drop=ones)
    g1 = orc.backward(*_args(inp), drop=ones)
    for k in ("logits", "h_c", "tok_loss"):
        assert np.array_equal(f0[k], f1[k])
    for k in g0:
        assert np.array_equal(g0[k], g1[k]), k
    # dropping a whole position leaves logits = b_out there and stops every gradient through it
    d = ones.copy(); d[2, 1, :] = 0.0
    f2 = orc.forward(*_args(inp), drop=d)
    assert np.allclose(f2["logits"][2, 1], inp.b_out.astype(np.float64), atol=0)
    assert np.all(f2["h_c"][2, 1] == 0)
    inp.targets[:] = np.where(np.arange(inp.T)[:, None] == 2, inp.targets, inp.pad_id)   # only step 2 counts
    inp.targets[2, 0] = inp.targets[2, 2] = inp.pad_id                                     # ... of sentence 1
    if inp.targets[2, 1] == inp.pad_id:
        inp.targets[2, 1] = 1
    g2 = orc.backward(*_args(inp), drop=d)
    for k in ("d_h_dec", "d_h_enc", "dW_a", "dW_c", "dW_out"):
        assert np.all(g2[k] == 0), k
    assert np.abs(g2["db_out"]).max() > 0


def test_scaling_h_tilde_equals_scaling_W_out():
    """A constant multiplier c on h~ is the same model as W_out scaled by c."""
    inp = make_custom(T=3, S=4, B=2, H=6, V=7, seed=22)
    c = 1.0 / 0.7
    drop = np.full((inp.T, inp.B, inp.H), c)
    a = list(_args(inp))
    f1 = orc.forward(*a, drop=drop)
    g1 = orc.backward(*a, drop=drop)
    a2 = list(a); a2[5] = inp.W_out.astype(np.float64) * c
    f2 = orc.forward(*a2)
    g2 = orc.backward(*a2)
    assert np.allclose(f1["logits"], f2["logits"], atol=1e-13)
    assert f1["loss_sum"] == pytest.approx(f2["loss_sum"], abs=1e-12)
    for k in ("d_h_dec", "d_h_enc", "dW_a", "dW_c", "db_out"):
        assert np.allclose(g1[k], g2[k], atol=1e-12), k
    assert np.allclose(g1["dW_out"], g2["dW_out"] * c, atol=1e-12)      # chain rule through the scaling


def test_central_finite_differences_with_a_fixed_mask():
    inp = make_custom(T=3, S=4, B=2, H=5, V=7, seed=33, w=0.6)
    inp.src_len[:] = [4, 2]
    inp.targets[1, 0] = inp.pad_id
    drop = tx.dropout_multiplier(inp.T, inp.B, inp.H, 0.3, seed=5)
    assert 0 < (drop == 0).sum() < drop.size
    base = [np.array(x, dtype=np.float64) for x in
            (inp.h_dec, inp.h_enc, inp.W_a, inp.W_c, inp.W_out, inp.b_out)]
    g = 0.6

    def loss_of(arrs):
        hd, he, wa, wc, wo, bo = arrs
        return orc.scaled_loss(hd, he, inp.src_len, wa, wc, wo, bo, inp.targets, inp.pad_id, g, drop=drop)

    hd, he, wa, wc, wo, bo = base
    grads = orc.backward(hd, he, inp.src_len, wa, wc, wo, bo, inp.targets, inp.pad_id, grad_scale=g, drop=drop)
    eps = 1e-6
    for idx, name in enumerate(["d_h_dec", "d_h_enc", "dW_a", "dW_c", "dW_out", "db_out"]):
        an = grads[name]
        num = np.zeros_like(an)
        it = np.nditer(base[idx], flags=["multi_index"])
        for _ in it:
            mi = it.multi_index
            old = base[idx][mi]
            base[idx][mi] = old + eps
            lp = loss_of(base)
            base[idx][mi] = old - eps
            lm = loss_of(base)
            base[idx][mi] = old
            num[mi] = (lp - lm) / (2 * eps)
        scale = max(np.abs(an).max(), 1e-3)
        assert np.abs(num - an).max() / scale < 1e-7, name


# ----------------------------------------------------------------------- Adam
def test_adam_first_step_and_constant_gradient_closed_forms():
    rng = np.random.default_rng(3)
    w0 = rng.normal(size=50)
    g = rng.normal(size=50)
    lr, eps = 1e-3, 1e-8
    w, m, v = tx.adam_step(w0, g, np.zeros(50), np.zeros(50), 1, lr=lr, eps=eps)
    # first step: m_hat = g, v_hat = g^2 -> a step of lr * g / (|g| + eps), whatever the betas
    assert np.allclose(w, w0 - lr * g / (np.abs(g) + eps), rtol=0, atol=1e-15)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)
    # a constant gradient keeps m_hat = g and v_hat = g^2 at every step
    for t in range(2, 12):
        w, m, v = tx.adam_step(w, g, m, v, t, lr=lr, eps=eps)
    assert np.allclose(w, w0 - 11 * lr * g / (np.abs(g) + eps), rtol=0, atol=1e-13)
    # zero gradient from the start: nothing moves
    w2, m2, v2 = tx.adam_step(w0, np.zeros(50), np.zeros(50), np.zeros(50), 1)
    assert np.array_equal(w2, w0) and not m2.any() and not v2.any()


def test_adam_matches_torch_optim_in_float64():
    rng = np.random.default_rng(4)
    w0 = rng.normal(size=(7, 5))
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t in range(1, 8):
        g = rng.normal(size=w0.shape) * (1.0 if t % 2 else 1e-3)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = tx.adam_step(w, g, m, v, t)
        assert np.allclose(w, p.detach().numpy(), rtol=0, atol=1e-14), t
