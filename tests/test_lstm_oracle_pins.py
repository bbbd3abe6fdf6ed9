"""Pins of the stacked-LSTM oracle (CPU only): a library routine that was written by others
(torch.nn.LSTM in float64 on packed sequences, values and autograd gradients), closed forms,
invariants of the padding rule, and central finite differences on every gradient."""
import math

import numpy as np
import pytest
import torch

from oracle import lstm_stack_oracle as lo


def _params(rng, L, I0, H, w=0.4):
    W_ih = [rng.uniform(-w, w, (4 * H, I0 if l == 0 else H)) for l in range(L)]
    W_hh = [rng.uniform(-w, w, (4 * H, H)) for l in range(L)]
    b = [rng.uniform(-w, w, 4 * H) for l in range(L)]
    return W_ih, W_hh, b


def _case(seed=0, T=6, B=4, I0=3, H=5, L=3, lengths=None):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, B, I0))
    if lengths is None:
        lengths = rng.integers(1, T + 1, size=B)
        lengths[0] = T
    W_ih, W_hh, b = _params(rng, L, I0, H)
    h0 = rng.standard_normal((L, B, H)) * 0.5
    c0 = rng.standard_normal((L, B, H)) * 0.5
    return x, np.asarray(lengths), W_ih, W_hh, b, h0, c0, rng


def _scalar(fwd, R, Rh, Rc):
    return float((fwd["y"] * R).sum() + (fwd["hT"] * Rh).sum() + (fwd["cT"] * Rc).sum())


# ------------------------------------------------------------------ library routine
@pytest.mark.parametrize("L", [1, 3])
def test_matches_torch_lstm_on_packed_sequences(L):
    x, lengths, W_ih, W_hh, b, h0, c0, rng = _case(seed=3, L=L)
    T, B, I0 = x.shape
    H = W_hh[0].shape[1]
    net = torch.nn.LSTM(I0, H, num_layers=L).double()
    with torch.no_grad():
        for l in range(L):
            getattr(net, f"weight_ih_l{l}").copy_(torch.from_numpy(W_ih[l]))
            getattr(net, f"weight_hh_l{l}").copy_(torch.from_numpy(W_hh[l]))
            getattr(net, f"bias_ih_l{l}").copy_(torch.from_numpy(b[l] * 0.25))      # the cell adds the two biases
            getattr(net, f"bias_hh_l{l}").copy_(torch.from_numpy(b[l] * 0.75))
    xt = torch.from_numpy(x).requires_grad_(True)
    h0t = torch.from_numpy(h0).requires_grad_(True)
    c0t = torch.from_numpy(c0).requires_grad_(True)
    packed = torch.nn.utils.rnn.pack_padded_sequence(xt, torch.from_numpy(lengths), enforce_sorted=False)
    out, (hn, cn) = net(packed, (h0t, c0t))
    y, _ = torch.nn.utils.rnn.pad_packed_sequence(out, total_length=T)
    f = lo.forward(x, lengths, W_ih, W_hh, b, h0, c0)
    assert np.allclose(f["y"], y.detach().numpy(), atol=1e-12)
    assert np.allclose(f["hT"], hn.detach().numpy(), atol=1e-12)
    assert np.allclose(f["cT"], cn.detach().numpy(), atol=1e-12)
    R, Rh, Rc = rng.standard_normal(f["y"].shape), rng.standard_normal(h0.shape), rng.standard_normal(c0.shape)
    loss = (y * torch.from_numpy(R)).sum() + (hn * torch.from_numpy(Rh)).sum() + (cn * torch.from_numpy(Rc)).sum()
    loss.backward()
    g = lo.backward(f, R, Rh, Rc)
    assert np.allclose(g["dx"], xt.grad.numpy(), atol=1e-11)
    assert np.allclose(g["dh0"], h0t.grad.numpy(), atol=1e-11)
    assert np.allclose(g["dc0"], c0t.grad.numpy(), atol=1e-11)
    for l in range(L):
        assert np.allclose(g["dW_ih"][l], getattr(net, f"weight_ih_l{l}").grad.numpy(), atol=1e-11)
        assert np.allclose(g["dW_hh"][l], getattr(net, f"weight_hh_l{l}").grad.numpy(), atol=1e-11)
        assert np.allclose(g["db"][l], getattr(net, f"bias_ih_l{l}").grad.numpy(), atol=1e-11)
        assert np.allclose(g["db"][l], getattr(net, f"bias_hh_l{l}").grad.numpy(), atol=1e-11)


# ------------------------------------------------------------------ closed forms
def test_zero_parameters_give_zero_states():
    T, B, I0, H = 5, 2, 3, 4
    x = np.random.default_rng(0).standard_normal((T, B, I0))
    z = lambda *s: np.zeros(s)
    f = lo.forward(x, [T, T], [z(4 * H, I0), z(4 * H, H)], [z(4 * H, H)] * 2, [z(4 * H)] * 2)
    # i = f = o = 1/2, g = 0: c stays 0, h = 0
    assert np.all(f["y"] == 0) and np.all(f["hT"] == 0) and np.all(f["cT"] == 0)


def test_bias_only_cell_follows_the_geometric_series():
    """W = 0: every unit runs c_t = s_f c_{t-1} + s_i tanh(b_g) from c_0 = 0, a geometric series."""
    T, H = 7, 3
    bi, bf, bg, bo = 0.3, -0.2, 0.9, 0.5
    b = np.concatenate([np.full(H, bi), np.full(H, bf), np.full(H, bg), np.full(H, bo)])
    f = lo.forward(np.zeros((T, 1, 2)), [T], [np.zeros((4 * H, 2))], [np.zeros((4 * H, H))], [b])
    sig = lambda a: 1.0 / (1.0 + math.exp(-a))
    for t in range(T):
        c = sig(bi) * math.tanh(bg) * (1.0 - sig(bf) ** (t + 1)) / (1.0 - sig(bf))
        assert np.allclose(f["y"][t], sig(bo) * math.tanh(c), atol=1e-14)
    assert np.allclose(f["cT"], c, atol=1e-14)


def test_saturated_gates_copy_the_candidate():
    """Input gate open, forget gate shut, output gate open: h_t = tanh(tanh(w x_t))."""
    T, H = 4, 2
    big = 60.0
    b = np.concatenate([np.full(H, big), np.full(H, -big), np.zeros(H), np.full(H, big)])
    W = np.zeros((4 * H, 1))
    W[2 * H:3 * H, 0] = [0.7, -1.3]
    x = np.array([0.5, -1.0, 2.0, 0.1]).reshape(T, 1, 1)
    f = lo.forward(x, [T], [W], [np.zeros((4 * H, H))], [b])
    expect = np.tanh(np.tanh(x[:, 0, :] * np.array([0.7, -1.3])))
    assert np.allclose(f["y"][:, 0], expect, atol=1e-13)


# ------------------------------------------------------------------ padding rule
def test_padded_steps_keep_the_state_and_output_zero():
    x, lengths, W_ih, W_hh, b, h0, c0, rng = _case(seed=5, lengths=[6, 3, 1, 0])
    f = lo.forward(x, lengths, W_ih, W_hh, b, h0, c0)
    for bb, n in enumerate(lengths):
        assert np.all(f["y"][n:, bb] == 0)
        # the final state is that of the sentence run alone at its true length
        if n > 0:
            alone = lo.forward(x[:n, bb:bb + 1], [n], W_ih, W_hh, b, h0[:, bb:bb + 1], c0[:, bb:bb + 1])
            assert np.allclose(f["hT"][:, bb], alone["hT"][:, 0], atol=1e-14)
            assert np.allclose(f["cT"][:, bb], alone["cT"][:, 0], atol=1e-14)
            assert np.allclose(f["y"][:n, bb], alone["y"][:, 0], atol=1e-14)
        else:
            assert np.array_equal(f["hT"][:, bb], h0[:, bb]) and np.array_equal(f["cT"][:, bb], c0[:, bb])


def test_padded_inputs_do_not_matter_and_get_zero_gradient():
    x, lengths, W_ih, W_hh, b, h0, c0, rng = _case(seed=6, lengths=[6, 2, 4, 1])
    R, Rh, Rc = rng.standard_normal((6, 4, 5)), rng.standard_normal(h0.shape), rng.standard_normal(c0.shape)
    f = lo.forward(x, lengths, W_ih, W_hh, b, h0, c0)
    g = lo.backward(f, R, Rh, Rc)
    x2 = x.copy()
    for bb, n in enumerate(lengths):
        x2[n:, bb] = 1e3 * rng.standard_normal(x2[n:, bb].shape)
        assert np.all(g["dx"][n:, bb] == 0)
    f2 = lo.forward(x2, lengths, W_ih, W_hh, b, h0, c0)
    g2 = lo.backward(f2, R, Rh, Rc)
    assert np.array_equal(f["y"], f2["y"]) and np.array_equal(f["hT"], f2["hT"])
    for l in range(3):
        assert np.allclose(g["dW_ih"][l], g2["dW_ih"][l], atol=1e-12)


# ------------------------------------------------------------------ structure
def test_two_chunks_with_the_state_handed_over_equal_one_run():
    x, lengths, W_ih, W_hh, b, h0, c0, _ = _case(seed=7, lengths=[6, 6, 6, 6])
    f = lo.forward(x, lengths, W_ih, W_hh, b, h0, c0)
    a = lo.forward(x[:2], [2] * 4, W_ih, W_hh, b, h0, c0)
    c = lo.forward(x[2:], [4] * 4, W_ih, W_hh, b, a["hT"], a["cT"])
    assert np.allclose(np.concatenate([a["y"], c["y"]]), f["y"], atol=1e-14)
    assert np.allclose(c["hT"], f["hT"], atol=1e-14) and np.allclose(c["cT"], f["cT"], atol=1e-14)


def test_weight_gradients_add_over_the_batch():
    x, lengths, W_ih, W_hh, b, h0, c0, rng = _case(seed=8)
    R, Rh, Rc = rng.standard_normal((6, 4, 5)), rng.standard_normal(h0.shape), rng.standard_normal(c0.shape)
    g = lo.backward(lo.forward(x, lengths, W_ih, W_hh, b, h0, c0), R, Rh, Rc)
    acc = [np.zeros_like(w) for w in g["dW_hh"]]
    for s in (slice(0, 1), slice(1, 4)):
        gs = lo.backward(lo.forward(x[:, s], lengths[s], W_ih, W_hh, b, h0[:, s], c0[:, s]), R[:, s], Rh[:, s], Rc[:, s])
        for l in range(3):
            acc[l] += gs["dW_hh"][l]
        assert np.allclose(gs["dx"], g["dx"][:, s], atol=1e-13)
    for l in range(3):
        assert np.allclose(acc[l], g["dW_hh"][l], atol=1e-12)


# ------------------------------------------------------------------ finite differences
def test_every_gradient_matches_central_differences():
    x, lengths, W_ih, W_hh, b, h0, c0, rng = _case(seed=11, T=4, B=3, I0=2, H=3, L=2, lengths=[4, 2, 3])
    R = rng.standard_normal((4, 3, 3))
    Rh, Rc = rng.standard_normal(h0.shape), rng.standard_normal(c0.shape)
    g = lo.backward(lo.forward(x, lengths, W_ih, W_hh, b, h0, c0), R, Rh, Rc)
    eps = 1e-6

    def numeric(arr):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            k = it.multi_index
            old = arr[k]
            arr[k] = old + eps
            up = _scalar(lo.forward(x, lengths, W_ih, W_hh, b, h0, c0), R, Rh, Rc)
            arr[k] = old - eps
            dn = _scalar(lo.forward(x, lengths, W_ih, W_hh, b, h0, c0), R, Rh, Rc)
            arr[k] = old
            out[k] = (up - dn) / (2 * eps)
        return out

    checks = [("dx", x, g["dx"]), ("dh0", h0, g["dh0"]), ("dc0", c0, g["dc0"])]
    for l in range(2):
        checks += [(f"dW_ih{l}", W_ih[l], g["dW_ih"][l]), (f"dW_hh{l}", W_hh[l], g["dW_hh"][l]), (f"db{l}", b[l], g["db"][l])]
    for name, arr, an in checks:
        nu = numeric(arr)
        err = np.abs(nu - an).max() / max(1.0, np.abs(an).max())
        assert err < 1e-7, (name, err)


# ------------------------------------------------------------------ dropout between the layers
def test_dropout_of_ones_changes_nothing_and_a_fixed_mask_matches_central_differences():
    x, lengths, W_ih, W_hh, b, h0, c0, rng = _case(seed=21, T=4, B=3, I0=2, H=3, L=3, lengths=[4, 2, 3])
    R = rng.standard_normal((4, 3, 3))
    Rh, Rc = rng.standard_normal(h0.shape), rng.standard_normal(c0.shape)
    plain = lo.forward(x, lengths, W_ih, W_hh, b, h0, c0)
    ones = lo.forward(x, lengths, W_ih, W_hh, b, h0, c0, drop=np.ones((2, 4, 3, 3)))
    assert np.array_equal(plain["y"], ones["y"]) and np.array_equal(plain["cT"], ones["cT"])
    drop = (rng.random((2, 4, 3, 3)) < 0.6) / 0.6            # a fixed mask with keep rate 0.6
    f = lo.forward(x, lengths, W_ih, W_hh, b, h0, c0, drop=drop)
    assert not np.allclose(f["y"], plain["y"])
    g = lo.backward(f, R, Rh, Rc)
    eps = 1e-6
    for name, arr, an in [("dx", x, g["dx"]), ("dW_hh0", W_hh[0], g["dW_hh"][0]), ("dW_ih1", W_ih[1], g["dW_ih"][1]),
                          ("db2", b[2], g["db"][2]), ("dh0", h0, g["dh0"])]:
        nu = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            k = it.multi_index
            old = arr[k]
            arr[k] = old + eps
            up = _scalar(lo.forward(x, lengths, W_ih, W_hh, b, h0, c0, drop=drop), R, Rh, Rc)
            arr[k] = old - eps
            dn = _scalar(lo.forward(x, lengths, W_ih, W_hh, b, h0, c0, drop=drop), R, Rh, Rc)
            arr[k] = old
            nu[k] = (up - dn) / (2 * eps)
        err = np.abs(nu - an).max() / max(1.0, np.abs(an).max())
        assert err < 1e-7, (name, err)


def test_a_fully_dropped_layer_output_cuts_the_stack():
    """All of layer 0's outputs dropped: the layers above see zeros, and nothing below receives gradient
    from the top layer's outputs."""
    x, lengths, W_ih, W_hh, b, h0, c0, rng = _case(seed=22, T=5, B=2, I0=3, H=4, L=2, lengths=[5, 3])
    drop = np.zeros((1, 5, 2, 4))
    f = lo.forward(x, lengths, W_ih, W_hh, b, h0, c0, drop=drop)
    alone = lo.forward(np.zeros((5, 2, 4)), lengths, W_ih[1:], W_hh[1:], b[1:], h0[1:], c0[1:])
    assert np.allclose(f["y"], alone["y"], atol=1e-15)
    g = lo.backward(f, rng.standard_normal((5, 2, 4)))
    assert np.all(g["dx"] == 0) and np.all(g["dW_ih"][0] == 0) and np.all(g["dW_hh"][0] == 0)
