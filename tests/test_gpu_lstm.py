"""GPU parity of the stacked-LSTM entry points (lstm_stack_fwd / lstm_stack_bwd), called through the
C ABI, against the float64 oracle on the same seeded inputs.  Everything here needs an MI355X."""
import numpy as np
import pytest

import parity_util as pu
from oracle import lstm_stack_oracle as lo
from synth_inputs import make_lstm_inputs

pytestmark = pytest.mark.gpu


def _host(t):
    return t.detach().float().cpu().numpy()


def run_gpu(inp, use_states=True, **kw):
    import torch
    import paper_1909_00562_amd as lib
    d = lib.DeviceLstm(inp.x, inp.lengths, inp.W_ih, inp.W_hh, inp.b, inp.h0 if use_states else None,
                       inp.c0 if use_states else None, dtype=inp.dtype, dropout_p=getattr(inp, "dropout_p", 0.0),
                       dropout_seed=getattr(inp, "dropout_seed", 0), **kw)
    d.fwd()
    d.sync()
    f = dict(y=_host(d.y), hT=_host(d.hT), cT=_host(d.cT))
    dev = d.dev
    dy = torch.from_numpy(inp.dy).to(dev)
    dhT = torch.from_numpy(inp.dhT).to(dev) if use_states else None
    dcT = torch.from_numpy(inp.dcT).to(dev) if use_states else None
    d.bwd(dy, dhT, dcT)
    d.sync()
    g = dict(dx=_host(d.dx), dh0=_host(d.dh0), dc0=_host(d.dc0), dW_ih=[_host(t) for t in d.dW_ih],
             dW_hh=[_host(t) for t in d.dW_hh], db=[_host(t) for t in d.db])
    return f, g, d


def oracle_drop(inp):
    """Multipliers on the connections between the layers, [L-1, T, B, H] (None when dropout is off)."""
    p = getattr(inp, "dropout_p", 0.0)
    if p <= 0.0 or inp.L < 2:
        return None
    from oracle import train_extras_oracle as tx
    return tx.dropout_multiplier((inp.L - 1) * inp.T, inp.B, inp.H, p, inp.dropout_seed).reshape(
        inp.L - 1, inp.T, inp.B, inp.H)


def run_oracle(inp, use_states=True):
    fo = lo.forward(inp.x, inp.lengths, inp.W_ih, inp.W_hh, inp.b, inp.h0 if use_states else None,
                    inp.c0 if use_states else None, drop=oracle_drop(inp))
    go = lo.backward(fo, inp.dy, inp.dhT if use_states else None, inp.dcT if use_states else None)
    return fo, go


def compare(inp, f, g, fo, go, log=None):
    dt = inp.dtype
    valid = fo["valid"]
    assert np.all(f["y"][~valid] == 0.0), "output at padded steps"
    for k in ("y", "hT", "cT"):
        pu.assert_close(f[k], fo[k], dt, k, log)
    assert np.all(g["dx"][~valid] == 0.0), "dx at padded steps"
    for k in ("dx", "dh0", "dc0"):
        pu.assert_close(g[k], go[k], dt, k, log)
    for l in range(inp.L):
        for k in ("dW_ih", "dW_hh", "db"):
            pu.assert_close(g[k][l], go[k][l], dt, f"{k}[{l}]", log)


SHAPES = [
    # T, B, I, H, L
    (1, 1, 8, 8, 1),
    (6, 4, 24, 16, 3),
    (9, 5, 72, 40, 2),          # ragged against every tile edge
    (20, 32, 64, 128, 4),
    (7, 130, 40, 264, 2),       # more sentences than one 128-row tile
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_lstm_parity(shape, dtype):
    T, B, I, H, L = shape
    inp = make_lstm_inputs(T, B, I, H, L, seed=500 + T + B + H, dtype=dtype)
    f, g, _ = run_gpu(inp)
    fo, go = run_oracle(inp)
    compare(inp, f, g, fo, go)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_lstm_zero_length_sentences_and_default_states(dtype):
    inp = make_lstm_inputs(8, 6, 16, 24, 2, seed=77, dtype=dtype)
    inp.lengths[:] = [8, 0, 3, 12, -2, 1]                 # clamped to [0, T]
    f, g, _ = run_gpu(inp, use_states=False)
    fo, go = run_oracle(inp, use_states=False)
    compare(inp, f, g, fo, go)
    assert np.all(f["hT"][:, 1] == 0) and np.all(f["cT"][:, 4] == 0)      # never stepped: the zero initial state
    inp2 = make_lstm_inputs(8, 6, 16, 24, 2, seed=77, dtype=dtype)
    inp2.lengths[:] = [8, 0, 3, 12, -2, 1]
    f2, g2, _ = run_gpu(inp2)
    assert np.array_equal(f2["hT"][:, 1], inp2.h0[:, 1]) and np.array_equal(g2["dh0"][:, 4], inp2.dhT[:, 4])


def test_lstm_two_runs_are_bit_identical():
    inp = make_lstm_inputs(12, 16, 64, 64, 3, seed=5, dtype="bf16")
    f1, g1, _ = run_gpu(inp)
    f2, g2, _ = run_gpu(inp)
    for k in f1:
        assert np.array_equal(f1[k], f2[k]), k
    for k in ("dx", "dh0", "dc0"):
        assert np.array_equal(g1[k], g2[k]), k
    for l in range(inp.L):
        for k in ("dW_ih", "dW_hh", "db"):
            assert np.array_equal(g1[k][l], g2[k][l]), (k, l)


def test_lstm_paper_size_sixteen_sentences():
    """Table 2's model (embedding 512, hidden 1024, depth 4) at 50 steps, a batch of 16 sentences:
    everything, including the weight gradients, against the oracle."""
    inp = make_lstm_inputs(50, 16, 512, 1024, 4, seed=1909, dtype="bf16", min_len=20)
    f, g, _ = run_gpu(inp)
    fo, go = run_oracle(inp)
    log = {}
    compare(inp, f, g, fo, go, log)
    print({k: (round(v["ratio"], 3), float(f"{v['norm']:.2e}")) for k, v in log.items()})


def test_lstm_paper_size_full_batch():
    """The configuration bench.py times (B = 128 at Table 2's size): every output and every gradient of the
    whole batch, weight gradients included, against the oracle run on the whole batch; the weight gradients of
    the batch must also equal the sum over 4 shards (fp32 summation order only)."""
    T, B, I, H, L = 50, 128, 512, 1024, 4
    inp = make_lstm_inputs(T, B, I, H, L, seed=50, dtype="bf16", min_len=20)
    f, g, _ = run_gpu(inp)
    fo, go = run_oracle(inp)
    compare(inp, f, g, fo, go)
    del fo, go
    acc = {k: [np.zeros_like(a, dtype=np.float64) for a in g[k]] for k in ("dW_ih", "dW_hh", "db")}
    q = B // 4
    for i in range(4):
        sl = slice(i * q, (i + 1) * q)
        sh = make_lstm_inputs(T, B, I, H, L, seed=50, dtype="bf16", min_len=20)
        sh.B = q
        sh.x, sh.lengths, sh.dy = inp.x[:, sl].copy(), inp.lengths[sl].copy(), inp.dy[:, sl].copy()
        sh.h0, sh.c0, sh.dhT, sh.dcT = (a[:, sl].copy() for a in (inp.h0, inp.c0, inp.dhT, inp.dcT))
        fs, gs, _ = run_gpu(sh)
        assert np.array_equal(fs["y"], f["y"][:, sl])           # a sentence does not see the batch around it
        for k in acc:
            for l in range(L):
                acc[k][l] += gs[k][l]
    for k in acc:
        for l in range(L):
            s = pu.err_stats(acc[k][l], g[k][l], "bf16")
            assert s["norm"] <= 5e-4, (k, l, s)


def test_encoder_decoder_attention_chain_fp32():
    """The interfaces fit: encoder LSTM -> decoder LSTM (initial state = the encoder's final state) ->
    attention-softmax forward/backward -> decoder backward -> encoder backward (which also receives the
    gradient of the decoder's initial state), fp32 storage, against the two oracles chained the same way."""
    import torch
    import paper_1909_00562_amd as lib
    from oracle import attn_softmax_oracle as orc
    from synth_inputs import make_custom
    S, T, B, I, H, L, V = 7, 6, 4, 12, 16, 2, 53
    enc_in = make_lstm_inputs(S, B, I, H, L, seed=31, dtype="f32")
    dec_in = make_lstm_inputs(T, B, I, H, L, seed=32, dtype="f32")
    att = make_custom(T=T, S=S, B=B, H=H, V=V, seed=33, dtype="f32", min_len=1)
    att.src_len = enc_in.lengths.copy()
    for b in range(B):                       # targets are padding exactly where the decoder's sentence has ended
        att.targets[:, b] = np.where(np.arange(T) < dec_in.lengths[b], np.maximum(att.targets[:, b], 1), att.pad_id)

    # oracle chain
    eo = lo.forward(enc_in.x, enc_in.lengths, enc_in.W_ih, enc_in.W_hh, enc_in.b)
    do = lo.forward(dec_in.x, dec_in.lengths, dec_in.W_ih, dec_in.W_hh, dec_in.b, eo["hT"], eo["cT"])
    args = (do["y"], eo["y"], att.src_len, att.W_a, att.W_c, att.W_out, att.b_out, att.targets, att.pad_id)
    fo = orc.forward(*args)
    go = orc.backward(*args, grad_scale=1.0)
    dgo = lo.backward(do, go["d_h_dec"])
    ego = lo.backward(eo, go["d_h_enc"], dgo["dh0"], dgo["dc0"])

    # GPU chain: device tensors handed from one entry point to the next
    enc = lib.DeviceLstm(enc_in.x, enc_in.lengths, enc_in.W_ih, enc_in.W_hh, enc_in.b, dtype="f32")
    dec = lib.DeviceLstm(dec_in.x, dec_in.lengths, dec_in.W_ih, dec_in.W_hh, dec_in.b, dtype="f32")
    enc.fwd()
    dec.h0, dec.c0 = enc.hT, enc.cT
    dec.fwd()
    db = lib.DeviceBatch(att)
    db.h_dec, db.h_enc = dec.y, enc.y
    db.fwd()
    db.bwd()
    dec.bwd(db.d_h_dec)
    enc.bwd(db.d_h_enc, dec.dh0, dec.dc0)
    enc.sync()
    assert int(db.n_tok.item()) == fo["n_tok"]
    assert abs(float(db.loss_sum.item()) - fo["loss_sum"]) <= 1e-4 * abs(fo["loss_sum"])
    pu.assert_close(_host(dec.dx), dgo["dx"], "f32", "decoder dx")
    pu.assert_close(_host(enc.dx), ego["dx"], "f32", "encoder dx")
    for l in range(L):
        pu.assert_close(_host(dec.dW_hh[l]), dgo["dW_hh"][l], "f32", f"decoder dW_hh[{l}]")
        pu.assert_close(_host(enc.dW_ih[l]), ego["dW_ih"][l], "f32", f"encoder dW_ih[{l}]")
        pu.assert_close(_host(enc.db[l]), ego["db"][l], "f32", f"encoder db[{l}]")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(6, 4, 24, 16, 3), (9, 5, 72, 40, 2), (20, 32, 64, 128, 4)])
def test_lstm_dropout_between_layers(shape, dtype):
    """Same words of the generator on both sides (the decision is integer work): with them every tensor
    agrees to the usual tolerance, and the run differs from the one without dropout."""
    T, B, I, H, L = shape
    inp = make_lstm_inputs(T, B, I, H, L, seed=900 + T + H, dtype=dtype)
    inp.dropout_p, inp.dropout_seed = 0.3, 20190900562 + T
    f, g, _ = run_gpu(inp)
    fo, go = run_oracle(inp)
    compare(inp, f, g, fo, go)
    plain = make_lstm_inputs(T, B, I, H, L, seed=900 + T + H, dtype=dtype)
    fp, _, _ = run_gpu(plain)
    assert not np.array_equal(fp["y"], f["y"])
    # rate 0 with a seed set is the same as no dropout, bit for bit
    zero = make_lstm_inputs(T, B, I, H, L, seed=900 + T + H, dtype=dtype)
    zero.dropout_p, zero.dropout_seed = 0.0, 77
    fz, gz, _ = run_gpu(zero)
    assert np.array_equal(fz["y"], fp["y"])


def test_lstm_dropout_paper_size_sixteen_sentences():
    inp = make_lstm_inputs(50, 16, 512, 1024, 4, seed=1910, dtype="bf16", min_len=20)
    inp.dropout_p, inp.dropout_seed = 0.3, 5
    f, g, _ = run_gpu(inp)
    fo, go = run_oracle(inp)
    compare(inp, f, g, fo, go)
