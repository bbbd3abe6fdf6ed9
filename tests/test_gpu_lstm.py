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
                       inp.c0 if use_states else None, dtype=inp.dtype, **kw)
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


def run_oracle(inp, use_states=True):
    fo = lo.forward(inp.x, inp.lengths, inp.W_ih, inp.W_hh, inp.b, inp.h0 if use_states else None,
                    inp.c0 if use_states else None)
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
