"""GPU parity of the training-step extras (dropout on the attentional state, Adam;
paper section 4.2) against the float64 oracle, through the C ABI."""
import copy

import numpy as np
import pytest

import parity_util as pu
from synth_inputs import make_custom, make_inputs

pytestmark = pytest.mark.gpu


def _with_dropout(inp, p=0.3, seed=0x5EED5EED1234):
    inp = copy.copy(inp)
    inp.dropout_p, inp.dropout_seed = p, seed
    return inp


def _check_mask_bits(f, inp):
    """The kept/dropped decision is integer work: exact."""
    drop = pu.oracle_drop(inp)
    got_zero = f["h_c"] == 0.0
    assert np.array_equal(got_zero, drop == 0.0), "dropout mask differs from the oracle's"


@pytest.mark.parametrize("name,dtype", [("tiny", "f32"), ("small", "f32"), ("small", "bf16")])
def test_dropout_parity(name, dtype):
    inp = _with_dropout(make_inputs(name, dtype=dtype))
    run = pu.GpuRun(inp)
    f, g = run.fwd(), run.bwd()
    fo, go = pu.run_oracle(inp)
    _check_mask_bits(f, inp)
    pu.compare_all(f, g, fo, go, inp.dtype, {})
    kept = (f["h_c"] != 0).mean()
    assert abs(kept - 0.7) < 0.02


@pytest.mark.parametrize("T,S,B,H,V,dtype", [
    (3, 5, 2, 6, 11, "f32"),        # H % 4 != 0: element-wise generator path
    (5, 7, 3, 24, 53, "f32"),
    (37, 45, 5, 136, 1003, "bf16"), # several tiles, ragged rows
    (1, 9, 7, 264, 300, "bf16"),    # one decoder step
])
def test_dropout_edge_shapes(T, S, B, H, V, dtype):
    inp = _with_dropout(make_custom(T=T, S=S, B=B, H=H, V=V, seed=400 + H, dtype=dtype), p=0.5, seed=77)
    run = pu.GpuRun(inp)
    f, g = run.fwd(), run.bwd()
    fo, go = pu.run_oracle(inp)
    _check_mask_bits(f, inp)
    pu.compare_all(f, g, fo, go, inp.dtype, {})


def test_dropout_switches_and_seeds():
    base = make_inputs("small", dtype="bf16")
    f0 = pu.GpuRun(base).fwd()
    # rate 0 with a seed set == no dropout, bit for bit
    fz = pu.GpuRun(_with_dropout(base, p=0.0, seed=123)).fwd()
    assert np.array_equal(f0["logits"], fz["logits"]) and f0["loss_sum"] == fz["loss_sum"]
    # same seed: same bits, forward and backward; another seed: another mask
    a = pu.GpuRun(_with_dropout(base, seed=1)); fa, ga = a.fwd(), a.bwd()
    b = pu.GpuRun(_with_dropout(base, seed=1)); fb, gb = b.fwd(), b.bwd()
    assert np.array_equal(fa["h_c"], fb["h_c"]) and fa["loss_sum"] == fb["loss_sum"]
    for k in ga:
        assert np.array_equal(ga[k], gb[k]), k
    fc = pu.GpuRun(_with_dropout(base, seed=2)).fwd()
    assert ((fa["h_c"] == 0) != (fc["h_c"] == 0)).mean() > 0.3
    # invalid rate is refused by the library
    import paper_1909_00562_amd as lib
    with pytest.raises(lib.AttnSoftmaxError):
        pu.GpuRun(_with_dropout(base, p=1.0))


def test_dropout_full_size_stress_sampled():
    """Stress shape as the benchmark launches it, dropout on: sampled sentences against the oracle."""
    inp = _with_dropout(make_inputs("stress"))
    idx = [0, 17, 128, 255]
    drop = pu.oracle_drop(inp)
    from oracle import attn_softmax_oracle as orc
    fo = orc.forward(*pu.oracle_args(inp), sentences=idx, drop=drop)
    go = orc.backward(*pu.oracle_args(inp), grad_scale=inp.grad_scale, sentences=idx, drop=drop)
    run = pu.GpuRun(inp)
    f = run.fwd(sentences=idx)
    m = fo["tgt_mask"][:, idx].astype(bool)
    assert np.array_equal(f["h_c"] == 0.0, drop[:, idx] == 0.0)
    for k in ("h_c", "lse", "logits"):
        pu.assert_close(f[k][m], fo[k][:, idx][m], inp.dtype, k)
    pu.assert_close(f["tok_loss"], fo["tok_loss"][:, idx], inp.dtype, "tok_loss")
    g = run.bwd(sentences=idx)
    pu.assert_close(g["d_h_dec"], go["d_h_dec"][:, idx], inp.dtype, "d_h_dec")
    pu.assert_close(g["d_h_enc"], go["d_h_enc"][:, idx], inp.dtype, "d_h_enc")


# ----------------------------------------------------------------------- Adam
def _adam_case(n, dtype, steps=3, seed=9):
    import torch
    import paper_1909_00562_amd as lib
    from oracle import train_extras_oracle as tx
    rng = np.random.default_rng(seed)
    w0 = rng.uniform(-0.1, 0.1, n).astype(np.float32)
    dev = "cuda:0"
    master = torch.from_numpy(w0.copy()).to(dev)
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    wout = torch.zeros(n, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=dev)
    wo, mo, vo = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    # hyper-parameters as the float32 values the C ABI carries
    lr, b1, b2, eps = (float(np.float32(x)) for x in (1e-3, 0.9, 0.999, 1e-8))
    for t in range(1, steps + 1):
        scale = [1.0, 1e-4, 30.0][t % 3]                     # gradient magnitudes across steps
        g = (rng.normal(size=n) * scale).astype(np.float32)
        g[::97] = 0.0
        hp = lib.AsAdam(lr, b1, b2, eps, t)
        lib.attn_softmax_adam_step(hp, n, torch.from_numpy(g).to(dev), master, m, v, wout,
                                   lib.AS_BF16 if dtype == "bf16" else lib.AS_F32)
        torch.cuda.synchronize()
        # the oracle steps from the state the GPU held before this step (fp32 values, fp64 arithmetic)
        m_prev, v_prev = mo, vo
        wo, mo, vo = tx.adam_step(wo, g, mo, vo, t, lr=lr, beta1=b1, beta2=b2, eps=eps)
        gw, gm, gv = master.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()
        # fp32: each moment is a sum of two rounded products (a few units of 2^-24 of the larger term)
        g64 = g.astype(np.float64)
        assert np.all(np.abs(gm - mo) <= 2e-7 * (np.abs(m_prev) + np.abs(g64)) + 1e-37), ("m", t)
        assert np.all(np.abs(gv - vo) <= 2e-7 * (np.abs(v_prev) + g64 * g64) + 1e-37), ("v", t)
        # fp32 arithmetic: a few ulp of the step (<= lr) plus the rounding of w itself
        assert np.all(np.abs(gw - wo) <= 1.2e-7 * np.abs(wo) + 1e-5 * lr), ("w", t, np.abs(gw - wo).max())
        if dtype == "bf16":   # the storage copy is the rounded master, exactly
            expect = master.to(torch.bfloat16)
            assert torch.equal(wout, expect)
        else:
            assert torch.equal(wout, master)
        wo, mo, vo = gw.astype(np.float64), gm.astype(np.float64), gv.astype(np.float64)


@pytest.mark.parametrize("n,dtype", [(1, "f32"), (7, "bf16"), (4096, "bf16"), (1000003, "bf16"), (262147, "f32")])
def test_adam_step_parity(n, dtype):
    _adam_case(n, dtype)


def test_adam_rejects_bad_arguments():
    import torch
    import paper_1909_00562_amd as lib
    x = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    for hp in (lib.AsAdam(1e-3, 0.9, 0.999, 1e-8, 0), lib.AsAdam(1e-3, 1.0, 0.999, 1e-8, 1)):
        with pytest.raises(lib.AttnSoftmaxError):
            lib.attn_softmax_adam_step(hp, 16, x, x, x, x, None, lib.AS_F32)
    with pytest.raises(lib.AttnSoftmaxError):
        lib.attn_softmax_adam_step(lib.AsAdam(1e-3, 0.9, 0.999, 1e-8, 1), 16, None, x, x, x, None, lib.AS_F32)


def test_training_steps_reduce_the_loss():
    """fwd + bwd + Adam on the four parameter tensors, a few steps on one batch: the loss falls."""
    import torch
    import paper_1909_00562_amd as lib
    inp = _with_dropout(make_inputs("tiny"), p=0.3, seed=5)
    db = lib.DeviceBatch(inp)
    params = [("W_a", "dW_a"), ("W_c", "dW_c"), ("W_out", "dW_out"), ("b_out", "db_out")]
    state = {p: (getattr(db, p).float().clone().contiguous(), torch.zeros_like(getattr(db, p), dtype=torch.float32),
                 torch.zeros_like(getattr(db, p), dtype=torch.float32)) for p, _ in params}
    losses = []
    for t in range(1, 9):
        db.shape.dropout_seed = 1000 + t
        db.fwd(); db.bwd(); db.sync()
        losses.append(float(db.loss_sum.item()))
        for p, gname in params:
            master, m, v = state[p]
            lib.attn_softmax_adam_step(lib.AsAdam(1e-2, 0.9, 0.999, 1e-8, t), master.numel(), getattr(db, gname),
                                       master, m, v, getattr(db, p), lib.AS_F32)
        db.sync()
    assert losses[-1] < 0.9 * losses[0], losses
