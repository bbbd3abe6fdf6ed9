"""GPU parity: the HIP library, called through its C ABI, against the float64
oracle on the same seeded inputs.  Everything here needs an MI355X."""
import numpy as np
import pytest

import parity_util as pu
from synth_inputs import make_custom, make_inputs

pytestmark = pytest.mark.gpu


SKIP = pytest.mark.parametrize("skip", [False, True], ids=["all_rows", "skip_pad_rows"])


def _full_parity(inp, dlogits=False, skip=False):
    """skip: row compaction (as_shape.skip_pad_rows), the mode the benchmark times."""
    run = pu.GpuRun(inp, skip_pad_rows=skip)
    f = run.fwd()
    g = run.bwd(dlogits=dlogits)
    fo, go = pu.run_oracle(inp, keep_dlogits=dlogits)
    log = {}
    pu.compare_all(f, g, fo, go, inp.dtype, log, pad_rows_hold=inp.pad_id if skip else None)
    if dlogits:
        m = fo["tgt_mask"].astype(bool)
        pu.assert_close(g["dlogits"], go["dlogits"], inp.dtype, "dlogits", log)
        assert np.all(g["dlogits"][~m] == 0.0)
        atol, rtol = pu.TOL[inp.dtype]
        rows = np.abs(g["dlogits"].astype(np.float64).sum(axis=-1))
        assert np.all(rows <= max(atol, 1e-5) + rtol), "dlogits rows do not sum to 0"
    return f, g, fo, go, log


# ----------------------------------------------------------------- the configs
@SKIP
def test_tiny_fp32_full(skip):
    inp = make_inputs("tiny")
    f, g, fo, go, log = _full_parity(inp, dlogits=True, skip=skip)
    # attention and output-softmax rows sum to 1
    valid = inp.src_len >= 1
    assert np.allclose(f["alpha"].sum(axis=-1)[valid], 1.0, atol=1e-5)
    m = f["tgt_mask"].astype(bool) if skip else np.ones_like(f["tgt_mask"], dtype=bool)
    p = np.exp(f["logits"][m].astype(np.float64) - f["lse"][m].astype(np.float64)[..., None])
    assert np.allclose(p.sum(axis=-1), 1.0, atol=1e-4)


@SKIP
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_full(dtype, skip):
    inp = make_inputs("small", dtype=dtype)
    _full_parity(inp, dlogits=True, skip=skip)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_skip_pad_rows_changes_no_result(dtype):
    """Row compaction is an execution detail: loss, masks, per-position outputs at word positions and the
    per-sentence gradients are bit-identical to the all-rows run (every row sees the same operands in the same
    order); the weight gradients, whose reduction over rows is regrouped, agree to fp32 summation order."""
    inp = make_inputs("small", dtype=dtype)
    a = pu.GpuRun(inp)
    fa, ga = a.fwd(), a.bwd(dlogits=True)
    b = pu.GpuRun(inp, skip_pad_rows=True)
    fb, gb = b.fwd(), b.bwd(dlogits=True)
    m = fa["tgt_mask"].astype(bool)
    assert fa["n_tok"] == fb["n_tok"] and np.array_equal(fa["tgt_mask"], fb["tgt_mask"])
    for k in ("alpha", "ctx", "h_c", "tok_loss", "attn_mask"):
        assert np.array_equal(fa[k], fb[k]), k
    for k in ("lse", "logits", "argmax"):
        assert np.array_equal(fa[k][m], fb[k][m]), k
    assert np.all(fb["argmax"][~m] == inp.pad_id)
    assert abs(fa["loss_sum"] - fb["loss_sum"]) <= 1e-6 * abs(fa["loss_sum"])
    assert np.array_equal(ga["dlogits"], gb["dlogits"])
    for k in ("d_h_dec", "d_h_enc", "dW_a", "dW_c"):
        assert np.array_equal(ga[k], gb[k]), k
    for k in ("dW_out", "db_out"):
        s = pu.err_stats(gb[k], ga[k], dtype)
        assert s["norm"] <= 1e-5, (k, s)


def test_grad_scale_is_applied_to_gradients_only():
    inp = make_custom(T=6, S=9, B=4, H=32, V=200, seed=77, dtype="f32", grad_scale=0.125)
    f, g, fo, go, _ = _full_parity(inp)
    inp1 = make_custom(T=6, S=9, B=4, H=32, V=200, seed=77, dtype="f32", grad_scale=1.0)
    f1 = pu.GpuRun(inp1).fwd()
    assert f1["loss_sum"] == f["loss_sum"]


# ----------------------------------------------------------------- edge shapes
EDGE_SHAPES = [
    # T, S, B, H, V : ragged against every tile edge (32/64/128/256, vectors of 4/8)
    (1, 1, 1, 8, 2),
    (1, 7, 3, 16, 17),          # per-step mode (T = 1), V not a multiple of the vector width
    (5, 7, 3, 24, 53),
    (37, 45, 5, 136, 1003),
    (9, 70, 2, 72, 259),        # S above one wavefront
    (130, 33, 2, 264, 515),     # T above one 128-row tile
]


@SKIP
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", EDGE_SHAPES)
def test_edge_shapes(shape, dtype, skip):
    T, S, B, H, V = shape
    inp = make_custom(T=T, S=S, B=B, H=H, V=V, seed=1000 + T + S + V, dtype=dtype, min_len=1,
                      pad_prob=0.3 if skip else 0.1)
    _full_parity(inp, dlogits=True, skip=skip)


@SKIP
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_data(dtype, skip):
    """Empty and over-long source lengths, out-of-range targets, an all-pad sentence."""
    inp = make_custom(T=7, S=11, B=6, H=40, V=301, seed=4242, dtype=dtype)
    inp.src_len[:] = [0, 11, 40, -3, 1, 5]          # clamped to [0, S]
    inp.targets[:, 1] = inp.pad_id                   # whole sentence padded
    inp.targets[0, 2] = inp.V + 9                    # outside the vocabulary -> padding
    inp.targets[1, 2] = -5
    inp.targets[2, 2] = inp.V - 1                    # last id is a real word
    f, g, fo, go, _ = _full_parity(inp, dlogits=True, skip=skip)
    assert np.all(f["alpha"][0] == 0) and np.all(f["alpha"][3] == 0)
    assert np.all(f["ctx"][:, 0] == 0)
    assert np.all(g["d_h_enc"][:, 0] == 0) and np.all(g["d_h_dec"][:, 1] == 0)
    assert f["tgt_mask"][0, 2] == 0 and f["tgt_mask"][1, 2] == 0 and f["tgt_mask"][2, 2] == 1


@SKIP
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_all_padding_batch_gives_zero_loss_and_gradients(dtype, skip):
    inp = make_custom(T=4, S=5, B=2, H=16, V=50, seed=9, dtype=dtype)
    inp.targets[:] = inp.pad_id
    run = pu.GpuRun(inp, skip_pad_rows=skip)
    f = run.fwd()
    g = run.bwd()
    assert f["loss_sum"] == 0.0 and f["n_tok"] == 0
    for k, v in g.items():
        assert np.all(v == 0.0), k


def test_zero_output_layer_gives_log_V():
    inp = make_custom(T=6, S=6, B=3, H=32, V=777, seed=10, dtype="bf16", pad_prob=0.2)
    inp.W_out[:] = 0
    inp.b_out[:] = 0
    f = pu.GpuRun(inp).fwd()
    m = f["tgt_mask"].astype(bool)
    assert np.allclose(f["tok_loss"][m], np.log(777.0), rtol=1e-6)
    assert np.all(f["argmax"] == 0)                  # all logits tie: lowest id


# -------------------------------------------------------- structural properties
@SKIP
def test_two_runs_are_bit_identical(skip):
    inp = make_inputs("small")
    a = pu.GpuRun(inp, skip_pad_rows=skip)
    fa, ga = a.fwd(), a.bwd()
    fb, gb = a.fwd(), a.bwd()                        # same buffers, second pass
    c = pu.GpuRun(inp, skip_pad_rows=skip)           # fresh buffers
    fc, gc = c.fwd(), c.bwd()
    for other_f, other_g in ((fb, gb), (fc, gc)):
        for k in fa:
            assert np.array_equal(np.asarray(fa[k]), np.asarray(other_f[k]), equal_nan=k in ("lse", "logits")), k
        for k in ga:
            assert np.array_equal(ga[k], other_g[k]), k


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_batch_shards_add_up(dtype):
    """Section 3.2: the batch is split equally over the GPUs and the parameter
    gradients are accumulated: four shards on one GPU must reproduce the batch."""
    inp = make_inputs("small", dtype=dtype)
    full = pu.GpuRun(inp)
    f, g = full.fwd(logits=False), full.bwd()
    acc = {k: np.zeros_like(g[k], dtype=np.float64) for k in ("dW_a", "dW_c", "dW_out", "db_out")}
    loss, ntok = 0.0, 0
    q = inp.B // 4
    for i in range(4):
        sh = inp.slice_batch(i * q, (i + 1) * q)
        r = pu.GpuRun(sh)
        fs, gs = r.fwd(logits=False), r.bwd()
        loss += fs["loss_sum"]
        ntok += fs["n_tok"]
        for k in acc:
            acc[k] += gs[k]
        # per-sentence results do not depend on the batch they are computed in
        sl = slice(i * q, (i + 1) * q)
        assert np.array_equal(fs["argmax"], f["argmax"][:, sl])
        assert np.array_equal(fs["alpha"], f["alpha"][sl])
        # (gradients pass through split-K sums whose split count depends on the batch size)
        gtol = 1e-5 if dtype == "f32" else 1e-3
        assert pu.err_stats(gs["d_h_dec"], g["d_h_dec"][:, sl], dtype)["norm"] <= gtol
        assert pu.err_stats(gs["d_h_enc"], g["d_h_enc"][:, sl], dtype)["norm"] <= gtol
    assert ntok == f["n_tok"]
    assert abs(loss - f["loss_sum"]) <= 1e-5 * abs(f["loss_sum"])
    for k in acc:
        s = pu.err_stats(acc[k], g[k], dtype)
        # summation order differs between one batch and four shards
        assert s["norm"] <= (1e-5 if dtype == "f32" else 5e-4), (k, s)


def test_all_steps_at_once_equals_step_by_step():
    """Section 3.2: alpha is computed at once for all decoder steps; T calls
    with one step each give the same rows."""
    inp = make_custom(T=6, S=13, B=5, H=64, V=400, seed=31, dtype="bf16", min_len=1)
    run = pu.GpuRun(inp)
    f, g = run.fwd(), run.bwd()
    d_enc = np.zeros_like(g["d_h_enc"], dtype=np.float64)
    for t in range(inp.T):
        one = make_custom(T=6, S=13, B=5, H=64, V=400, seed=31, dtype="bf16", min_len=1)
        one.T = 1
        one.h_dec = np.ascontiguousarray(inp.h_dec[t:t + 1])
        one.targets = np.ascontiguousarray(inp.targets[t:t + 1])
        r = pu.GpuRun(one)
        ft, gt = r.fwd(), r.bwd()
        assert np.array_equal(ft["alpha"][:, 0], f["alpha"][:, t])
        assert np.array_equal(ft["argmax"][0], f["argmax"][t])
        assert np.array_equal(ft["tok_loss"][0], f["tok_loss"][t])
        assert pu.err_stats(gt["d_h_dec"][0], g["d_h_dec"][t], "bf16")["norm"] <= 1e-3
        d_enc += gt["d_h_enc"]
    s = pu.err_stats(d_enc, g["d_h_enc"], "bf16")
    assert s["norm"] <= 1e-3, s


# -------------------------------------------- full-size configs, sampled sentences
def _sample_sentences(B, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, B // 2, B - 1]
    rest = [int(x) for x in rng.permutation(B) if int(x) not in fixed][:5]
    return sorted(fixed + rest)


_WHOLE_BATCH = {}


def _oracle_whole_batch(inp, chunks=8):
    """The oracle's backward pass over the whole batch of a full-size configuration (once per configuration,
    both row modes share it): every gradient, the weight gradients accumulated over all sentences as section
    3.2 describes.  Run in chunks of sentences so that a line of progress appears between them."""
    import sys
    if inp.name in _WHOLE_BATCH:
        return _WHOLE_BATCH[inp.name]
    _WHOLE_BATCH.clear()                       # one configuration at a time: stress holds 2 GB of dW_out alone
    total = None
    step = (inp.B + chunks - 1) // chunks
    for c, b0 in enumerate(range(0, inp.B, step)):
        part = orc_backward(inp, list(range(b0, min(b0 + step, inp.B))))
        if total is None:
            total = part
        else:
            for k in total:
                total[k] += part[k]            # per-sentence arrays are zero outside the chunk's sentences
        sys.__stderr__.write(f"[oracle {inp.name}: sentences {min(b0 + step, inp.B)}/{inp.B}]\n")
        sys.__stderr__.flush()
    _WHOLE_BATCH[inp.name] = total
    return total


def orc_backward(inp, sentences):
    return pu.orc.backward(*pu.oracle_args(inp), grad_scale=inp.grad_scale, sentences=sentences)


@SKIP
@pytest.mark.parametrize("name", ["mid", "large", "stress"])
def test_full_size_config_sampled(name, skip):
    """The configuration at its full size, as the benchmark launches it.

    Per-sentence forward results (alpha, ctx, h_c, logits, loss, argmax) are
    compared for 8 sampled sentences against the oracle, and those sentences
    are also run as a batch of their own and compared in full.  All six
    gradients of the full batch, as the timed launch configuration computes
    them, are compared element by element with the oracle run over the whole
    batch (mid and large in both row modes, stress in the mode the benchmark
    times); the full batch must also equal the sum of GPU shards.  The rest
    is checked through properties that hold at any size."""
    inp = make_inputs(name)
    idx = _sample_sentences(inp.B, 7)
    sub = inp.take_sentences(idx)
    fo, go = pu.run_oracle(sub)
    m = fo["tgt_mask"].astype(bool)
    log = {}

    # (1) the sampled sentences as their own batch: everything, including weight gradients
    hold = inp.pad_id if skip else None
    rs = pu.GpuRun(sub, skip_pad_rows=skip)
    fs, gs = rs.fwd(), rs.bwd()
    pu.compare_all(fs, gs, fo, go, inp.dtype, log, pad_rows_hold=hold)
    del rs

    # (2) the full batch
    run = pu.GpuRun(inp, skip_pad_rows=skip)
    f = run.fwd(sentences=idx)
    assert f["n_tok"] == inp.n_nonpad()
    for k in ("alpha", "ctx", "tok_loss"):
        pu.assert_close(f[k], fo[k], inp.dtype, k)
    for k in ("h_c", "lse", "logits"):
        pu.assert_close(f[k][m], fo[k][m], inp.dtype, k)
    assert np.array_equal(f["attn_mask"], fo["attn_mask"]) and np.array_equal(f["tgt_mask"], fo["tgt_mask"])
    pu.check_argmax(f["argmax"], f["logits"], fo["logits"], fo["tgt_mask"], inp.dtype, hold)
    # per-sentence results are independent of the batch around them
    assert np.array_equal(f["argmax"], fs["argmax"]) and np.array_equal(f["alpha"], fs["alpha"])
    db = run.db
    import torch
    tl = db.tok_loss.double().sum().item()
    assert abs(tl - f["loss_sum"]) <= 1e-5 * abs(tl)
    mean_loss = f["loss_sum"] / f["n_tok"]
    assert abs(mean_loss - np.log(inp.V)) < 0.5 * np.log(inp.V)       # random-init model: near log V
    del f

    g = run.bwd(sentences=idx, dlogits=True)
    pu.assert_close(g["d_h_dec"], go["d_h_dec"], inp.dtype, "d_h_dec")
    pu.assert_close(g["d_h_enc"], go["d_h_enc"], inp.dtype, "d_h_enc")
    dl = g["dlogits"].astype(np.float64)
    assert np.all(dl[~m] == 0.0)
    assert np.all(np.abs(dl.sum(axis=-1)) <= 2e-2)
    # properties over the whole batch
    assert abs(float(db.db_out.double().sum().item())) <= 1e-3 * inp.n_nonpad()   # sum_v db_out = sum of row sums = 0
    tm = db.tgt_mask.bool()
    assert torch.all(db.d_h_dec[~tm] == 0)
    for k in ("dW_a", "dW_c", "dW_out", "db_out", "d_h_dec", "d_h_enc"):
        assert bool(torch.isfinite(getattr(db, k)).all()), k
    # (3) additivity: full batch == sum over 4 GPU shards (fp32 summation order only)
    full = {k: getattr(db, k).double().cpu().numpy() for k in ("dW_a", "dW_c", "db_out")}
    dW_out_full = db.dW_out.double()
    if name != "stress" or skip:
        # (2b) every gradient of the timed launch configuration against the oracle over the whole batch
        gw = _oracle_whole_batch(inp)
        for k in ("dW_a", "dW_c", "db_out"):
            pu.assert_close(full[k], gw[k], inp.dtype, k + " (whole batch)", log)
        pu.assert_close(pu._host(db.dW_out), gw["dW_out"], inp.dtype, "dW_out (whole batch)", log)
        pu.assert_close(pu._host(db.d_h_dec), gw["d_h_dec"], inp.dtype, "d_h_dec (whole batch)", log)
        pu.assert_close(pu._host(db.d_h_enc), gw["d_h_enc"], inp.dtype, "d_h_enc (whole batch)", log)
        del gw
    acc = {k: np.zeros_like(v) for k, v in full.items()}
    acc_out = torch.zeros_like(dW_out_full)
    del run, db
    q = inp.B // 4
    for i in range(4):
        r = pu.GpuRun(inp.slice_batch(i * q, (i + 1) * q), skip_pad_rows=skip)
        r.db.fwd()
        r.db.bwd()
        r.db.sync()
        for k in acc:
            acc[k] += getattr(r.db, k).double().cpu().numpy()
        acc_out += r.db.dW_out.double()
        del r
    for k in acc:
        s = pu.err_stats(acc[k], full[k], inp.dtype)
        assert s["norm"] <= 5e-4, (k, s)
    rel = float((acc_out - dW_out_full).norm() / dW_out_full.norm())
    assert rel <= 5e-4, rel


# ------------------------------------------------------------------ HIP graph capture
@SKIP
def test_forward_backward_replays_from_a_hip_graph(skip):
    """The entry points only enqueue on the caller's stream (no allocation, no synchronisation, no host
    read-back), so a forward+backward pair can be captured into a HIP graph.  Every replay, with eager work and
    synchronisations of the program in between, must reproduce the eager result bit for bit."""
    import torch
    inp = make_inputs("small", dtype="bf16")
    run = pu.GpuRun(inp, skip_pad_rows=skip)
    f0, g0 = run.fwd(), run.bwd()                     # eager reference (also warms every kernel up)
    db = run.db
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        db.fwd()
        db.bwd()
    for rep in range(3):
        for t in (db.loss_sum, db.dW_out, db.dW_a, db.d_h_dec, db.d_h_enc, db.db_out):
            t.zero_()                                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert float(db.loss_sum.item()) == f0["loss_sum"], rep
        assert int(db.n_tok.item()) == f0["n_tok"]
        for k in ("d_h_dec", "d_h_enc", "dW_a", "dW_c", "dW_out", "db_out"):
            assert np.array_equal(pu._host(getattr(db, k)), g0[k]), (k, rep)
