"""Pins for the float64 CPU oracle (no GPU).

The paper prints no worked numerical example for the attention-softmax part,
so the oracle is pinned to what its equations (section 3.2, Eq. 1-6) and the
mathematics fix: invariants, closed forms, special cases that reduce to a
library routine (scipy logsumexp / sigmoid), the paper's structural claims
(all decoder steps at once == step by step; a batch == the sum of its shards),
loop-only brute force, and central finite differences on every gradient
element.  Each test is chosen so that a plausible slip in the oracle (a dropped
term, a wrong sign or axis, a transposed operand) fails it.
"""
import math

import numpy as np
import pytest
from scipy.special import expit, logsumexp

from oracle import attn_softmax_oracle as orc
from synth_inputs import make_custom, make_inputs


def _args(inp):
    return (inp.h_dec, inp.h_enc, inp.src_len, inp.W_a, inp.W_c, inp.W_out, inp.b_out,
            inp.targets, inp.pad_id)


def _small(seed=7, **kw):
    d = dict(T=5, S=6, B=3, H=8, V=11, seed=seed)
    d.update(kw)
    inp = make_custom(**d)
    inp.targets[1, 0] = inp.pad_id          # at least one pad and one non-pad position
    if inp.targets[0, 0] == inp.pad_id:
        inp.targets[0, 0] = 1
    return inp


# ---------------------------------------------------------------- invariants
def test_attention_rows_sum_to_one_and_mask_is_exact_zero():
    inp = _small(min_len=1)
    inp.src_len[:] = [6, 3, 1]
    f = orc.forward(*_args(inp))
    assert np.allclose(f["alpha"].sum(axis=2), 1.0, atol=1e-12)
    for b, L in enumerate(inp.src_len):
        assert np.all(f["alpha"][b, :, L:] == 0.0)          # exactly zero, not exp(-big)
        assert np.all(f["alpha"][b, :, :L] > 0.0)
        assert list(f["attn_mask"][b]) == [1] * L + [0] * (inp.S - L)


def test_output_softmax_rows_sum_to_one_and_lse_matches_scipy():
    inp = _small()
    f = orc.forward(*_args(inp))
    p = np.exp(f["logits"] - f["lse"][..., None])
    assert np.allclose(p.sum(axis=-1), 1.0, atol=1e-12)
    assert np.allclose(f["lse"], logsumexp(f["logits"], axis=-1), atol=1e-12)


def test_loss_is_log_V_for_zero_logits():
    inp = _small(V=37)
    inp.W_out[:] = 0
    inp.b_out[:] = 0
    f = orc.forward(*_args(inp))
    m = f["tgt_mask"].astype(bool)
    assert m.sum() == f["n_tok"] and 0 < f["n_tok"] < m.size
    assert np.allclose(f["tok_loss"][m], math.log(37), atol=1e-12)
    assert np.all(f["tok_loss"][~m] == 0.0)
    assert abs(f["loss_sum"] / f["n_tok"] - math.log(37)) < 1e-12


def test_dlogits_rows_sum_to_zero_and_pad_rows_vanish():
    inp = _small(grad_scale=1.0)
    g = orc.backward(*_args(inp), grad_scale=0.7, keep_dlogits=True)
    f = orc.forward(*_args(inp))
    m = f["tgt_mask"].astype(bool)
    assert np.allclose(g["dlogits"].sum(axis=-1), 0.0, atol=1e-13)
    assert np.all(g["dlogits"][~m] == 0.0)
    # non-pad rows: 0.7 * (p - onehot)
    p = np.exp(f["logits"] - f["lse"][..., None])
    t, b = np.nonzero(m)
    p[t, b, inp.targets[t, b]] -= 1.0
    assert np.allclose(g["dlogits"][m], 0.7 * p[m], atol=1e-14)
    assert np.allclose(g["db_out"], g["dlogits"].sum(axis=(0, 1)), atol=1e-13)


def test_pad_positions_contribute_nothing():
    inp = _small(seed=11)
    f0 = orc.forward(*_args(inp))
    g0 = orc.backward(*_args(inp))
    m = f0["tgt_mask"].astype(bool)
    assert (~m).any()
    # change the decoder state at pad positions: no loss / weight-gradient change
    inp2 = _small(seed=11)
    rng = np.random.default_rng(0)
    noise = rng.standard_normal(inp2.h_dec.shape).astype(np.float32)
    inp2.h_dec[~m] += noise[~m]
    f1 = orc.forward(*_args(inp2))
    g1 = orc.backward(*_args(inp2))
    assert f1["loss_sum"] == pytest.approx(f0["loss_sum"], abs=1e-12)
    for k in ("dW_a", "dW_c", "dW_out", "db_out", "d_h_enc"):
        assert np.allclose(g0[k], g1[k], atol=1e-12), k
    assert np.all(g0["d_h_dec"][~m] == 0.0)
    # out-of-range targets are padding too
    inp3 = _small(seed=11)
    inp3.targets[~m] = inp3.V + 5
    inp3.targets[0, 0] = -3
    f3 = orc.forward(*_args(inp3))
    assert f3["tgt_mask"][0, 0] == 0
    assert f3["n_tok"] == f0["n_tok"] - int(m[0, 0])


def test_masked_source_rows_get_exact_zero_gradient_and_garbage_is_ignored():
    inp = _small(seed=5)
    inp.src_len[:] = [4, 6, 2]
    g = orc.backward(*_args(inp))
    for b, L in enumerate(inp.src_len):
        assert np.all(g["d_h_enc"][L:, b] == 0.0)
        assert np.any(g["d_h_enc"][:L, b] != 0.0)
    f0 = orc.forward(*_args(inp))
    inp.h_enc[5, 0] = 1e3
    inp.h_enc[3, 2] = -77.0
    f1 = orc.forward(*_args(inp))
    g1 = orc.backward(*_args(inp))
    assert f1["loss_sum"] == f0["loss_sum"]
    for k in g:
        assert np.array_equal(g[k], g1[k]), k


def test_empty_source_sentence_is_defined():
    inp = _small(seed=3)
    inp.src_len[:] = [0, 6, -2]
    f = orc.forward(*_args(inp))
    g = orc.backward(*_args(inp))
    assert np.all(f["alpha"][0] == 0) and np.all(f["alpha"][2] == 0)
    assert np.all(f["ctx"][:, 0] == 0)
    assert np.all(np.isfinite(f["tok_loss"]))
    assert np.all(g["d_h_enc"][:, 0] == 0) and np.all(g["d_h_enc"][:, 2] == 0)
    for k in g:
        assert np.all(np.isfinite(g[k])), k
    # with no source, h~ = tanh(W_c[:,H:] h_t)
    H = inp.H
    ht = np.tanh(inp.h_dec[:, 0].astype(np.float64) @ inp.W_c[:, H:].astype(np.float64).T)
    assert np.allclose(f["h_c"][:, 0], ht, atol=1e-14)


# ---------------------------------------------------------------- closed forms
def test_zero_Wa_gives_uniform_attention_and_mean_context():
    inp = _small(seed=2, min_len=1)
    inp.W_a[:] = 0
    inp.src_len[:] = [6, 4, 1]
    f = orc.forward(*_args(inp))
    for b, L in enumerate(inp.src_len):
        assert np.allclose(f["alpha"][b, :, :L], 1.0 / L, atol=1e-15)
        mean = inp.h_enc[:L, b].astype(np.float64).mean(axis=0)
        assert np.allclose(f["ctx"][:, b], mean[None, :], atol=1e-14)
    # L = 1: alpha = 1 and c = h_enc[0]
    assert np.all(f["alpha"][2, :, 0] == 1.0)
    assert np.allclose(f["ctx"][:, 2], inp.h_enc[0, 2][None, :], atol=0)


def test_sharp_attention_picks_the_matching_source_position():
    # one-hot states, W_a = kappa * I: score[t,s] = kappa * [dec(t) == enc(s)]
    T, S, B, H, V = 4, 4, 1, 4, 5
    inp = make_custom(T, S, B, H, V, seed=1)
    inp.h_dec[:] = 0
    inp.h_enc[:] = 0
    perm = [2, 0, 3, 1]
    for t in range(T):
        inp.h_dec[t, 0, t] = 1.0
    for s in range(S):
        inp.h_enc[s, 0, perm[s]] = 1.0
    inp.W_a[:] = 50.0 * np.eye(H, dtype=np.float32)
    inp.src_len[:] = S
    f = orc.forward(*_args(inp))
    for t in range(T):
        s_match = perm.index(t)
        assert f["alpha"][0, t, s_match] > 1 - 1e-15
        assert np.allclose(f["ctx"][t, 0], inp.h_enc[s_match, 0], atol=1e-15)


def test_zero_Wc_reduces_to_softmax_of_bias():
    inp = _small(seed=4)
    inp.W_c[:] = 0
    f = orc.forward(*_args(inp))
    g = orc.backward(*_args(inp))
    b64 = inp.b_out.astype(np.float64)
    assert np.all(f["h_c"] == 0)
    m = f["tgt_mask"].astype(bool)
    expect = logsumexp(b64) - b64[inp.targets]
    assert np.allclose(f["tok_loss"][m], expect[m], atol=1e-13)
    # gradients: dW_out = 0 (h~ = 0); db_out = n_tok*softmax(b) - counts
    assert np.all(g["dW_out"] == 0)
    counts = np.bincount(inp.targets[m], minlength=inp.V)
    sm = np.exp(b64 - logsumexp(b64))
    assert np.allclose(g["db_out"], f["n_tok"] * sm - counts, atol=1e-12)
    # every row predicts argmax(b_out)
    assert np.all(f["argmax"] == int(np.argmax(b64)))


def test_single_word_vocabulary_has_zero_loss():
    inp = make_custom(3, 4, 2, 5, 1, seed=9)
    a = list(_args(inp))
    a[-1] = -1                       # nothing is padding
    f = orc.forward(*a)
    g = orc.backward(*a, keep_dlogits=True)
    assert f["n_tok"] == 6 and np.all(f["tok_loss"] == 0.0)
    for k in g:
        assert np.all(g[k] == 0.0), k


def test_scalar_worked_example():
    """H = 1, S = 2, T = 1, V = 2: everything reduces to scalar tanh / sigmoid.

    Values from tests/golden/scalar_example.txt (derived there by hand)."""
    import os
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "scalar_example.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    a, s1, s2, wa = vals["h_dec"], vals["h_enc1"], vals["h_enc2"], vals["W_a"]
    wc_c, wc_h = vals["W_c_c"], vals["W_c_h"]
    wo0, wo1, b0, b1 = vals["W_out0"], vals["W_out1"], vals["b_out0"], vals["b_out1"]
    args = (np.array([[[a]]]), np.array([[[s1]], [[s2]]]), np.array([2]), np.array([[wa]]),
            np.array([[wc_c, wc_h]]), np.array([[wo0], [wo1]]), np.array([b0, b1]),
            np.array([[1]]), -1)
    f = orc.forward(*args)
    # two-way softmax == logistic sigmoid of the score difference
    a1 = expit(a * wa * (s1 - s2))
    assert f["alpha"][0, 0, 0] == pytest.approx(a1, abs=1e-15)
    assert f["alpha"][0, 0, 0] == pytest.approx(vals["alpha1"], abs=1e-9)
    c = a1 * s1 + (1 - a1) * s2
    ht = math.tanh(wc_c * c + wc_h * a)
    assert f["h_c"][0, 0, 0] == pytest.approx(ht, abs=1e-15)
    assert f["h_c"][0, 0, 0] == pytest.approx(vals["h_tilde"], abs=1e-9)
    # two-way output softmax: -log p(y=1) = softplus(l0 - l1)
    l0, l1 = wo0 * ht + b0, wo1 * ht + b1
    loss = math.log1p(math.exp(l0 - l1))
    assert f["loss_sum"] == pytest.approx(loss, abs=1e-14)
    assert f["loss_sum"] == pytest.approx(vals["loss"], abs=1e-9)
    g = orc.backward(*args)
    # d loss / d b_out = (p0, p1 - 1)
    p0 = expit(l0 - l1)
    assert g["db_out"][0] == pytest.approx(p0, abs=1e-14)
    assert g["db_out"][1] == pytest.approx(-p0, abs=1e-14)
    assert g["db_out"][0] == pytest.approx(vals["db_out0"], abs=1e-9)
    # d loss / d h~ = p0 * (wo0 - wo1); chain through tanh to W_c's h column
    dz = p0 * (wo0 - wo1) * (1 - ht * ht)
    assert g["dW_c"][0, 1] == pytest.approx(dz * a, abs=1e-14)
    assert g["dW_c"][0, 0] == pytest.approx(dz * c, abs=1e-14)
    # d c / d score diff = alpha1 (1 - alpha1)(s1 - s2); score_i = a * wa * s_i
    dc = dz * wc_c
    dwa = dc * a1 * (1 - a1) * (s1 - s2) * a * (s1 - s2)
    assert g["dW_a"][0, 0] == pytest.approx(dwa, abs=1e-14)
    assert g["dW_a"][0, 0] == pytest.approx(vals["dW_a"], abs=1e-9)
    dhdec = dz * wc_h + dc * a1 * (1 - a1) * (s1 - s2) * wa * (s1 - s2)
    assert g["d_h_dec"][0, 0, 0] == pytest.approx(dhdec, abs=1e-14)
    dsenc1 = dc * a1 + dc * a1 * (1 - a1) * (s1 - s2) * a * wa
    assert g["d_h_enc"][0, 0, 0] == pytest.approx(dsenc1, abs=1e-14)


# ------------------------------------------------------- invariances / structure
def test_shift_invariances():
    inp = _small(seed=6)
    f0 = orc.forward(*_args(inp))
    g0 = orc.backward(*_args(inp))
    a = list(_args(inp))
    a[6] = inp.b_out.astype(np.float64) + 3.25           # constant added to every logit
    f1 = orc.forward(*a)
    g1 = orc.backward(*a)
    assert f1["loss_sum"] == pytest.approx(f0["loss_sum"], abs=1e-11)
    for k in g0:
        assert np.allclose(g0[k], g1[k], atol=1e-12), k


def test_source_permutation_and_extra_masked_positions():
    inp = _small(seed=8, B=1, min_len=4)
    inp.src_len[:] = 4
    f0 = orc.forward(*_args(inp))
    g0 = orc.backward(*_args(inp))
    perm = np.array([2, 0, 3, 1, 4, 5])
    a = list(_args(inp))
    a[1] = inp.h_enc[perm]
    f1 = orc.forward(*a)
    g1 = orc.backward(*a)
    assert np.allclose(f1["ctx"], f0["ctx"], atol=1e-14)
    assert f1["loss_sum"] == pytest.approx(f0["loss_sum"], abs=1e-12)
    assert np.allclose(f1["alpha"], f0["alpha"][:, :, perm], atol=1e-14)
    assert np.allclose(g1["d_h_enc"], g0["d_h_enc"][perm], atol=1e-13)
    for k in ("dW_a", "dW_c", "dW_out", "db_out", "d_h_dec"):
        assert np.allclose(g0[k], g1[k], atol=1e-12), k
    # appending masked source positions changes nothing
    a = list(_args(inp))
    a[1] = np.concatenate([inp.h_enc, 9 * np.ones((3, 1, inp.H), np.float32)], axis=0)
    f2 = orc.forward(*a)
    g2 = orc.backward(*a)
    assert f2["loss_sum"] == f0["loss_sum"]
    assert np.array_equal(f2["alpha"][:, :, :6], f0["alpha"]) and np.all(f2["alpha"][:, :, 6:] == 0)
    assert np.array_equal(g2["d_h_enc"][:6], g0["d_h_enc"]) and np.all(g2["d_h_enc"][6:] == 0)
    assert np.array_equal(g2["dW_out"], g0["dW_out"])


def test_all_steps_at_once_equals_step_by_step():
    """Section 3.2: alpha can be computed at once for all decoder steps."""
    inp = _small(seed=12)
    f = orc.forward(*_args(inp))
    g = orc.backward(*_args(inp))
    acc = {k: np.zeros_like(v) for k, v in g.items()}
    loss = 0.0
    for t in range(inp.T):
        a = list(_args(inp))
        a[0] = inp.h_dec[t:t + 1]
        a[7] = inp.targets[t:t + 1]
        ft = orc.forward(*a)
        gt = orc.backward(*a)
        loss += ft["loss_sum"]
        assert np.allclose(ft["alpha"][:, 0], f["alpha"][:, t], atol=1e-15)
        assert np.array_equal(ft["argmax"][0], f["argmax"][t])
        acc["d_h_dec"][t] = gt["d_h_dec"][0]
        for k in ("d_h_enc", "dW_a", "dW_c", "dW_out", "db_out"):
            acc[k] += gt[k]
    assert loss == pytest.approx(f["loss_sum"], abs=1e-12)
    for k in g:
        assert np.allclose(acc[k], g[k], atol=1e-12), k


def test_batch_additivity():
    """Section 3.2: the mini-batch is split equally over GPUs and the parameter
    gradients accumulated; so a batch equals the sum of its shards."""
    inp = _small(seed=13, B=4)
    f = orc.forward(*_args(inp))
    g = orc.backward(*_args(inp))
    loss = 0.0
    acc = {k: np.zeros_like(g[k]) for k in ("dW_a", "dW_c", "dW_out", "db_out")}
    for b0 in (0, 2):
        sh = inp.slice_batch(b0, b0 + 2)
        fs = orc.forward(*_args(sh))
        gs = orc.backward(*_args(sh))
        loss += fs["loss_sum"]
        for k in acc:
            acc[k] += gs[k]
        assert np.allclose(gs["d_h_dec"], g["d_h_dec"][:, b0:b0 + 2], atol=1e-14)
        assert np.allclose(gs["d_h_enc"], g["d_h_enc"][:, b0:b0 + 2], atol=1e-14)
        assert np.array_equal(fs["argmax"], f["argmax"][:, b0:b0 + 2])
    assert loss == pytest.approx(f["loss_sum"], abs=1e-12)
    for k in acc:
        assert np.allclose(acc[k], g[k], atol=1e-12), k
    # the `sentences` argument computes the same shard
    gsub = orc.backward(*_args(inp), sentences=[2, 3])
    gsh = orc.backward(*_args(inp.slice_batch(2, 4)))
    assert np.allclose(gsub["dW_out"], gsh["dW_out"], atol=1e-14)
    assert np.all(gsub["d_h_dec"][:, :2] == 0)


# ---------------------------------------------------------------- brute force
def test_forward_matches_loop_only_brute_force():
    inp = make_custom(T=3, S=4, B=2, H=5, V=7, seed=21)
    inp.src_len[:] = [4, 2]
    f = orc.forward(*_args(inp))
    T, S, B, H, V = inp.T, inp.S, inp.B, inp.H, inp.V
    hd, he = inp.h_dec.astype(float), inp.h_enc.astype(float)
    Wa, Wc, Wo, bo = (x.astype(float) for x in (inp.W_a, inp.W_c, inp.W_out, inp.b_out))
    total = 0.0
    for b in range(B):
        L = int(inp.src_len[b])
        for t in range(T):
            sc = []
            for s in range(L):
                v = 0.0
                for i in range(H):
                    for j in range(H):
                        v += hd[t, b, i] * Wa[i, j] * he[s, b, j]
                sc.append(v)
            mx = max(sc)
            ex = [math.exp(v - mx) for v in sc]
            al = [e / sum(ex) for e in ex]
            c = [sum(al[s] * he[s, b, j] for s in range(L)) for j in range(H)]
            cat = c + [hd[t, b, j] for j in range(H)]
            ht = [math.tanh(sum(Wc[k, j] * cat[j] for j in range(2 * H))) for k in range(H)]
            lg = [sum(Wo[v, k] * ht[k] for k in range(H)) + bo[v] for v in range(V)]
            lse = math.log(sum(math.exp(x) for x in lg))
            y = int(inp.targets[t, b])
            for s in range(L):
                assert f["alpha"][b, t, s] == pytest.approx(al[s], abs=1e-14)
            for k in range(H):
                assert f["h_c"][t, b, k] == pytest.approx(ht[k], abs=1e-14)
                assert f["ctx"][t, b, k] == pytest.approx(c[k], abs=1e-14)
            for v in range(V):
                assert f["logits"][t, b, v] == pytest.approx(lg[v], abs=1e-14)
            assert f["argmax"][t, b] == max(range(V), key=lambda v: (lg[v], -v))
            if y != inp.pad_id:
                total += lse - lg[y]
                assert f["tok_loss"][t, b] == pytest.approx(lse - lg[y], abs=1e-13)
    assert f["loss_sum"] == pytest.approx(total, abs=1e-12)


def test_argmax_ties_go_to_lowest_id():
    inp = _small(seed=14)
    inp.W_out[:] = 0
    inp.b_out[:] = 0
    inp.b_out[[3, 7]] = 1.0
    f = orc.forward(*_args(inp))
    assert np.all(f["argmax"] == 3)


# ---------------------------------------------------------- finite differences
@pytest.mark.parametrize("seed,g", [(31, 1.0), (32, 0.37)])
def test_central_finite_differences_every_gradient_element(seed, g):
    inp = make_custom(T=3, S=4, B=2, H=5, V=7, seed=seed, w=0.6)
    inp.src_len[:] = [4, 2]
    inp.targets[1, 0] = inp.pad_id
    base = [np.array(x, dtype=np.float64) for x in
            (inp.h_dec, inp.h_enc, inp.W_a, inp.W_c, inp.W_out, inp.b_out)]

    def loss_of(arrs):
        hd, he, wa, wc, wo, bo = arrs
        return orc.scaled_loss(hd, he, inp.src_len, wa, wc, wo, bo, inp.targets, inp.pad_id, g)

    hd, he, wa, wc, wo, bo = base
    grads = orc.backward(hd, he, inp.src_len, wa, wc, wo, bo, inp.targets, inp.pad_id, grad_scale=g)
    names = ["d_h_dec", "d_h_enc", "dW_a", "dW_c", "dW_out", "db_out"]
    eps = 1e-6
    for idx, name in enumerate(names):
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
        err = np.abs(num - an).max() / scale
        assert err < 1e-7, (name, err)
        assert np.abs(an).max() > 0, name


# --------------------------------------------------------------- input recipe
def test_input_generator_is_seeded_and_matches_recipe():
    a = make_inputs("tiny")
    b = make_inputs("tiny")
    for k in a.FLOAT_FIELDS:
        assert np.array_equal(getattr(a, k), getattr(b, k))
    assert a.dtype == "f32" and a.h_dec.shape == (8, 4, 64) and a.W_out.shape == (1000, 64)
    assert a.src_len.min() >= 1 and a.src_len.max() <= 8
    assert np.abs(a.W_c).max() <= 0.1 and np.abs(a.h_dec).max() < 1
    assert (a.targets == 0).mean() > 0 and a.targets.max() <= 999
    s = make_inputs("small")
    assert s.dtype == "bf16"
    # bf16-representable: low 16 bits of the float32 pattern are zero
    assert np.all((s.W_out.view(np.uint32) & 0xFFFF) == 0)
    # right-padded targets, Zipf head is token 1
    T = s.T
    for b_ in range(s.B):
        col = s.targets[:, b_]
        n = int((col != 0).sum())
        assert 10 <= n <= 30 and np.all(col[:n] != 0) and np.all(col[n:] == 0)
    ids, cnt = np.unique(s.targets[s.targets != 0], return_counts=True)
    assert ids[np.argmax(cnt)] == 1
    # same draws for both storage types (f32 values round to the bf16 ones)
    s32 = make_inputs("small", dtype="f32")
    assert np.array_equal(s32.targets, s.targets)
    assert np.max(np.abs(s32.h_dec - s.h_dec)) <= 2.0 ** -8
