#!/usr/bin/env python3
"""Benchmark of the attention-softmax path on one MI355X.

One step = one forward + one backward pass of the whole path (every kernel of
attn_softmax_fwd and attn_softmax_bwd) over one batch of synthetic input that
is already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload stress|large|mid|small|tiny]
                    [--dtype bf16|f32] [--no-cpu-baseline] [--all-rows]

value      = non-pad target tokens per second, fwd+bwd, whole job (one GPU)
rows       = R, the rows the vocabulary part of the path runs on: the non-pad target
             positions (row compaction, as_shape.skip_pad_rows = 1, the default here), or
             all N = T*B positions with --all-rows
roofline   = the kernel that takes the most time (a vocabulary GEMM): the flops it
             executes, 2*R*H*V per launch / its average launch duration, measured with
             HIP events on the launch stream inside the timed region, against the
             dense bf16 MFMA peak (2.5 PFLOP/s)
roofline_hbm = the two streaming softmax-cross-entropy kernels against the 8 TB/s
             HBM peak (algorithmic bytes R*V*e for the statistics pass, 2*R*V*e for
             the in-place dlogits pass); plain_stream_ceilings = plain read-only / copy /
             in-place streams over the same bytes with the same grids (no arithmetic)
cpu_baseline = the float64 numpy oracle timed on this machine's host cores on a few
             sentences of the same workload (a reported baseline, not a target)
adam       = the fused Adam update of the four parameter tensors (outside the timed
             steps unless --train-step): 30 bytes per element (bf16 storage copy)
             or 32 (f32) against the HBM peak
ms_per_step_hip_graph_replay = the same forward + backward captured once into a HIP graph and replayed (the
             headline value is the eager one)
per_step   = the per-step mode (T = 1) at the paper's model size, outside the timed steps: microseconds
             per decoder step of attn_softmax_fwd called with T = 1 and of attn_softmax_step_fwd
lstm_stack = the stacked-LSTM part that produces the hidden states (lstm_stack_fwd / lstm_stack_bwd), outside
             the timed steps, at the paper's model size (Table 2: embedding 512, hidden 1024, depth 4; B = 128,
             50 steps per side): encoder forward, decoder forward from the encoder's final states, decoder
             backward, encoder backward; per-step kernel time against the bytes a step must move
--train-step makes a step = forward with dropout 0.3 + backward + Adam on the four
             parameter tensors (the headline metric stays forward + backward)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
GEMM_STAGES = {  # stage -> flops per launch; N = all positions, R = rows of the vocabulary part
    "gemm_logits": lambda N, R, H, V: 2.0 * R * H * V,
    "gemm_dwout": lambda N, R, H, V: 2.0 * R * H * V,
    "gemm_dhc": lambda N, R, H, V: 2.0 * R * H * V,
    "gemm_q": lambda N, R, H, V: 2.0 * N * H * H,
    "gemm_hc": lambda N, R, H, V: 4.0 * N * H * H,
    "gemm_dwc": lambda N, R, H, V: 4.0 * N * H * H,      # both halves of dW_c in one launch
    "gemm_dch": lambda N, R, H, V: 2.0 * N * H * H,      # per launch (two launches per step)
    "gemm_dwa": lambda N, R, H, V: 2.0 * N * H * H,
    "gemm_dh": lambda N, R, H, V: 2.0 * N * H * H,
}


def _source_digest(names):
    """sha256 (16 hex digits) of each listed kernel source, as the traffic summary records them."""
    import hashlib
    out = {}
    for n in names:
        try:
            with open(os.path.join(ROOT, "paper_1909_00562_amd", "csrc", n), "rb") as fh:
                out[n] = hashlib.sha256(fh.read()).hexdigest()[:16]
        except OSError:
            out[n] = None
    return out


def _traffic_from_profiles(workload: str, stage: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if present AND taken with the kernel
    sources as they are now (the summary records their digests): a counter figure of an older kernel is not
    reported as this one's."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as fh:
            prof = json.load(fh)
    except (OSError, ValueError):
        return None
    rec = prof.get(workload, {}).get(stage)
    if rec is None:
        return None
    want = prof.get("_sources", {})
    if not want or _source_digest(sorted(want)) != want:
        return None
    return dict(rec, profile_commit=prof.get("_commit"))


def stream_ceilings(lib, torch, rows, V, e, iters=5):
    """What this machine's memory system gives plain streams over the bytes the cross-entropy kernels move
    (attn_softmax_stream_probe: same grids and loads in flight, no arithmetic): read-only, copy, in-place
    read-modify-write, GB/s by HIP events on the launch stream."""
    row_bytes = (V * e + 15) // 16 * 16
    nbytes = rows * row_bytes
    dev = torch.device("cuda:0")
    a = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    b = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    a.fill_(1)
    st = int(torch.cuda.current_stream().cuda_stream)
    out = {"bytes": nbytes}
    for kind, name, moved in ((0, "read_only", nbytes), (1, "copy", 2 * nbytes), (2, "in_place", 2 * nbytes)):
        lib.attn_softmax_stream_probe(kind, a, b, rows, row_bytes, st)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            lib.attn_softmax_stream_probe(kind, a, b, rows, row_bytes, st)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        out[name] = {"ms": ms, "GB/s": moved / (ms * 1e-3) / 1e9, "frac_of_peak": moved / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
    del a, b
    return out


def vendor_gemm_reference(torch, inp, iters, workload):
    """torch.matmul (the vendor BLAS) on the shapes of the three vocabulary products, random bf16 operands:
    logits = h_c W_out^T, d_h_c = dlogits W_out, dW_out = dlogits^T h_c over the R non-pad rows."""
    R, H, V = inp.n_nonpad(), inp.H, inp.V
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    h = (torch.rand(R, H, device=dev, generator=g) - 0.5).bfloat16()
    W = (torch.rand(V, H, device=dev, generator=g) - 0.5).bfloat16()
    dz = (torch.rand(R, V, device=dev, generator=g) - 0.5).bfloat16()
    outs = (torch.empty(R, V, device=dev, dtype=torch.bfloat16), torch.empty(R, H, device=dev, dtype=torch.bfloat16),
            torch.empty(V, H, device=dev, dtype=torch.bfloat16))
    prods = (("logits", lambda: torch.matmul(h, W.t(), out=outs[0])), ("d_h_c", lambda: torch.matmul(dz, W, out=outs[1])),
             ("dW_out", lambda: torch.matmul(dz.t(), h, out=outs[2])))
    res = {"workload": workload, "R": R, "H": H, "V": V, "flops_per_product": 2.0 * R * H * V,
           "library": "torch.matmul (vendor BLAS), bf16 in, bf16 out", "iters": iters}
    for name, fn in prods:
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        res[name] = {"ms": ms, "TFLOP/s": 2.0 * R * H * V / (ms * 1e-3) / 1e12,
                     "frac_of_peak": 2.0 * R * H * V / (ms * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS}
    return res


def cpu_baseline(inp, budget_s: float = 40.0):
    """Oracle fwd+bwd on the first sentences of the batch, about `budget_s` seconds."""
    from oracle import attn_softmax_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:  # pragma: no cover
        cores = os.cpu_count() or 1
    args = (inp.h_dec, inp.h_enc, inp.src_len, inp.W_a, inp.W_c, inp.W_out, inp.b_out, inp.targets, inp.pad_id)

    def run(sent):
        t0 = time.perf_counter()
        orc.forward(*args, keep_logits=False, sentences=sent)
        orc.backward(*args, grad_scale=inp.grad_scale, sentences=sent)
        return time.perf_counter() - t0

    t1 = run([0])                      # one sentence: sizes the sample (and warms the BLAS threads)
    n = int(max(1, min(inp.B, budget_s / max(t1, 1e-6))))
    sent = list(range(n))
    dt = run(sent)
    tgt = inp.targets[:, :n]
    tokens = int(((tgt != inp.pad_id) & (tgt >= 0) & (tgt < inp.V)).sum())
    return {"value": tokens / dt, "unit": "target tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"float64 numpy oracle fwd+bwd on sentences 0..{n - 1} of the {inp.name} batch "
                      f"({tokens} non-pad tokens, {inp.T * n} positions) in {dt:.2f} s",
            "positions_per_s": inp.T * n / dt}


def per_step_probe(lib, torch, B=128, S=50, H=1024, V=32000, iters=200):
    """Per-step mode (one decoder step, T = 1) at the paper's model size: microseconds per step of the general
    forward entry point called with T = 1 and of the step entry point (cached encoder-side score half, fused
    attention kernel), and the step's algorithmic HBM bytes (K' float + h_enc + W_c + W_out read, logits
    written and read once) against the HBM peak."""
    from synth_inputs import make_custom
    from paper_1909_00562_amd import binding as bd
    inp = make_custom(T=1, S=S, B=B, H=H, V=V, seed=11, dtype="bf16")
    db = lib.DeviceBatch(inp)

    def timed(fn):
        for _ in range(5):
            fn()
        db.sync()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        db.sync()
        return (time.perf_counter() - t0) / iters * 1e6

    us_general = timed(db.fwd)
    sh = bd.AsShape(1, S, B, H, V, inp.pad_id, bd.AS_BF16, 1.0, 0.0, 0)
    nbytes = lib.attn_softmax_step_workspace_bytes(sh)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=db.dev)
    h_t, tgt = db.h_dec[0].clone(), db.targets[0].clone()
    tok = torch.zeros(B, dtype=torch.float32, device=db.dev)
    amax = torch.zeros(B, dtype=torch.int32, device=db.dev)
    st = int(torch.cuda.current_stream().cuda_stream)
    lib.attn_softmax_step_prepare(sh, db.h_enc, db.W_a, ws, nbytes, st)
    us_step = timed(lambda: lib.attn_softmax_step_fwd(sh, h_t, db.h_enc, db.src_len, db.W_c, db.W_out, db.b_out, tgt,
                                                      db.loss_sum, db.n_tok, tok, amax, ws, nbytes, st))
    # 16 steps captured once into a HIP graph and replayed: what a decoding loop pays per step without
    # the host's launch calls (the entry point only enqueues, so it can be captured)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    db.sync()
    with torch.cuda.graph(graph, stream=side):
        gst = int(torch.cuda.current_stream().cuda_stream)
        for _ in range(16):
            lib.attn_softmax_step_fwd(sh, h_t, db.h_enc, db.src_len, db.W_c, db.W_out, db.b_out, tgt,
                                      db.loss_sum, db.n_tok, tok, amax, ws, nbytes, gst)
    us_step_graph = timed(graph.replay) / 16
    del graph
    bytes_step = S * B * H * (4 + 2) + 2 * H * H * 2 + V * H * 2 + 2 * B * V * 2
    return {"workload": f"T=1 B={B} S={S} H={H} V={V} bf16", "us_fwd_T1_general": us_general,
            "us_step_fwd": us_step, "us_step_fwd_hip_graph_replay": us_step_graph, "bound": "hbm",
            "bytes_per_step": bytes_step,
            "achieved": bytes_step / (us_step * 1e-6) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": bytes_step / (us_step * 1e-6) / 1e9 / PEAK_HBM_GBS}


def lstm_probe(lib, torch, T=50, B=128, I=512, H=1024, L=4, iters=5):
    """Encoder + decoder of the proposed model without input feeding (section 3.2, Fig. 3) at Table 2's size:
    ms per training step of the LSTM part and of its pieces, source+target tokens per second, the average
    duration of one time step of one layer (forward / backward kernel), and that step's algorithmic bytes
    (W_hh, h as value + remainder, the input half of the pre-activations read, gates + c + h written; backward:
    W_hh, gate gradients of the next step as value + remainder, saved gates and cell states read, gate gradients
    written twice) against the HBM peak."""
    from synth_inputs import make_lstm_inputs
    enc_in = make_lstm_inputs(T, B, I, H, L, seed=50, dtype="bf16", min_len=20)
    dec_in = make_lstm_inputs(T, B, I, H, L, seed=51, dtype="bf16", min_len=20)
    enc = lib.DeviceLstm(enc_in.x, enc_in.lengths, enc_in.W_ih, enc_in.W_hh, enc_in.b, dtype="bf16")
    dec = lib.DeviceLstm(dec_in.x, dec_in.lengths, dec_in.W_ih, dec_in.W_hh, dec_in.b, dtype="bf16")
    dec.h0, dec.c0 = enc.hT, enc.cT                           # the decoder starts from the encoder's final states
    dy_dec = torch.from_numpy(dec_in.dy).to(enc.dev)          # stand-ins for d_h_dec / d_h_enc of the attention part
    dy_enc = torch.from_numpy(enc_in.dy).to(enc.dev)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def run(timed):
        marks = [ev() for _ in range(5)]
        marks[0].record(); enc.fwd()
        marks[1].record(); dec.fwd()
        marks[2].record(); dec.bwd(dy_dec)
        marks[3].record(); enc.bwd(dy_enc, dec.dh0, dec.dc0)
        marks[4].record()
        if timed:
            enc.sync()
            return [marks[i].elapsed_time(marks[i + 1]) for i in range(4)]
        return None

    for _ in range(2):
        run(False)
    enc.sync()
    acc = [0.0] * 4
    for _ in range(iters):
        for i, v in enumerate(run(True)):
            acc[i] += v / iters
    total = sum(acc)
    tokens = int(enc_in.lengths.sum() + dec_in.lengths.sum())
    # one layer-step: the fused kernel's share of a forward / backward call (the large products over all steps
    # are a minor part; the per-kernel figure is in profiles/)
    e = 2
    fwd_bytes = 4 * H * H * e + 2 * B * H * e + B * 4 * H * 4 * 2 + B * H * (4 + 4 + 2 * 4)
    bwd_bytes = 4 * H * H * e + 2 * B * 4 * H * e + B * 4 * H * 4 + B * H * 4 * 5 + 4 * B * 4 * H * e
    us_f = acc[0] / (T * L) * 1e3
    us_b = acc[3] / (T * L) * 1e3
    return {"workload": f"encoder+decoder T={T} B={B} I={I} H={H} L={L} bf16, no input feeding",
            "ms_enc_fwd": acc[0], "ms_dec_fwd": acc[1], "ms_dec_bwd": acc[2], "ms_enc_bwd": acc[3], "ms_total": total,
            "src_plus_tgt_tokens_per_sec": tokens / (total * 1e-3), "tokens": tokens,
            "us_per_layer_step_fwd": us_f, "us_per_layer_step_bwd": us_b,
            "bound": "hbm", "bytes_per_layer_step_fwd": fwd_bytes, "bytes_per_layer_step_bwd": bwd_bytes,
            "achieved": fwd_bytes / (us_f * 1e-6) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": fwd_bytes / (us_f * 1e-6) / 1e9 / PEAK_HBM_GBS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="stress", choices=["tiny", "small", "mid", "large", "stress"])
    ap.add_argument("--dtype", default=None, choices=["bf16", "f32"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--train-step", action="store_true",
                    help="a step = fwd with dropout 0.3 + bwd + Adam update of W_a, W_c, W_out, b_out")
    ap.add_argument("--all-rows", action="store_true",
                    help="run the vocabulary part on all T*B positions (skip_pad_rows = 0) instead of the "
                         "non-pad ones")
    ap.add_argument("--no-stage-events", action="store_true",
                    help="do not bracket kernels with HIP events inside the timed region")
    ap.add_argument("--main-only", action="store_true",
                    help="only the timed forward + backward steps: no HIP-graph replay, no per-step / LSTM / stream "
                         "probes (for rocprofv3 --pmc runs, whose counter collection does not survive long graph "
                         "replays)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 1 GiB device-to-device copy kernel (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--vendor-gemm-reference", action="store_true",
                    help="only time the vendor BLAS (torch.matmul, bf16) on the three vocabulary products of the "
                         "workload and exit: a yardstick for the hand-written kernels, never part of the path")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the path on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1909_00562_amd as lib
    from synth_inputs import make_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    lib.load_library()                                   # fails loudly if the HIP library is not built
    if a.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4}))
        return

    if a.vendor_gemm_reference:
        print(json.dumps(vendor_gemm_reference(torch, make_inputs(a.workload, dtype=a.dtype), a.steps, a.workload)))
        return

    inp = make_inputs(a.workload, dtype=a.dtype)
    if a.train_step:
        inp.dropout_p, inp.dropout_seed = 0.3, 20190900562
    db = lib.DeviceBatch(inp, skip_pad_rows=not a.all_rows)
    T, S, B, H, V = inp.T, inp.S, inp.B, inp.H, inp.V
    N = T * B
    e = 2 if inp.dtype == "bf16" else 4
    n_tok = inp.n_nonpad()
    R = N if a.all_rows else n_tok                       # rows of the vocabulary part

    # Adam state of the four parameter tensors: float master copy and both moments
    params = [("W_a", "dW_a"), ("W_c", "dW_c"), ("W_out", "dW_out"), ("b_out", "db_out")]
    adam_state = {p: (getattr(db, p).float().contiguous(), torch.zeros_like(getattr(db, p), dtype=torch.float32),
                      torch.zeros_like(getattr(db, p), dtype=torch.float32)) for p, _ in params}
    n_params = sum(getattr(db, p).numel() for p, _ in params)
    store = lib.AS_BF16 if inp.dtype == "bf16" else lib.AS_F32
    adam_t = [0]

    def adam():
        adam_t[0] += 1
        hp = lib.AsAdam(1e-3, 0.9, 0.999, 1e-8, adam_t[0])
        st = int(torch.cuda.current_stream().cuda_stream)
        for p, gname in params:
            master, m1, m2 = adam_state[p]
            lib.attn_softmax_adam_step(hp, master.numel(), getattr(db, gname), master, m1, m2, getattr(db, p),
                                       store, st)

    def step():
        if a.train_step:
            db.shape.dropout_seed += 1
        db.fwd()
        db.bwd()
        if a.train_step:
            adam()

    for _ in range(a.warmup):
        step()
    db.sync()
    # inside the timed region only the kernels the rooflines are about carry HIP events (the vocabulary GEMMs and
    # the two cross-entropy passes: > 90 % of the step); the per-stage table of all kernels is taken afterwards
    timed_stages = ["gemm_logits", "gemm_dwout", "gemm_dhc", "xent_stats", "xent_dlogits"]
    lib.attn_softmax_profile_enable(not a.no_stage_events)
    if not a.no_stage_events:
        lib.attn_softmax_profile_select(timed_stages)
    db.sync()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    db.sync()
    dt = time.perf_counter() - t0
    stages = lib.attn_softmax_profile_read()
    lib.attn_softmax_profile_enable(False)
    assert int(db.n_tok.item()) == n_tok
    if not a.no_stage_events:   # every stage, outside the timed region (the timed ones keep their in-region figures)
        lib.attn_softmax_profile_enable(True)
        extra = max(3, a.steps // 4)
        for _ in range(extra):
            step()
        db.sync()
        for k, v in lib.attn_softmax_profile_read().items():
            if k not in timed_stages and v["launches"]:
                stages[k] = {"ms": v["ms"] * a.steps / extra, "launches": v["launches"] * a.steps // extra}
        lib.attn_softmax_profile_enable(False)

    # the same step replayed from a HIP graph (one capture of forward + backward): what the launches cost
    graph_ms = None
    if not a.train_step and not a.main_only:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        db.sync()
        with torch.cuda.graph(graph, stream=side):
            db.fwd()
            db.bwd()
        graph.replay()
        db.sync()
        g0 = time.perf_counter()
        for _ in range(a.steps):
            graph.replay()
        db.sync()
        graph_ms = (time.perf_counter() - g0) / a.steps * 1e3
        assert int(db.n_tok.item()) == n_tok
        del graph

    # the Adam update on its own (gradients of the last step), HIP events on the launch stream
    adam(); db.sync()
    lib.attn_softmax_profile_enable(True)
    n_adam = 5
    for _ in range(n_adam):
        adam()
    db.sync()
    adam_ms = lib.attn_softmax_profile_read()["adam"]["ms"] / n_adam
    lib.attn_softmax_profile_enable(False)
    adam_bytes = n_params * (30.0 if inp.dtype == "bf16" else 32.0)

    ms_step = dt / a.steps * 1e3
    per_stage = {k: (v["ms"] / v["launches"] if v["launches"] else 0.0) for k, v in stages.items()}
    step_ms_by_stage = {k: v["ms"] / a.steps for k, v in stages.items() if v["launches"]}

    roofline = None
    roofline_hbm = None
    if not a.no_stage_events:
        gemm_ms = {k: step_ms_by_stage.get(k, 0.0) for k in GEMM_STAGES}
        dom = max(gemm_ms, key=gemm_ms.get)
        flops = GEMM_STAGES[dom](N, R, H, V)
        avg_ms = per_stage[dom]
        ach = flops / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else 0.0
        bf = inp.dtype == "bf16"
        peak = PEAK_MFMA_BF16_TFLOPS if bf else PEAK_FP32_TFLOPS
        roofline = {"kernel": dom, "bound": "mfma" if bf else "alu", "achieved": ach, "peak": peak,
                    "unit": "TFLOP/s", "frac": ach / peak, "avg_launch_ms": avg_ms,
                    "flops_per_launch": flops, "traffic": _traffic_from_profiles(a.workload, dom)}
        # all three vocabulary GEMMs together (they are >90 % of the path's flops)
        voc_ms = sum(step_ms_by_stage.get(k, 0.0) for k in ("gemm_logits", "gemm_dwout", "gemm_dhc"))
        if voc_ms > 0:
            roofline["vocab_gemms_tflops"] = 6.0 * R * H * V / (voc_ms * 1e-3) / 1e12
        sb = float(R) * V * e
        st_ms, dl_ms = per_stage.get("xent_stats", 0.0), per_stage.get("xent_dlogits", 0.0)
        tot = st_ms + dl_ms
        if tot > 0:
            ach_b = 3.0 * sb / (tot * 1e-3) / 1e9
            roofline_hbm = {"kernel": "xent_stats+xent_dlogits", "bound": "hbm", "achieved": ach_b,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach_b / PEAK_HBM_GBS,
                            "bytes_per_step": 3.0 * sb,
                            "xent_stats": {"avg_launch_ms": st_ms, "GB/s": sb / (st_ms * 1e-3) / 1e9 if st_ms else 0},
                            "xent_dlogits": {"avg_launch_ms": dl_ms,
                                             "GB/s": 2 * sb / (dl_ms * 1e-3) / 1e9 if dl_ms else 0},
                            "traffic": _traffic_from_profiles(a.workload, "xent")}

    out = {
        "metric": "attn_softmax_fwd_bwd_target_tokens_per_sec",
        "value": n_tok / (dt / a.steps),
        "unit": "target tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": inp.dtype, "data": "synthetic",
        "config": {"workload": a.workload, "B": B, "T": T, "S": S, "H": H, "V": V, "positions": N,
                   "non_pad_tokens": n_tok, "grad_scale": inp.grad_scale,
                   "skip_pad_rows": 0 if a.all_rows else 1, "rows_in_vocabulary_part": R},
        "positions_per_sec": N / (dt / a.steps),
        "path_tflops": (6.0 * R * H * V + 18.0 * N * H * H + 12.0 * B * T * S * H) / (dt / a.steps) / 1e12,
        "roofline": roofline,
        "roofline_hbm": roofline_hbm,
        "stage_ms_per_step": {k: round(v, 5) for k, v in step_ms_by_stage.items()},
        "adam": {"kernel": "adam_step (W_a, W_c, W_out, b_out)", "bound": "hbm", "elements": n_params,
                 "ms": adam_ms, "achieved": adam_bytes / (adam_ms * 1e-3) / 1e9 if adam_ms > 0 else 0.0,
                 "peak": PEAK_HBM_GBS, "unit": "GB/s",
                 "frac": adam_bytes / (adam_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if adam_ms > 0 else 0.0},
        "step_is": "fwd(dropout 0.3)+bwd+adam" if a.train_step else "fwd+bwd",
        "ms_per_step_hip_graph_replay": graph_ms,
    }
    del adam_state
    del db
    torch.cuda.empty_cache()
    if roofline_hbm is not None and not a.main_only:
        # the same bytes as plain streams: this box's ceilings next to the kernels' figures
        roofline_hbm["plain_stream_ceilings"] = stream_ceilings(lib, torch, R, V, e)
    if not a.main_only:
        out["per_step"] = per_step_probe(lib, torch)
        out["lstm_stack"] = lstm_probe(lib, torch)
    if not a.no_cpu_baseline and not a.main_only:
        out["cpu_baseline"] = cpu_baseline(inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
