"""Seeded synthetic inputs for the attention-softmax path.

This module only draws random tensors and rounds them to the storage type.
It holds none of the method's arithmetic and is the one piece of code that
both the CPU oracle's tests and the HIP path's tests/bench may share.

The paper trains on WMT14/WMT17 English-German with a 32K joint-BPE
vocabulary, hidden size 1024 and per-GPU batches of 56-64 sentences (its
Table 1-3).  Those corpora are not used here: the configurations below stand
in for them with the same shapes, variable sentence lengths with padding, and
a Zipf-like target-id distribution as in natural-language BPE vocabularies.

Recipe (identical bits for the oracle and the GPU):
  rng   = numpy.random.Generator(PCG64(190900562 + config_index))
  order = h_dec, h_enc, W_a, W_c, W_out, b_out, src_len, (tgt_len,) targets
  floats are drawn in float64, cast to float32 and, for the bf16 path,
  rounded once to bf16 (round-to-nearest-even); the rounded values are what
  both sides see.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

BASE_SEED = 190900562

# name -> recipe.  "index" is the position in the benchmark's config list.
CONFIGS: Dict[str, dict] = {
    "tiny": dict(index=0, B=4, S=8, T=8, H=64, V=1000, dtype="f32", w=0.1,
                 len_lo=1, len_hi=8, targets="uniform", zipf_s=None, force_max=False),
    "small": dict(index=1, B=64, S=30, T=30, H=512, V=16000, dtype="bf16", w=0.1,
                  len_lo=10, len_hi=30, targets="zipf", zipf_s=1.1, force_max=False),
    "mid": dict(index=2, B=128, S=50, T=50, H=1024, V=32000, dtype="bf16", w=0.1,
                len_lo=20, len_hi=50, targets="zipf", zipf_s=1.1, force_max=False),
    "large": dict(index=3, B=128, S=80, T=80, H=1024, V=64000, dtype="bf16", w=0.1,
                  len_lo=10, len_hi=80, targets="zipf", zipf_s=1.1, force_max=True),
    "stress": dict(index=4, B=256, S=64, T=64, H=2048, V=128000, dtype="bf16", w=0.05,
                   len_lo=32, len_hi=64, targets="zipf", zipf_s=1.05, force_max=False),
}

PAD_ID = 0


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bit patterns.

    Inputs here are finite, so NaN handling is not needed.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Inputs:
    """One batch of synthetic inputs.  Float arrays are float32 holding the
    values of the storage type (already bf16-representable when dtype == "bf16")."""
    name: str
    dtype: str            # "f32" or "bf16": storage type of states/weights on the GPU
    T: int
    S: int
    B: int
    H: int
    V: int
    pad_id: int
    h_dec: np.ndarray     # [T,B,H]
    h_enc: np.ndarray     # [S,B,H]
    src_len: np.ndarray   # [B] int32
    W_a: np.ndarray       # [H,H]
    W_c: np.ndarray       # [H,2H]
    W_out: np.ndarray     # [V,H]
    b_out: np.ndarray     # [V]
    targets: np.ndarray   # [T,B] int32
    grad_scale: float = 1.0
    dropout_p: float = 0.0   # rate of the dropout on the attentional state (0 = off) and its seed
    dropout_seed: int = 0
    extra: dict = field(default_factory=dict)

    FLOAT_FIELDS = ("h_dec", "h_enc", "W_a", "W_c", "W_out", "b_out")

    def slice_batch(self, b0: int, b1: int) -> "Inputs":
        """Sentences b0..b1-1 of this batch (weights shared)."""
        return Inputs(name=f"{self.name}[{b0}:{b1}]", dtype=self.dtype, T=self.T, S=self.S,
                      B=b1 - b0, H=self.H, V=self.V, pad_id=self.pad_id,
                      h_dec=np.ascontiguousarray(self.h_dec[:, b0:b1]),
                      h_enc=np.ascontiguousarray(self.h_enc[:, b0:b1]),
                      src_len=np.ascontiguousarray(self.src_len[b0:b1]),
                      W_a=self.W_a, W_c=self.W_c, W_out=self.W_out, b_out=self.b_out,
                      targets=np.ascontiguousarray(self.targets[:, b0:b1]),
                      grad_scale=self.grad_scale)

    def take_sentences(self, idx) -> "Inputs":
        """The listed sentences as a batch of their own (weights shared)."""
        idx = np.asarray(idx, dtype=np.int64)
        return Inputs(name=f"{self.name}[{len(idx)} sentences]", dtype=self.dtype, T=self.T, S=self.S,
                      B=len(idx), H=self.H, V=self.V, pad_id=self.pad_id,
                      h_dec=np.ascontiguousarray(self.h_dec[:, idx]),
                      h_enc=np.ascontiguousarray(self.h_enc[:, idx]),
                      src_len=np.ascontiguousarray(self.src_len[idx]),
                      W_a=self.W_a, W_c=self.W_c, W_out=self.W_out, b_out=self.b_out,
                      targets=np.ascontiguousarray(self.targets[:, idx]),
                      grad_scale=self.grad_scale)

    def n_nonpad(self) -> int:
        t = self.targets
        return int(np.count_nonzero((t != self.pad_id) & (t >= 0) & (t < self.V)))


def _zipf_cdf(V: int, s: float) -> np.ndarray:
    k = np.arange(1, V, dtype=np.float64)
    p = k ** (-s)
    c = np.cumsum(p)
    return c / c[-1]


def _round_storage(x64: np.ndarray, dtype: str) -> np.ndarray:
    x32 = x64.astype(np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x32))
    return x32


def make_inputs(name: str, dtype: Optional[str] = None, grad_scale: float = 1.0) -> Inputs:
    """Build the named configuration.  `dtype` overrides the configuration's
    storage type ("f32" / "bf16"); the random draws are the same either way."""
    cfg = CONFIGS[name]
    dtype = dtype or cfg["dtype"]
    if dtype not in ("f32", "bf16"):
        raise ValueError(f"unknown dtype {dtype!r}")
    T, S, B, H, V, w = cfg["T"], cfg["S"], cfg["B"], cfg["H"], cfg["V"], cfg["w"]
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + cfg["index"]))

    h_dec = _round_storage(np.tanh(rng.standard_normal((T, B, H))), dtype)
    h_enc = _round_storage(np.tanh(rng.standard_normal((S, B, H))), dtype)
    W_a = _round_storage(rng.uniform(-w, w, (H, H)), dtype)
    W_c = _round_storage(rng.uniform(-w, w, (H, 2 * H)), dtype)
    W_out = _round_storage(rng.uniform(-w, w, (V, H)), dtype)
    b_out = _round_storage(rng.uniform(-w, w, (V,)), dtype)

    lo, hi = cfg["len_lo"], cfg["len_hi"]
    src_len = rng.integers(lo, hi + 1, size=B).astype(np.int32)
    if cfg["targets"] == "uniform":
        # Tiny: ids uniform in 1..V-1, each position independently pad with prob 0.1.
        targets = rng.integers(1, V, size=(T, B)).astype(np.int32)
        pad = rng.random((T, B)) < 0.1
        targets[pad] = PAD_ID
    else:
        tgt_len = rng.integers(lo, hi + 1, size=B).astype(np.int32)
        if cfg["force_max"]:
            src_len[0] = hi
            tgt_len[0] = hi
        cdf = _zipf_cdf(V, cfg["zipf_s"])
        u = rng.random((T, B))
        ids = np.searchsorted(cdf, u, side="left") + 1      # rank k -> token id k
        ids = np.minimum(ids, V - 1)
        targets = ids.astype(np.int32)
        t_idx = np.arange(T, dtype=np.int32)[:, None]
        targets[t_idx >= tgt_len[None, :]] = PAD_ID
    if cfg["force_max"] and cfg["targets"] == "uniform":
        src_len[0] = hi

    return Inputs(name=name, dtype=dtype, T=T, S=S, B=B, H=H, V=V, pad_id=PAD_ID,
                  h_dec=h_dec, h_enc=h_enc, src_len=src_len, W_a=W_a, W_c=W_c,
                  W_out=W_out, b_out=b_out, targets=targets, grad_scale=grad_scale)


def make_custom(T: int, S: int, B: int, H: int, V: int, seed: int, dtype: str = "f32",
                w: float = 0.1, pad_prob: float = 0.15, min_len: int = 0,
                grad_scale: float = 1.0) -> Inputs:
    """Small ad-hoc shapes for edge-case tests (ragged tiles, empty sources...)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    h_dec = _round_storage(np.tanh(rng.standard_normal((T, B, H))), dtype)
    h_enc = _round_storage(np.tanh(rng.standard_normal((S, B, H))), dtype)
    W_a = _round_storage(rng.uniform(-w, w, (H, H)), dtype)
    W_c = _round_storage(rng.uniform(-w, w, (H, 2 * H)), dtype)
    W_out = _round_storage(rng.uniform(-w, w, (V, H)), dtype)
    b_out = _round_storage(rng.uniform(-w, w, (V,)), dtype)
    src_len = rng.integers(min_len, S + 1, size=B).astype(np.int32)
    targets = rng.integers(0, V, size=(T, B)).astype(np.int32)
    pad = rng.random((T, B)) < pad_prob
    targets[pad] = PAD_ID
    return Inputs(name=f"custom{seed}", dtype=dtype, T=T, S=S, B=B, H=H, V=V, pad_id=PAD_ID,
                  h_dec=h_dec, h_enc=h_enc, src_len=src_len, W_a=W_a, W_c=W_c,
                  W_out=W_out, b_out=b_out, targets=targets, grad_scale=grad_scale)


@dataclass
class LstmInputs:
    """One side (encoder or decoder) of the stacked LSTM: word embeddings of all steps, sentence lengths,
    per-layer weights, initial states, and the incoming gradients of a backward pass."""
    dtype: str
    T: int
    B: int
    I: int
    H: int
    L: int
    x: np.ndarray            # [T,B,I] embeddings
    lengths: np.ndarray      # [B]
    W_ih: list
    W_hh: list
    b: list
    h0: np.ndarray           # [L,B,H] float32
    c0: np.ndarray
    dy: np.ndarray           # [T,B,H] float32: gradient w.r.t. the top layer's outputs
    dhT: np.ndarray          # [L,B,H] float32: gradient w.r.t. the final states
    dcT: np.ndarray


def make_lstm_inputs(T: int, B: int, I: int, H: int, L: int, seed: int, dtype: str = "f32", w: float = 0.1,
                     min_len: int = 1, force_max: bool = True) -> LstmInputs:
    """Stand-in for a batch of embedded sentences (Table 2 of the paper: embedding 512, hidden 1024, depth 4):
    embeddings tanh(N(0,1)) like the hidden states of the other configurations, weights and biases U(-w, w),
    lengths uniform in min_len..T with sentence 0 at full length, initial states and incoming gradients
    N(0,1) scaled to 0.5 / 0.1.  Draw order: x, lengths, per layer (W_ih, W_hh, b), h0, c0, dy, dhT, dcT."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _round_storage(np.tanh(rng.standard_normal((T, B, I))), dtype)
    lengths = rng.integers(min_len, T + 1, size=B).astype(np.int32)
    if force_max:
        lengths[0] = T
    W_ih, W_hh, b = [], [], []
    for l in range(L):
        W_ih.append(_round_storage(rng.uniform(-w, w, (4 * H, I if l == 0 else H)), dtype))
        W_hh.append(_round_storage(rng.uniform(-w, w, (4 * H, H)), dtype))
        b.append(_round_storage(rng.uniform(-w, w, (4 * H,)), dtype))
    f32 = lambda a: a.astype(np.float32)
    h0 = f32(0.5 * rng.standard_normal((L, B, H)))
    c0 = f32(0.5 * rng.standard_normal((L, B, H)))
    dy = f32(0.1 * rng.standard_normal((T, B, H)))
    dhT = f32(0.1 * rng.standard_normal((L, B, H)))
    dcT = f32(0.1 * rng.standard_normal((L, B, H)))
    return LstmInputs(dtype=dtype, T=T, B=B, I=I, H=H, L=L, x=x, lengths=lengths, W_ih=W_ih, W_hh=W_hh, b=b,
                      h0=h0, c0=c0, dy=dy, dhT=dhT, dcT=dcT)
