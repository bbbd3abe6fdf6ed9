"""ctypes binding of include/attn_softmax.h: same names, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in
the HIP library.  There is no fallback: if libattn_softmax.so is missing the
first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libattn_softmax.so")
_lib = None

AS_F32, AS_BF16 = 0, 1
AS_VIEW_ALPHA, AS_VIEW_CTX, AS_VIEW_HC, AS_VIEW_LOGITS, AS_VIEW_LSE, AS_VIEW_ROW_POS = range(6)
STATUS_NAMES = {0: "AS_OK", 1: "AS_ERR_NULL", 2: "AS_ERR_SHAPE", 3: "AS_ERR_DTYPE",
                4: "AS_ERR_WORKSPACE", 5: "AS_ERR_ALIGN", 6: "AS_ERR_HIP"}
STAGE_NAMES = ["gemm_q", "attn_score", "attn_softmax", "attn_ctx", "gemm_hc", "gemm_logits",
               "xent_stats", "xent_dlogits", "gemm_dwout", "gemm_dhc", "gemm_dwc", "gemm_dch",
               "attn_bwd", "attn_softmax_bwd", "gemm_dwa", "gemm_dh", "misc", "adam", "compact"]
AS_STATIC_SCRATCH_BYTES = 64 << 20
EXPORTS = ["attn_softmax_workspace_bytes", "attn_softmax_fwd", "attn_softmax_fwd_static", "attn_softmax_bwd", "attn_softmax_view",
           "attn_softmax_last_error", "attn_softmax_profile_enable", "attn_softmax_profile_read",
           "attn_softmax_profile_select", "attn_softmax_stream_probe",
           "attn_softmax_adam_step", "attn_softmax_step_workspace_bytes", "attn_softmax_step_prepare",
           "attn_softmax_step_fwd", "lstm_stack_workspace_bytes", "lstm_stack_fwd", "lstm_stack_bwd"]


class AttnSoftmaxError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(code, code)}: {msg}")
        self.code = code


class AsShape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("S", ctypes.c_int32), ("B", ctypes.c_int32),
                ("H", ctypes.c_int32), ("V", ctypes.c_int32), ("pad_id", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("grad_scale", ctypes.c_float),
                ("dropout_p", ctypes.c_float), ("dropout_seed", ctypes.c_uint64),
                ("skip_pad_rows", ctypes.c_int32)]


class LsShape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("B", ctypes.c_int32), ("I", ctypes.c_int32), ("H", ctypes.c_int32),
                ("L", ctypes.c_int32), ("dtype", ctypes.c_int32), ("dropout_p", ctypes.c_float),
                ("dropout_seed", ctypes.c_uint64)]


class AsAdam(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("step", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libattn_softmax.so (built by `python -m paper_1909_00562_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with __graft_entry__.build() "
                           "or `python paper_1909_00562_amd/build.py`; there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    lib.attn_softmax_workspace_bytes.restype = sz
    lib.attn_softmax_workspace_bytes.argtypes = [ctypes.POINTER(AsShape)]
    lib.attn_softmax_fwd.restype = ctypes.c_int
    lib.attn_softmax_fwd.argtypes = [ctypes.POINTER(AsShape)] + [vp] * 14 + [vp, sz, vp]
    lib.attn_softmax_fwd_static.restype = ctypes.c_int
    lib.attn_softmax_fwd_static.argtypes = [ctypes.POINTER(AsShape)] + [vp] * 14 + [vp]
    lib.attn_softmax_bwd.restype = ctypes.c_int
    lib.attn_softmax_bwd.argtypes = [ctypes.POINTER(AsShape)] + [vp] * 8 + [vp, sz] + [vp] * 6 + [vp]
    lib.attn_softmax_view.restype = ctypes.c_int
    lib.attn_softmax_view.argtypes = [ctypes.POINTER(AsShape), vp, ctypes.c_int, ctypes.POINTER(vp),
                                      ctypes.POINTER(sz), ctypes.POINTER(ctypes.c_int64)]
    lib.attn_softmax_last_error.restype = ctypes.c_char_p
    lib.attn_softmax_last_error.argtypes = []
    lib.attn_softmax_profile_enable.restype = ctypes.c_int
    lib.attn_softmax_profile_enable.argtypes = [ctypes.c_int]
    lib.attn_softmax_profile_select.restype = ctypes.c_int
    lib.attn_softmax_profile_select.argtypes = [ctypes.c_uint64]
    lib.attn_softmax_profile_read.restype = ctypes.c_int
    lib.attn_softmax_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.attn_softmax_stream_probe.restype = ctypes.c_int
    lib.attn_softmax_stream_probe.argtypes = [ctypes.c_int, vp, vp, ctypes.c_int32, sz, vp]
    lib.attn_softmax_step_workspace_bytes.restype = sz
    lib.attn_softmax_step_workspace_bytes.argtypes = [ctypes.POINTER(AsShape)]
    lib.attn_softmax_step_prepare.restype = ctypes.c_int
    lib.attn_softmax_step_prepare.argtypes = [ctypes.POINTER(AsShape), vp, vp, vp, sz, vp]
    lib.attn_softmax_step_fwd.restype = ctypes.c_int
    lib.attn_softmax_step_fwd.argtypes = [ctypes.POINTER(AsShape)] + [vp] * 11 + [vp, sz, vp]
    lib.attn_softmax_adam_step.restype = ctypes.c_int
    lib.attn_softmax_adam_step.argtypes = [ctypes.POINTER(AsAdam), sz, vp, vp, vp, vp, vp, ctypes.c_int32, vp]
    lib.lstm_stack_workspace_bytes.restype = sz
    lib.lstm_stack_workspace_bytes.argtypes = [ctypes.POINTER(LsShape)]
    lib.lstm_stack_fwd.restype = ctypes.c_int
    lib.lstm_stack_fwd.argtypes = [ctypes.POINTER(LsShape)] + [vp] * 10 + [vp, sz, vp]
    lib.lstm_stack_bwd.restype = ctypes.c_int
    lib.lstm_stack_bwd.argtypes = [ctypes.POINTER(LsShape)] + [vp] * 7 + [vp, sz] + [vp] * 6 + [vp]
    _lib = lib
    return lib


def _ptr(x) -> Optional[int]:
    """Device/host address of a torch tensor, an int address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _check(code: int):
    if code != 0:
        raise AttnSoftmaxError(code, attn_softmax_last_error())


def attn_softmax_last_error() -> str:
    return load_library().attn_softmax_last_error().decode()


def attn_softmax_workspace_bytes(shape: AsShape) -> int:
    return int(load_library().attn_softmax_workspace_bytes(ctypes.byref(shape)))


def attn_softmax_fwd(shape, h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, loss_sum, n_tok,
                     tok_loss, argmax, attn_mask, tgt_mask, workspace, workspace_bytes, stream=0, check=True) -> int:
    rc = load_library().attn_softmax_fwd(
        ctypes.byref(shape) if shape is not None else None,
        _ptr(h_dec), _ptr(h_enc), _ptr(src_len), _ptr(W_a), _ptr(W_c), _ptr(W_out), _ptr(b_out), _ptr(targets),
        _ptr(loss_sum), _ptr(n_tok), _ptr(tok_loss), _ptr(argmax), _ptr(attn_mask), _ptr(tgt_mask),
        _ptr(workspace), int(workspace_bytes), stream or None)
    if check:
        _check(rc)
    return rc


def attn_softmax_fwd_static(shape, h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, loss_sum, n_tok,
                            tok_loss, argmax, attn_mask, tgt_mask, stream=0, check=True) -> int:
    """attn_softmax_fwd on the library's own static scratch (no workspace argument, nothing allocated)."""
    rc = load_library().attn_softmax_fwd_static(
        ctypes.byref(shape) if shape is not None else None,
        _ptr(h_dec), _ptr(h_enc), _ptr(src_len), _ptr(W_a), _ptr(W_c), _ptr(W_out), _ptr(b_out), _ptr(targets),
        _ptr(loss_sum), _ptr(n_tok), _ptr(tok_loss), _ptr(argmax), _ptr(attn_mask), _ptr(tgt_mask), stream or None)
    if check:
        _check(rc)
    return rc


def attn_softmax_bwd(shape, h_dec, h_enc, src_len, W_a, W_c, W_out, b_out, targets, workspace, workspace_bytes,
                     d_h_dec, d_h_enc, dW_a, dW_c, dW_out, db_out, stream=0, check=True) -> int:
    rc = load_library().attn_softmax_bwd(
        ctypes.byref(shape) if shape is not None else None,
        _ptr(h_dec), _ptr(h_enc), _ptr(src_len), _ptr(W_a), _ptr(W_c), _ptr(W_out), _ptr(b_out), _ptr(targets),
        _ptr(workspace), int(workspace_bytes),
        _ptr(d_h_dec), _ptr(d_h_enc), _ptr(dW_a), _ptr(dW_c), _ptr(dW_out), _ptr(db_out), stream or None)
    if check:
        _check(rc)
    return rc


def attn_softmax_view(shape, workspace, which: int):
    """Returns (address, bytes, row_stride_elements) of a saved activation."""
    p, n, ld = ctypes.c_void_p(), ctypes.c_size_t(), ctypes.c_int64()
    _check(load_library().attn_softmax_view(ctypes.byref(shape), _ptr(workspace), which, ctypes.byref(p),
                                            ctypes.byref(n), ctypes.byref(ld)))
    return int(p.value), int(n.value), int(ld.value)


def attn_softmax_step_workspace_bytes(shape: AsShape) -> int:
    return int(load_library().attn_softmax_step_workspace_bytes(ctypes.byref(shape)))


def attn_softmax_step_prepare(shape, h_enc, W_a, workspace, workspace_bytes, stream=0, check=True) -> int:
    rc = load_library().attn_softmax_step_prepare(ctypes.byref(shape) if shape is not None else None, _ptr(h_enc),
                                                  _ptr(W_a), _ptr(workspace), workspace_bytes, stream)
    if check:
        _check(rc)
    return rc


def attn_softmax_step_fwd(shape, h_t, h_enc, src_len, W_c, W_out, b_out, targets, loss_sum, n_tok, tok_loss,
                          argmax, workspace, workspace_bytes, stream=0, check=True) -> int:
    rc = load_library().attn_softmax_step_fwd(ctypes.byref(shape) if shape is not None else None, _ptr(h_t),
                                              _ptr(h_enc), _ptr(src_len), _ptr(W_c), _ptr(W_out), _ptr(b_out),
                                              _ptr(targets), _ptr(loss_sum), _ptr(n_tok), _ptr(tok_loss),
                                              _ptr(argmax), _ptr(workspace), workspace_bytes, stream)
    if check:
        _check(rc)
    return rc


def attn_softmax_adam_step(hyper: AsAdam, n: int, grad, master, m, v, weights_out, dtype: int, stream: int = 0,
                           check=True) -> int:
    rc = load_library().attn_softmax_adam_step(ctypes.byref(hyper) if hyper is not None else None, n, _ptr(grad),
                                               _ptr(master), _ptr(m), _ptr(v), _ptr(weights_out), dtype, stream)
    if check:
        _check(rc)
    return rc


def _ptr_array(tensors):
    """Host array of device addresses (one per layer); None stays NULL."""
    if tensors is None:
        return None
    arr = (ctypes.c_void_p * len(tensors))(*[_ptr(t) for t in tensors])
    return ctypes.cast(arr, ctypes.c_void_p), arr      # the second element keeps the array alive


def lstm_stack_workspace_bytes(shape: LsShape) -> int:
    return int(load_library().lstm_stack_workspace_bytes(ctypes.byref(shape)))


def lstm_stack_fwd(shape, x, lengths, W_ih, W_hh, b, h0, c0, y, hT, cT, workspace, workspace_bytes, stream=0,
                   check=True) -> int:
    """W_ih, W_hh, b: sequences of L device tensors (or addresses)."""
    arrs = [_ptr_array(a) for a in (W_ih, W_hh, b)]
    rc = load_library().lstm_stack_fwd(ctypes.byref(shape) if shape is not None else None, _ptr(x), _ptr(lengths),
                                       *[a[0] if a else None for a in arrs], _ptr(h0), _ptr(c0), _ptr(y), _ptr(hT),
                                       _ptr(cT), _ptr(workspace), int(workspace_bytes), stream or None)
    if check:
        _check(rc)
    return rc


def lstm_stack_bwd(shape, x, lengths, W_ih, W_hh, dy, dhT, dcT, workspace, workspace_bytes, dx, dW_ih, dW_hh, db,
                   dh0, dc0, stream=0, check=True) -> int:
    ins = [_ptr_array(a) for a in (W_ih, W_hh)]
    outs = [_ptr_array(a) for a in (dW_ih, dW_hh, db)]
    rc = load_library().lstm_stack_bwd(ctypes.byref(shape) if shape is not None else None, _ptr(x), _ptr(lengths),
                                       *[a[0] if a else None for a in ins], _ptr(dy), _ptr(dhT), _ptr(dcT),
                                       _ptr(workspace), int(workspace_bytes), _ptr(dx),
                                       *[a[0] if a else None for a in outs], _ptr(dh0), _ptr(dc0), stream or None)
    if check:
        _check(rc)
    return rc


def attn_softmax_stream_probe(kind: int, buf, buf2, rows: int, row_bytes: int, stream=0, check=True) -> int:
    rc = load_library().attn_softmax_stream_probe(int(kind), _ptr(buf), _ptr(buf2), int(rows), int(row_bytes),
                                                  stream or None)
    if check:
        _check(rc)
    return rc


def attn_softmax_profile_enable(enable: bool):
    _check(load_library().attn_softmax_profile_enable(1 if enable else 0))


def attn_softmax_profile_select(stages) -> None:
    """Time only the named stages (names as in STAGE_NAMES) until profiling is enabled again."""
    mask = 0
    for name in stages:
        mask |= 1 << STAGE_NAMES.index(name)
    _check(load_library().attn_softmax_profile_select(mask))


def attn_softmax_profile_read() -> Dict[str, dict]:
    n = len(STAGE_NAMES)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _check(load_library().attn_softmax_profile_read(ms, cnt))
    return {STAGE_NAMES[i]: {"ms": ms[i], "launches": int(cnt[i])} for i in range(n)}


class DeviceBatch:
    """Device buffers for one batch: uploads the inputs, owns outputs and the
    workspace, and forwards to the C ABI.  No arithmetic happens here."""

    def __init__(self, inp, device="cuda:0", skip_pad_rows=False):
        import torch
        self.torch = torch
        self.inp = inp
        self.dev = torch.device(device)
        bf = inp.dtype == "bf16"
        self.shape = AsShape(inp.T, inp.S, inp.B, inp.H, inp.V, inp.pad_id, AS_BF16 if bf else AS_F32,
                             float(inp.grad_scale), float(getattr(inp, "dropout_p", 0.0)),
                             int(getattr(inp, "dropout_seed", 0)), 1 if skip_pad_rows else 0)
        tdt = torch.bfloat16 if bf else torch.float32
        self.tdt = tdt

        def up(a):   # values are already representable in the storage type
            return torch.from_numpy(np.ascontiguousarray(a)).to(tdt).to(self.dev)

        self.h_dec, self.h_enc = up(inp.h_dec), up(inp.h_enc)
        self.W_a, self.W_c, self.W_out, self.b_out = up(inp.W_a), up(inp.W_c), up(inp.W_out), up(inp.b_out)
        self.src_len = torch.from_numpy(inp.src_len.astype(np.int32)).to(self.dev)
        self.targets = torch.from_numpy(np.ascontiguousarray(inp.targets, dtype=np.int32)).to(self.dev)
        T, S, B, H, V = inp.T, inp.S, inp.B, inp.H, inp.V
        f32, i32, u8 = torch.float32, torch.int32, torch.uint8
        self.loss_sum = torch.zeros(1, dtype=f32, device=self.dev)
        self.n_tok = torch.zeros(1, dtype=i32, device=self.dev)
        self.tok_loss = torch.zeros(T, B, dtype=f32, device=self.dev)
        self.argmax = torch.zeros(T, B, dtype=i32, device=self.dev)
        self.attn_mask = torch.zeros(B, S, dtype=u8, device=self.dev)
        self.tgt_mask = torch.zeros(T, B, dtype=u8, device=self.dev)
        self.ws_bytes = attn_softmax_workspace_bytes(self.shape)
        if self.ws_bytes == 0:
            raise AttnSoftmaxError(2, "invalid shape for workspace")
        self.workspace = torch.empty(self.ws_bytes, dtype=u8, device=self.dev)
        self.d_h_dec = torch.empty(T, B, H, dtype=f32, device=self.dev)
        self.d_h_enc = torch.empty(S, B, H, dtype=f32, device=self.dev)
        self.dW_a = torch.empty(H, H, dtype=f32, device=self.dev)
        self.dW_c = torch.empty(H, 2 * H, dtype=f32, device=self.dev)
        self.dW_out = torch.empty(V, H, dtype=f32, device=self.dev)
        self.db_out = torch.empty(V, dtype=f32, device=self.dev)

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream(self.dev).cuda_stream)

    def fwd(self):
        attn_softmax_fwd(self.shape, self.h_dec, self.h_enc, self.src_len, self.W_a, self.W_c, self.W_out,
                         self.b_out, self.targets, self.loss_sum, self.n_tok, self.tok_loss, self.argmax,
                         self.attn_mask, self.tgt_mask, self.workspace, self.ws_bytes, self._stream())

    def bwd(self):
        attn_softmax_bwd(self.shape, self.h_dec, self.h_enc, self.src_len, self.W_a, self.W_c, self.W_out,
                         self.b_out, self.targets, self.workspace, self.ws_bytes, self.d_h_dec, self.d_h_enc,
                         self.dW_a, self.dW_c, self.dW_out, self.db_out, self._stream())

    def view(self, which: int):
        """Saved activation as a torch tensor aliasing the workspace.  With skip_pad_rows the logits and lse
        views are [N, V] / [N] with one row per non-pad position (AS_VIEW_ROW_POS maps (t, b) to its row)."""
        torch = self.torch
        addr, nbytes, ld = attn_softmax_view(self.shape, self.workspace, which)
        off = addr - self.workspace.data_ptr()
        raw = self.workspace[off:off + nbytes]
        T, S, B, H, V = self.inp.T, self.inp.S, self.inp.B, self.inp.H, self.inp.V
        if which == AS_VIEW_ALPHA:
            return raw.view(torch.float32).view(B, T, S)
        compact = self.shape.skip_pad_rows != 0
        if which == AS_VIEW_ROW_POS:
            return raw.view(torch.int32).view(T, B)
        if which == AS_VIEW_LSE:
            return raw.view(torch.float32).view(T * B) if compact else raw.view(torch.float32).view(T, B)
        if which in (AS_VIEW_CTX, AS_VIEW_HC):
            return raw.view(self.tdt).view(T, B, H)
        if which == AS_VIEW_LOGITS:
            if compact:
                return raw.view(self.tdt).view(T * B, ld)[:, :V]
            return raw.view(self.tdt).view(T, B, ld)[:, :, :V]
        raise ValueError(which)

    def sync(self):
        self.torch.cuda.synchronize(self.dev)


class DeviceLstm:
    """Device buffers for one side (encoder or decoder) of the stacked LSTM: uploads the inputs, owns the
    outputs and the workspace, and forwards to the C ABI.  No arithmetic happens here.
    x [T,B,I], lengths [B], W_ih / W_hh / b: lists of L arrays, h0 / c0 [L,B,H] or None (numpy, values already
    representable in the storage type)."""

    def __init__(self, x, lengths, W_ih, W_hh, b, h0=None, c0=None, dtype="f32", device="cuda:0", dropout_p=0.0,
                 dropout_seed=0):
        import torch
        self.torch = torch
        self.dev = torch.device(device)
        bf = dtype == "bf16"
        tdt = torch.bfloat16 if bf else torch.float32
        self.tdt = tdt
        T, B, I = x.shape
        L, H = len(W_ih), W_hh[0].shape[1]
        self.T, self.B, self.I, self.H, self.L = T, B, I, H, L
        self.shape = LsShape(T, B, I, H, L, AS_BF16 if bf else AS_F32, float(dropout_p), int(dropout_seed))
        f32 = torch.float32

        def up(a, dt=tdt):
            return torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(self.dev)

        self.x = up(x)
        self.lengths = torch.from_numpy(np.asarray(lengths, dtype=np.int32)).to(self.dev)
        self.W_ih = [up(w) for w in W_ih]
        self.W_hh = [up(w) for w in W_hh]
        self.b = [up(v) for v in b]
        self.h0 = up(h0, f32) if h0 is not None else None
        self.c0 = up(c0, f32) if c0 is not None else None
        self.y = torch.empty(T, B, H, dtype=tdt, device=self.dev)
        self.hT = torch.empty(L, B, H, dtype=f32, device=self.dev)
        self.cT = torch.empty(L, B, H, dtype=f32, device=self.dev)
        self.ws_bytes = lstm_stack_workspace_bytes(self.shape)
        if self.ws_bytes == 0:
            raise AttnSoftmaxError(2, "invalid shape for the LSTM workspace")
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        self.dx = torch.empty(T, B, I, dtype=f32, device=self.dev)
        self.dW_ih = [torch.empty(w.shape, dtype=f32, device=self.dev) for w in self.W_ih]
        self.dW_hh = [torch.empty(w.shape, dtype=f32, device=self.dev) for w in self.W_hh]
        self.db = [torch.empty(v.shape, dtype=f32, device=self.dev) for v in self.b]
        self.dh0 = torch.empty(L, B, H, dtype=f32, device=self.dev)
        self.dc0 = torch.empty(L, B, H, dtype=f32, device=self.dev)

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream(self.dev).cuda_stream)

    def fwd(self):
        lstm_stack_fwd(self.shape, self.x, self.lengths, self.W_ih, self.W_hh, self.b, self.h0, self.c0, self.y,
                       self.hT, self.cT, self.workspace, self.ws_bytes, self._stream())

    def bwd(self, dy, dhT=None, dcT=None):
        """dy [T,B,H], dhT / dcT [L,B,H]: float32 device tensors (or None)."""
        lstm_stack_bwd(self.shape, self.x, self.lengths, self.W_ih, self.W_hh, dy, dhT, dcT, self.workspace,
                       self.ws_bytes, self.dx, self.dW_ih, self.dW_hh, self.db, self.dh0, self.dc0, self._stream())

    def sync(self):
        self.torch.cuda.synchronize(self.dev)
