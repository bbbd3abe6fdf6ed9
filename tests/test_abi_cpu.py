"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_1909_00562_amd as lib
from paper_1909_00562_amd import binding as bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b((?:attn_softmax|lstm_stack)_\w+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    handle = lib.load_library()
    names = _header_functions()
    assert set(names) == set(bd.EXPORTS)
    for n in names:
        assert getattr(handle, n) is not None


def _shape(**kw):
    d = dict(T=8, S=8, B=4, H=64, V=1000, pad_id=0, dtype=bd.AS_F32, grad_scale=1.0)
    d.update(kw)
    return bd.AsShape(d["T"], d["S"], d["B"], d["H"], d["V"], d["pad_id"], d["dtype"], d["grad_scale"])


def test_workspace_bytes():
    assert bd.attn_softmax_workspace_bytes(_shape()) > 0
    assert bd.attn_softmax_workspace_bytes(_shape(T=0)) == 0
    assert bd.attn_softmax_workspace_bytes(_shape(pad_id=1000)) == 0
    assert bd.attn_softmax_workspace_bytes(_shape(dtype=7)) == 0
    assert bd.attn_softmax_workspace_bytes(_shape(dtype=bd.AS_BF16, H=60)) == 0
    small = bd.attn_softmax_workspace_bytes(_shape(dtype=bd.AS_BF16))
    big = bd.attn_softmax_workspace_bytes(_shape(dtype=bd.AS_BF16, V=2000))
    assert big > small
    # the stress configuration: logits dominate (N * V * 2 bytes = 4.19 GB)
    s = _shape(T=64, S=64, B=256, H=2048, V=128000, dtype=bd.AS_BF16)
    assert 4.19e9 < bd.attn_softmax_workspace_bytes(s) < 6e9


def _call_fwd(shape, ptrs=None, ws_bytes=1 << 40, **over):
    # fake, 16-byte aligned, never dereferenced addresses: every check below fails before a launch
    a = dict(h_dec=0x1000, h_enc=0x2000, src_len=0x3000, W_a=0x4000, W_c=0x5000, W_out=0x6000, b_out=0x7000,
             targets=0x8000, loss_sum=0x9000, n_tok=0xA000, tok_loss=None, argmax=None, attn_mask=None,
             tgt_mask=None, workspace=0xB000)
    a.update(over)
    return bd.attn_softmax_fwd(shape, a["h_dec"], a["h_enc"], a["src_len"], a["W_a"], a["W_c"], a["W_out"],
                               a["b_out"], a["targets"], a["loss_sum"], a["n_tok"], a["tok_loss"], a["argmax"],
                               a["attn_mask"], a["tgt_mask"], a["workspace"], ws_bytes, 0, check=False)


def _call_bwd(shape, ws_bytes=1 << 40, **over):
    a = dict(h_dec=0x1000, h_enc=0x2000, src_len=0x3000, W_a=0x4000, W_c=0x5000, W_out=0x6000, b_out=0x7000,
             targets=0x8000, workspace=0xB000, d_h_dec=0xC000, d_h_enc=0xD000, dW_a=0xE000, dW_c=0xF000,
             dW_out=0x10000, db_out=0x11000)
    a.update(over)
    return bd.attn_softmax_bwd(shape, a["h_dec"], a["h_enc"], a["src_len"], a["W_a"], a["W_c"], a["W_out"],
                               a["b_out"], a["targets"], a["workspace"], ws_bytes, a["d_h_dec"], a["d_h_enc"],
                               a["dW_a"], a["dW_c"], a["dW_out"], a["db_out"], 0, check=False)


def test_fwd_rejects_bad_arguments_before_launch():
    assert _call_fwd(None) == 1                                   # AS_ERR_NULL
    assert _call_fwd(_shape(), h_enc=None) == 1
    assert _call_fwd(_shape(), loss_sum=None) == 1
    assert "NULL" in bd.attn_softmax_last_error()
    assert _call_fwd(_shape(S=0)) == 2                            # AS_ERR_SHAPE
    assert _call_fwd(_shape(pad_id=-1)) == 2
    assert _call_fwd(_shape(dtype=5)) == 3                        # AS_ERR_DTYPE
    assert _call_fwd(_shape(), ws_bytes=128) == 4                 # AS_ERR_WORKSPACE
    assert "needed" in bd.attn_softmax_last_error()
    assert _call_fwd(_shape(), W_out=0x6004) == 5                 # AS_ERR_ALIGN
    assert _call_fwd(_shape(dtype=bd.AS_BF16, H=60)) == 5


def test_bwd_rejects_bad_arguments_before_launch():
    assert _call_bwd(None) == 1
    assert _call_bwd(_shape(), dW_out=None) == 1
    assert _call_bwd(_shape(V=0)) == 2
    assert _call_bwd(_shape(dtype=-1)) == 3
    assert _call_bwd(_shape(), ws_bytes=0) == 4
    assert _call_bwd(_shape(), db_out=0x11008) == 5


def test_view_offsets_are_inside_the_workspace():
    s = _shape(dtype=bd.AS_BF16, V=1003)
    n = bd.attn_softmax_workspace_bytes(s)
    base = 0x100000
    seen = []
    for which in range(5):
        addr, nbytes, ld = bd.attn_softmax_view(s, base, which)
        assert base <= addr and addr + nbytes <= base + n and addr % 16 == 0
        seen.append((addr, addr + nbytes))
        if which == bd.AS_VIEW_LOGITS:
            assert ld == 1008                                     # rows padded to a multiple of 8
    seen.sort()
    for (a0, a1), (b0, b1) in zip(seen, seen[1:]):
        assert a1 <= b0                                           # views do not overlap
    with pytest.raises(bd.AttnSoftmaxError):
        bd.attn_softmax_view(s, base, 99)


def test_profile_calls_work_without_a_device():
    bd.attn_softmax_profile_enable(False)
    r = bd.attn_softmax_profile_read()
    assert set(r) == set(bd.STAGE_NAMES) and all(v["launches"] == 0 for v in r.values())


def test_dropout_rate_is_validated():
    s = _shape()
    s.dropout_p = 0.3
    s.dropout_seed = 2 ** 63 + 5
    assert bd.attn_softmax_workspace_bytes(s) == bd.attn_softmax_workspace_bytes(_shape())
    for bad in (1.0, -0.1, float("nan")):
        s.dropout_p = bad
        assert bd.attn_softmax_workspace_bytes(s) == 0
        assert _call_fwd(s) == 2


def test_adam_rejects_bad_arguments_before_any_launch():
    ok = bd.AsAdam(1e-3, 0.9, 0.999, 1e-8, 1)
    call = lambda hp, n=64, grad=0x1000, master=0x2000, m=0x3000, v=0x4000, out=None, dtype=bd.AS_F32: \
        bd.attn_softmax_adam_step(hp, n, grad, master, m, v, out, dtype, 0, check=False)
    assert call(None) == 1
    assert call(ok, grad=None) == 1 and call(ok, v=None) == 1
    assert call(ok, n=0) == 2
    assert call(bd.AsAdam(1e-3, 0.9, 0.999, 1e-8, 0)) == 2
    assert call(bd.AsAdam(1e-3, 1.0, 0.999, 1e-8, 1)) == 2
    assert call(bd.AsAdam(1e-3, 0.9, -0.5, 1e-8, 1)) == 2
    assert call(ok, out=0x5000, dtype=9) == 3
    assert call(ok, m=0x3004) == 5


def test_step_mode_rejects_bad_arguments():
    s = bd.AsShape(1, 8, 4, 64, 100, 0, bd.AS_F32, 1.0, 0.0, 0)
    n = lib.attn_softmax_step_workspace_bytes(s)
    assert n > lib.attn_softmax_workspace_bytes(s)          # the cached K' comes on top
    assert lib.attn_softmax_step_workspace_bytes(bd.AsShape(1, 8, 4, 60, 100, 0, bd.AS_BF16, 1.0, 0.0, 0)) == 0
    assert lib.attn_softmax_step_prepare(s, 0x1000, 0x2000, 0x3000, n - 1, 0, check=False) == 4
    assert lib.attn_softmax_step_prepare(s, None, 0x2000, 0x3000, n, 0, check=False) == 1
    # h_t missing, workspace too small, misaligned pointer: refused before any launch
    args = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 0x8000, 0x9000, None, None, 0xA000]
    assert lib.attn_softmax_step_fwd(s, None, *args[1:], n, 0, check=False) == 1
    assert lib.attn_softmax_step_fwd(s, *args, n - 1, 0, check=False) == 4
    assert lib.attn_softmax_step_fwd(s, 0x1004, *args[1:], n, 0, check=False) == 5


# ---------------------------------------------------------------- lstm_stack_*
def _ls(**kw):
    d = dict(T=5, B=3, I=16, H=8, L=2, dtype=bd.AS_F32)
    d.update(kw)
    return bd.LsShape(d["T"], d["B"], d["I"], d["H"], d["L"], d["dtype"])


def test_lstm_workspace_bytes():
    assert bd.lstm_stack_workspace_bytes(_ls()) > 0
    for bad in (dict(T=0), dict(B=0), dict(I=0), dict(H=0), dict(L=0), dict(L=17), dict(dtype=5),
                dict(dtype=bd.AS_BF16, H=12), dict(dtype=bd.AS_BF16, I=12)):
        assert bd.lstm_stack_workspace_bytes(_ls(**bad)) == 0, bad
    assert bd.lstm_stack_workspace_bytes(_ls(L=4)) > bd.lstm_stack_workspace_bytes(_ls(L=2))
    for p_drop, ok in ((0.3, True), (0.0, True), (1.0, False), (-0.1, False)):
        sh = _ls()
        sh.dropout_p = p_drop
        assert (bd.lstm_stack_workspace_bytes(sh) > 0) == ok, p_drop


def test_lstm_rejects_bad_arguments_before_any_launch():
    # fake, aligned, never dereferenced device addresses
    sh = _ls()
    W = [0x1000, 0x2000]
    ok = dict(x=0x100, lengths=0x200, W_ih=W, W_hh=W, b=W, h0=None, c0=None, y=0x300, hT=None, cT=None,
              workspace=0x400, workspace_bytes=1 << 40)

    def fwd(shape=sh, **over):
        a = dict(ok)
        a.update(over)
        return bd.lstm_stack_fwd(shape, a["x"], a["lengths"], a["W_ih"], a["W_hh"], a["b"], a["h0"], a["c0"], a["y"],
                                 a["hT"], a["cT"], a["workspace"], a["workspace_bytes"], 0, check=False)

    assert fwd(shape=_ls(T=0)) == 2 and "bad shape" in bd.attn_softmax_last_error()
    assert fwd(shape=_ls(dtype=9)) == 3
    assert fwd(shape=_ls(dtype=bd.AS_BF16, H=12)) == 5
    assert fwd(x=None) == 1
    assert fwd(W_hh=None) == 1
    assert fwd(W_ih=[0x1000, None]) == 1
    assert fwd(b=[0x1000, 0x2004]) == 5
    assert fwd(y=0x301) == 5
    assert fwd(workspace_bytes=16) == 4
    rc = bd.lstm_stack_bwd(sh, 0x100, 0x200, W, W, None, None, None, 0x400, 1 << 40, 0x500, W, W, W, None, None, 0,
                           check=False)
    assert rc == 1                                       # dy is required
    rc = bd.lstm_stack_bwd(sh, 0x100, 0x200, W, W, 0x600, None, None, 0x400, 1 << 40, 0x500, W, None, W, None, None, 0,
                           check=False)
    assert rc == 1                                       # dW_hh is required


# ---------------------------------------------------------------- skip_pad_rows
def test_skip_pad_rows_is_validated_and_sizes_the_workspace():
    s0 = _shape(dtype=bd.AS_BF16)
    s1 = _shape(dtype=bd.AS_BF16)
    s1.skip_pad_rows = 1
    assert bd.attn_softmax_workspace_bytes(s1) > bd.attn_softmax_workspace_bytes(s0) > 0
    bad = _shape(dtype=bd.AS_BF16)
    bad.skip_pad_rows = 2
    assert bd.attn_softmax_workspace_bytes(bad) == 0
    assert _call_fwd(bad) == 2 and "skip_pad_rows=2" in bd.attn_softmax_last_error()
    # the row map exists only with row compaction
    p, n, ld = ctypes.c_void_p(), ctypes.c_size_t(), ctypes.c_int64()
    h = lib.load_library()
    rc = h.attn_softmax_view(ctypes.byref(s0), 0xB000, bd.AS_VIEW_ROW_POS, ctypes.byref(p), ctypes.byref(n),
                             ctypes.byref(ld))
    assert rc == 2
    rc = h.attn_softmax_view(ctypes.byref(s1), 0xB000, bd.AS_VIEW_ROW_POS, ctypes.byref(p), ctypes.byref(n),
                             ctypes.byref(ld))
    assert rc == 0 and n.value == s1.T * s1.B * 4 and ld.value == s1.B
    # the per-step entry points ignore the flag
    assert bd.attn_softmax_step_workspace_bytes(s1) == bd.attn_softmax_step_workspace_bytes(s0)


def test_fwd_static_rejects_on_the_host_before_any_hip_call():
    """The allocation-free forward entry point: argument errors and shapes beyond the library's static scratch
    are turned away on the host (this runs without a GPU)."""
    a = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 0x8000, 0x9000, 0xA000, None, None, None, None]
    big = _shape(T=4, S=50, B=128, H=1024, V=32000, dtype=bd.AS_BF16)
    assert bd.attn_softmax_workspace_bytes(big) > bd.AS_STATIC_SCRATCH_BYTES
    assert bd.attn_softmax_fwd_static(big, *a, 0, check=False) == 4          # AS_ERR_WORKSPACE
    assert "static scratch" in bd.attn_softmax_last_error()
    assert bd.attn_softmax_fwd_static(None, *a, 0, check=False) == 1         # AS_ERR_NULL
    ok = _shape(T=1, S=50, B=128, H=1024, V=32000, dtype=bd.AS_BF16)
    assert bd.attn_softmax_workspace_bytes(ok) <= bd.AS_STATIC_SCRATCH_BYTES
    b = list(a)
    b[8] = None                                                              # loss_sum
    assert bd.attn_softmax_fwd_static(ok, *b, 0, check=False) == 1
    b = list(a)
    b[0] = 0x1004                                                            # misaligned h_dec
    assert bd.attn_softmax_fwd_static(ok, *b, 0, check=False) == 5           # AS_ERR_ALIGN
    assert bd.attn_softmax_fwd_static(_shape(dtype=9), *a, 0, check=False) == 3
