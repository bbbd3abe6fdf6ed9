"""MI355X-native attention-softmax forward/backward (section 3.2 of the hybrid
data-model parallel Seq2Seq RNN MT paper), and the stacked-LSTM part that feeds
it, as a C-ABI HIP library plus this thin ctypes binding.  Importing the package does not load the library; the first
call does, and fails loudly if it has not been built."""
from .binding import (  # noqa: F401
    AS_BF16, AS_F32, STAGE_NAMES, AsAdam, AsShape, AttnSoftmaxError, DeviceBatch, DeviceLstm, LsShape,
    attn_softmax_adam_step, lstm_stack_bwd, lstm_stack_fwd, lstm_stack_workspace_bytes,
    attn_softmax_bwd, attn_softmax_fwd_static, attn_softmax_stream_probe,
    attn_softmax_fwd, attn_softmax_last_error, attn_softmax_profile_enable,
    attn_softmax_profile_read, attn_softmax_profile_select, attn_softmax_step_fwd, attn_softmax_step_prepare,
    attn_softmax_step_workspace_bytes, attn_softmax_view, attn_softmax_workspace_bytes, library_path, load_library)
