"""MI355X-native FF-INT8 layer-local train step: thin ctypes binding over libffint8.so.

Every step of the path runs in the library's HIP kernels; this package only marshals
arguments (torch is used for device memory and streams).  There is no CPU fallback:
importing the binding without a built library raises."""
from .binding import (  # noqa: F401
    FFError, Net, lib, layer_desc, ff_pitch, ff_pitch32, ff_stream_tag, ff_status_string, ff_version,
    ff_goodness_shift, ff_layer_dw_chunks, ff_layer_workspace_bytes, ff_quantize, ff_layer_forward, ff_goodness_loss, ff_layer_handoff, ff_lookahead,
    ff_layer_backward_local, ff_layer_backward_local_noalloc, ff_noalloc_scratch_bytes, ff_chain_gradients, ff_layer_input_grad, ff_layer_update, ff_train_step, ff_train_step_at, ff_workspace_bytes,
    ff_timing_enable, ff_timing_clock_probe, ff_probe_mfma_ceiling, ff_timing_fused_stamps, ff_timing_reset, ff_timing_read, KERNEL_CLASSES,
    ROUND_NEAREST, ROUND_STOCHASTIC, PASS_POS, PASS_NEG, KIND_ACT, KIND_GRAD, KIND_CHAIN, WS_MIN_BYTES,
)
