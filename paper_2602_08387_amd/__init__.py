"""MI355X (gfx950) decoder-layer training step: thin Python binding over the C-ABI library.

Every function here only marshals arguments (device pointers of torch tensors, sizes, the
current stream) into the entry point of the same name declared in include/dlayer.h.  All
arithmetic runs in the HIP kernels of libdlayer.so; there is no CPU or PyTorch fallback:
importing the binding without the built library raises.
"""
from .binding import (  # noqa: F401
    DLayerError, LayerCfg, lib, lib_path,
    dlayer_version, dlayer_saved_bytes, dlayer_workspace_bytes, dlayer_forward, dlayer_backward,
    ce_loss_workspace_bytes, ce_loss_fwd_bwd,
    rmsnorm_forward, rmsnorm_backward, rmsnorm_backward_workspace_bytes,
    linear_forward, linear_backward, linear_backward_workspace_bytes,
    rope_apply, attention_forward, attention_backward, attention_backward_workspace_bytes,
    swiglu_forward, swiglu_backward, embed_forward, embed_backward,
    EXPORTED_SYMBOLS, WEIGHT_FIELDS,
)
