"""MI355X (gfx950) decoder-layer training step: thin Python binding over the C-ABI library.

Every function here only marshals arguments (device pointers of torch tensors, sizes, the
current stream) into the entry point of the same name declared in include/dlayer.h.  All
arithmetic runs in the HIP kernels of libdlayer.so; there is no CPU or PyTorch fallback: the first
use of any name of the binding without the built library raises.

The binding is loaded on first use, not on import, so that `paper_2602_08387_amd.build` (which
compiles the library) can be imported on a tree that holds no library yet.
"""
import importlib

_BINDING_NAMES = (
    "DLayerError", "LayerCfg", "lib", "lib_path", "DLAYER_ACCUMULATE_WGRADS", "DLAYER_REUSE_TRANSPOSED_WEIGHTS", "DLAYER_RECOMPUTE_NORMS", "DLAYER_RECOMPUTE_SWIGLU",
    "dlayer_version", "dlayer_saved_bytes", "dlayer_workspace_bytes", "dlayer_forward", "dlayer_backward",
    "ce_loss_workspace_bytes", "ce_loss_fwd_bwd", "ce_loss_fwd_bwd_static", "lm_head_ce_workspace_bytes", "lm_head_ce_fwd_bwd",
    "rmsnorm_forward", "rmsnorm_backward", "rmsnorm_backward_workspace_bytes",
    "linear_forward", "qkv_rope_workspace_bytes", "qkv_rope_forward", "linear_swiglu_forward", "linear_swiglu_backward",
    "linear_swiglu_backward_workspace_bytes", "linear_backward", "linear_backward_workspace_bytes", "linear_wgrad_group",
    "rope_apply", "attention_forward", "attention_backward", "attention_backward_workspace_bytes",
    "swiglu_forward", "swiglu_backward", "embed_forward", "embed_backward_workspace_bytes", "embed_backward",
    "grad_sq_norm_workspace_bytes", "grad_sq_norm", "adamw_step", "issue_rate_probe",
    "EXPORTED_SYMBOLS", "WEIGHT_FIELDS",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_BINDING_NAMES))
