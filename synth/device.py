"""Host <-> device marshalling of bf16 bit patterns for the tests, the benchmark and the smoke run.
Storage plumbing only: no arithmetic of the layer lives here."""
import numpy as np
import torch

from . import inputs as si


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the GPU (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_f64(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float64 NumPy array (bf16 through its bit pattern: exact)."""
    if t.dtype == torch.bfloat16:
        return si.bf16_bits_to_f64(t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16))
    return t.detach().cpu().numpy().astype(np.float64)
