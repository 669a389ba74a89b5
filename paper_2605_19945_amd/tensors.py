"""Moving host buffers to the device and back (argument marshalling, no arithmetic of the layer).

The layer consumes bf16 tensors; on the host they are uint16 bit patterns (numpy has no bf16)."""
import numpy as np


def to_dev_bf16(bits, device="cuda"):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on the device."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def to_dev(a, device="cuda"):
    """numpy array -> device tensor of the same dtype."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def bits_of(t):
    """torch.bfloat16 tensor -> uint16 bit patterns on the host."""
    import torch
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def f64_of_bf16(t):
    """torch.bfloat16 tensor -> float64 numpy array (exact widening)."""
    return (bits_of(t).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
