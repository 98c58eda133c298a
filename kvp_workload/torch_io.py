"""bf16 bit patterns <-> torch tensors.  Plumbing only: no arithmetic of the method.

The generator hands out uint16 bit patterns; the GPU path wants torch.bfloat16
tensors on the device.  These two views never change a bit."""
import numpy as np


def bits_to_torch(bits, device="cuda:0"):
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on `device`."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def torch_to_bits(t):
    """torch.bfloat16 tensor -> uint16 bit patterns on the host."""
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
