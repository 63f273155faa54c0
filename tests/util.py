"""Helpers shared by the tests: bf16-bit <-> torch conversions and error metrics."""
import numpy as np
import torch


def bits_to_torch(bits_u16, device="cuda"):
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 tensor on `device`."""
    t = torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).view(torch.bfloat16)
    return t.to(device)


def torch_to_bits(t):
    """torch.bfloat16 tensor -> numpy uint16 bit patterns (host)."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def rel_errors(got, ref):
    """Per-row norm-wise relative error and the global max-wise relative error."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    normwise = np.linalg.norm(got - ref, axis=-1) / np.linalg.norm(ref, axis=-1)
    maxwise = np.abs(got - ref).max() / np.abs(ref).max()
    return normwise, maxwise
