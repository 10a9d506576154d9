"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import torch


def to_device(Gw: np.ndarray) -> torch.Tensor:
    """Worker-major host array (fp32, or uint16 bf16 bits) -> device tensor [p, n]."""
    if Gw.dtype == np.uint16:
        return torch.from_numpy(Gw.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(Gw).cuda()


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    nb = float(np.linalg.norm(b))
    return float(np.linalg.norm(a - b)) / (nb if nb > 0 else 1.0)


def announce(*args) -> None:
    print("[gpu-case]", *args, flush=True)
