"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import torch


def to_device(Gw: np.ndarray) -> torch.Tensor:
    """Worker-major host array (fp32, or uint16 bf16 bits) -> device tensor [p, n].

    The library wants every gradient 16-byte aligned, so the rows live in a buffer whose row
    pitch is rounded up to 16 bytes; the returned tensor is the [p, n] view of it."""
    p, n = Gw.shape
    per16 = 8 if Gw.dtype == np.uint16 else 4
    ld = (n + per16 - 1) // per16 * per16
    if Gw.dtype == np.uint16:
        buf = torch.zeros((p, ld), dtype=torch.bfloat16, device="cuda")
        buf[:, :n] = torch.from_numpy(Gw.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        buf = torch.zeros((p, ld), dtype=torch.float32, device="cuda")
        buf[:, :n] = torch.from_numpy(Gw).cuda()
    return buf[:, :n]


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    nb = float(np.linalg.norm(b))
    return float(np.linalg.norm(a - b)) / (nb if nb > 0 else 1.0)


_capture = None


def set_capture_manager(capman) -> None:
    """conftest hands over pytest's capture manager, so that progress lines reach the terminal
    while a long case is still running (captured output only shows up when a case fails)."""
    global _capture
    _capture = capman


def announce(*args) -> None:
    line = "[gpu-case] " + " ".join(str(a) for a in args)
    if _capture is not None:
        with _capture.global_and_fixture_disabled():
            print("\n" + line, flush=True)
    else:
        print(line, flush=True)
