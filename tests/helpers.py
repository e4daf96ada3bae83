"""Shared helpers of the GPU parity tests (no method arithmetic)."""
import numpy as np


def to_dev(bits: np.ndarray):
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on cuda:0 (bit-preserving)."""
    import torch

    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to("cuda:0").view(torch.bfloat16)


def mask_dev(mask: np.ndarray):
    import torch

    return torch.from_numpy(np.ascontiguousarray(mask, dtype=np.uint8)).to("cuda:0")


def bits_of(t) -> np.ndarray:
    """torch bf16/int16 tensor -> uint16 bit patterns on the host."""
    import torch

    if t.dtype == torch.bfloat16:
        t = t.view(torch.int16)
    return t.cpu().numpy().view(np.uint16)


# the benchmark spec tolerances: relative Frobenius error <= 1e-3, max elementwise error <= 1e-2 * RMS(oracle)
REL_FRO = 1e-3
MAX_ABS_RMS = 1e-2


def check_close(y_gpu: np.ndarray, y_or: np.ndarray, what: str = ""):
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    assert y_gpu.shape == y_or.shape, (what, y_gpu.shape, y_or.shape)
    assert np.isfinite(y_gpu).all(), what
    if not y_or.any():
        assert not y_gpu.any(), f"{what}: oracle is exactly zero, device is not"
        return 0.0, 0.0
    fro = float(np.linalg.norm(y_gpu - y_or) / np.linalg.norm(y_or))
    rms = float(np.sqrt((y_or ** 2).mean()))
    mx = float(np.abs(y_gpu - y_or).max() / rms)
    assert fro <= REL_FRO, f"{what}: rel Frobenius {fro:.3e} > {REL_FRO}"
    assert mx <= MAX_ABS_RMS, f"{what}: max abs / rms {mx:.3e} > {MAX_ABS_RMS}"
    return fro, mx
