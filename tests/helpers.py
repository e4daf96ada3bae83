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


def stratified_tokens(T, n_sample, tile=128, boundary=256):
    """Token sample for the oracle: the first and the last token, one seeded draw from every `tile` tokens (every
    token tile of every kernel holds a checked token), both sides of every multiple of `boundary` (the seams between
    token tiles), topped up with uniform draws to n_sample."""
    rng = np.random.default_rng(T)
    sel = {0, T - 1}
    for t0 in range(0, T, tile):
        sel.add(int(rng.integers(t0, min(t0 + tile, T))))
    for e in range(boundary, T, boundary):
        sel.update((e - 1, e))
    if len(sel) < n_sample:
        sel.update(int(t) for t in rng.choice(T, size=n_sample - len(sel), replace=False))
    return np.array(sorted(sel))


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
