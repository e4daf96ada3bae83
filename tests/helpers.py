"""Shared helpers of the GPU parity tests (no method arithmetic)."""
import numpy as np

from paper_2507_03117_amd import synth


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


def long_row_case(rng, b, nbi=12, nbc=48):
    """Gate/up masks with block rows that the 16-block chunk plan cuts - in gate only, in up only, in both, barely
    (17 and 20 blocks) - next to empty and ordinary rows; a uniform down mask.  The weights of a block row are
    scaled by its length, so that every row of H is of order one: bf16 rounds H on both sides, and one rounding
    that falls the other way in an entry of 20 among entries of 0.1 would alone exceed the tolerance on Y."""
    E, I = nbc * b, nbi * b
    d = synth.gauss_bf16(rng, (E, I), 0.02)
    mg, mu = (synth.uniform_mask(rng, nbi, nbc, 0.9) for _ in range(2))
    md = synth.uniform_mask(rng, nbc, nbi, 0.6)
    mg[0, :], mu[0, :] = 1, 0
    mu[0, 5:8] = 1
    mg[1, :], mu[1, :] = 0, 1
    mg[1, 40:42] = 1
    mg[2, :], mu[2, :] = 1, 1
    mg[3, :], mu[3, :] = 0, 0
    mg[3, 3:23], mu[3, 30:47] = 1, 1
    mg[4, :], mu[4, :] = 0, 1
    mg[5, :], mu[5, :] = 0, 0
    g, u = (synth.f32_to_bf16_bits((rng.standard_normal((I, E)) *
                                    np.repeat(0.8 / np.sqrt(np.maximum(m.sum(1), 1) * b), b)[:, None]).astype(np.float32))
            for m in (mg, mu))
    return E, I, (g, u, d), (mg, mu, md)


def long_scratch_bytes(packed, b, T, chunk=16):
    """fp32 scratch the MLP workspace carries for the cut rows of gate and up, per matrix T x b values for every
    chunk of a cut row and for every cut row (the whole side of that row in the other matrix), counted by their
    upper bounds: slots = the most rows that can hold more than 16 of the matrix' blocks, chunks <= nnz/16 + slots."""
    total = 0
    for m in packed:
        slots = min(m.rows // b, m.nnz // (chunk + 1)) if m.max_row_blocks > chunk else 0
        chunks = m.nnz // chunk + slots if slots else 0
        total += -(-((chunks + slots) * b * T * 4) // 256) * 256
    return total
