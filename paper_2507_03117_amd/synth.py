"""Seeded synthetic inputs: Llama-shaped block-sparse MLP workloads.

This module only *draws inputs*: Gaussian bf16 tensors and boolean block masks.
It holds none of the method's arithmetic (no scoring, packing, multiplication),
imports neither the HIP binding nor the CPU oracle, and is consumed unchanged by
both sides of every parity test.

The paper evaluates the MLP blocks of the Llama family (Sec. 5.2) with weights
pruned from trained checkpoints; those checkpoints are not available, so
Gaussian weights of the same shapes with uniform / top-k / Zipf block masks
stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 20250703

# --------------------------------------------------------------------------
# bf16 <-> fp32 on raw bit patterns (numpy has no bf16 dtype)
# --------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (round-to-nearest-even), return uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def gauss_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    """N(0, std^2) samples rounded once to bf16; returned as uint16 bit patterns."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return f32_to_bf16_bits(x)


# --------------------------------------------------------------------------
# block masks
# --------------------------------------------------------------------------


def n_zero_blocks(n_blocks: int, sparsity: float) -> int:
    """Blocks to zero so that the zero fraction first reaches `sparsity`
    (ceiling, evaluated in integers on basis points)."""
    s_bp = int(round(sparsity * 10000))
    return (s_bp * n_blocks + 9999) // 10000


def uniform_mask(rng: np.random.Generator, nbr: int, nbc: int, sparsity: float) -> np.ndarray:
    """Exactly n_zero_blocks() blocks zeroed, chosen by a seeded permutation."""
    n = nbr * nbc
    mask = np.ones(n, dtype=np.uint8)
    perm = rng.permutation(n)
    mask[perm[: n_zero_blocks(n, sparsity)]] = 0
    return mask.reshape(nbr, nbc)


def zipf_row_counts(rng: np.random.Generator, nbr: int, nbc: int, nnz: int, alpha: float) -> np.ndarray:
    """Per-block-row nonzero counts with weight ~ rank^-alpha, capped at nbc.

    Capped largest-remainder apportionment: rows whose share exceeds the cap are
    pinned at the cap and their surplus is re-apportioned over the others until
    stable; leftover units go to the largest fractional parts (ties: lower rank).
    Ranks are assigned to rows by a seeded permutation.
    """
    if nnz > nbr * nbc:
        raise ValueError("nnz exceeds the matrix")
    w = np.arange(1, nbr + 1, dtype=np.float64) ** (-alpha)
    capped = np.zeros(nbr, dtype=bool)
    share = np.zeros(nbr, dtype=np.float64)
    while True:
        free = ~capped
        remaining = nnz - int(capped.sum()) * nbc
        share[:] = 0.0
        share[capped] = nbc
        if free.any():
            share[free] = remaining * w[free] / w[free].sum()
        over = free & (share > nbc)
        if not over.any():
            break
        capped |= over
    counts = np.floor(share).astype(np.int64)
    counts[capped] = nbc
    left = nnz - int(counts.sum())
    if left > 0:
        frac = share - counts
        frac[counts >= nbc] = -1.0
        order = np.lexsort((np.arange(nbr), -frac))  # fractional part desc, rank asc
        k = 0
        while left > 0:
            r = order[k % nbr]
            if counts[r] < nbc:
                counts[r] += 1
                left -= 1
            k += 1
    row_of_rank = rng.permutation(nbr)
    out = np.zeros(nbr, dtype=np.int64)
    out[row_of_rank] = counts
    return out


def zipf_mask(rng: np.random.Generator, nbr: int, nbc: int, sparsity: float, alpha: float = 1.2) -> np.ndarray:
    """Block mask whose per-row counts follow zipf_row_counts(); columns inside a
    row are a seeded uniform sample without replacement."""
    nnz = nbr * nbc - n_zero_blocks(nbr * nbc, sparsity)
    counts = zipf_row_counts(rng, nbr, nbc, nnz, alpha)
    mask = np.zeros((nbr, nbc), dtype=np.uint8)
    for r in range(nbr):
        c = int(counts[r])
        if c:
            mask[r, rng.choice(nbc, size=c, replace=False)] = 1
    return mask


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------


@dataclass
class Workload:
    """One configuration of the benchmark spec `configs`, parameterised."""

    name: str
    config_id: int
    kind: str  # "linear" | "mlp" (gate/up/down) | "mlp2" (two matrices)
    hidden: int  # E (for "linear": cols K)
    inter: int  # I (for "linear": rows M)
    b: int
    sparsity: float
    mask_kind: str  # "uniform" | "topk" | "zipf"
    tokens: Tuple[int, ...]
    w_std: float = 0.02
    x_std: float = 1.0


WORKLOADS: Dict[str, Workload] = {
    "linear_1024x4096_b32_s90": Workload("linear_1024x4096_b32_s90", 0, "linear", 4096, 1024, 32, 0.90, "uniform", (64,)),
    "llama1b_b64_s90": Workload("llama1b_b64_s90", 1, "mlp", 2048, 8192, 64, 0.90, "uniform", (1, 16, 128, 2048)),
    # the same layer with the smallest block size of the paper's block-size sweeps (same seed: same dense weights)
    "llama1b_b16_s90": Workload("llama1b_b16_s90", 1, "mlp", 2048, 8192, 16, 0.90, "uniform", (1, 16, 128, 2048)),
    "llama3b_b64_s70": Workload("llama3b_b64_s70", 2, "mlp", 3072, 8192, 64, 0.70, "topk", (4096,)),
    "llama3b_b64_s80": Workload("llama3b_b64_s80", 2, "mlp", 3072, 8192, 64, 0.80, "topk", (4096,)),
    "llama3b_b64_s90": Workload("llama3b_b64_s90", 2, "mlp", 3072, 8192, 64, 0.90, "topk", (4096,)),
    "llama3b_b64_s95": Workload("llama3b_b64_s95", 2, "mlp", 3072, 8192, 64, 0.95, "topk", (4096,)),
    "llama8b_b128_s95": Workload("llama8b_b128_s95", 3, "mlp", 4096, 14336, 128, 0.95, "uniform", (1, 2, 4, 8, 16, 32)),
    # two-matrix MLP of a GPT2-XL block (E = 1600, I = 4E), 80 % sparsity as in the paper's pretraining run;
    # b = 64 because 1600 is not a multiple of 128
    "gpt2xl_b64_s80": Workload("gpt2xl_b64_s80", 5, "mlp2", 1600, 6400, 64, 0.80, "uniform", (1, 16, 2048)),
    "llama405b_b128_s95_zipf": Workload("llama405b_b128_s95_zipf", 4, "mlp", 16384, 53248, 128, 0.95, "zipf", (2048,)),
}


def _streams(wl: Workload, seed: Optional[int]) -> List[np.random.Generator]:
    s = BASE_SEED * 10 + wl.config_id if seed is None else seed
    return [np.random.Generator(np.random.PCG64(c)) for c in np.random.SeedSequence(s).spawn(8)]


def _dense_or_sparse_weight(rng, rows, cols, b, std, mask, fill_all: bool) -> np.ndarray:
    """Dense bf16 weight (bit patterns).  When `fill_all` is False only the kept
    blocks get Gaussian values and the rest stay zero: mask-mode packing never
    reads a dropped block, and this keeps the 405B-class layer cheap to draw."""
    if fill_all or mask is None:
        return gauss_bf16(rng, (rows, cols), std)
    w = np.zeros((rows, cols), dtype=np.uint16)
    nbr, nbc = mask.shape
    wv = w.reshape(nbr, b, nbc, b)
    rr, cc = np.nonzero(mask)
    vals = gauss_bf16(rng, (rr.size, b, b), std)
    wv[rr, :, cc, :] = vals
    return w


def make_mask(rng, wl: Workload, nbr: int, nbc: int) -> Optional[np.ndarray]:
    if wl.mask_kind == "uniform":
        return uniform_mask(rng, nbr, nbc, wl.sparsity)
    if wl.mask_kind == "zipf":
        return zipf_mask(rng, nbr, nbc, wl.sparsity, 1.2)
    return None  # "topk": the mask is computed by the packer under test


@dataclass
class LinearInputs:
    W: np.ndarray  # [M, K] uint16 bf16 bits
    mask: Optional[np.ndarray]  # [M/b, K/b] uint8, None for top-k workloads
    b: int
    sparsity: float


@dataclass
class MlpInputs:
    gate: LinearInputs  # I x E
    up: LinearInputs  # I x E
    down: LinearInputs  # E x I
    extras: dict = field(default_factory=dict)


def make_linear(wl: Workload, seed: Optional[int] = None) -> LinearInputs:
    st = _streams(wl, seed)
    m, k, b = wl.inter, wl.hidden, wl.b
    mask = make_mask(st[4], wl, m // b, k // b)
    w = _dense_or_sparse_weight(st[0], m, k, b, wl.w_std, mask, fill_all=True)
    return LinearInputs(w, mask, b, wl.sparsity)


def make_mlp(wl: Workload, seed: Optional[int] = None, fill_all: Optional[bool] = None) -> MlpInputs:
    st = _streams(wl, seed)
    e, i, b = wl.hidden, wl.inter, wl.b
    if fill_all is None:
        fill_all = wl.mask_kind == "topk" or e * i <= (1 << 26)
    mg = make_mask(st[4], wl, i // b, e // b)
    mu = make_mask(st[5], wl, i // b, e // b)
    md = make_mask(st[6], wl, e // b, i // b)
    g = _dense_or_sparse_weight(st[0], i, e, b, wl.w_std, mg, fill_all)
    u = _dense_or_sparse_weight(st[1], i, e, b, wl.w_std, mu, fill_all)
    d = _dense_or_sparse_weight(st[2], e, i, b, wl.w_std, md, fill_all)
    return MlpInputs(LinearInputs(g, mg, b, wl.sparsity), LinearInputs(u, mu, b, wl.sparsity),
                     LinearInputs(d, md, b, wl.sparsity))


def make_mlp2(wl: Workload, seed: Optional[int] = None) -> Tuple[LinearInputs, LinearInputs]:
    """(W1: I x E, W2: E x I) of a two-matrix MLP."""
    st = _streams(wl, seed)
    e, i, b = wl.hidden, wl.inter, wl.b
    m1 = make_mask(st[4], wl, i // b, e // b)
    m2 = make_mask(st[6], wl, e // b, i // b)
    w1 = _dense_or_sparse_weight(st[0], i, e, b, wl.w_std, m1, True)
    w2 = _dense_or_sparse_weight(st[2], e, i, b, wl.w_std, m2, True)
    return LinearInputs(w1, m1, b, wl.sparsity), LinearInputs(w2, m2, b, wl.sparsity)


def make_x(wl: Workload, tokens: int, seed: Optional[int] = None) -> np.ndarray:
    """Activations, token-major [tokens, hidden] bf16 bits (element (k, t) at X[t, k])."""
    st = _streams(wl, seed)
    return gauss_bf16(st[3], (tokens, wl.hidden), wl.x_std)


def small_case(seed: int, rows: int, cols: int, b: int, sparsity: float, tokens: int,
               w_std: float = 0.02, x_std: float = 1.0, empty_rows=(), full_rows=()):
    """Small ad-hoc single-matrix case for property tests: (W bits, mask, X bits token-major)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    nbr, nbc = rows // b, cols // b
    mask = uniform_mask(rng, nbr, nbc, sparsity)
    for r in empty_rows:
        mask[r % nbr, :] = 0
    for r in full_rows:
        mask[r % nbr, :] = 1
    w = gauss_bf16(rng, (rows, cols), w_std)
    x = gauss_bf16(rng, (tokens, cols), x_std)
    return w, mask, x
