"""ctypes front-end of the C oracle (oracle/blast_oracle.c).

TEST INFRASTRUCTURE ONLY: used by tests/, the smoke check and the benchmark's
cpu_baseline leg.  The product path never imports this module.

Conventions: weights are `out x in` row-major bf16 bit patterns (uint16);
X is passed as a logical K x T matrix through element strides; results are
fp64 arrays of logical shape [rows, T].
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        i64, i32, dbl, vp = C.c_int64, C.c_int32, C.c_double, C.c_void_p
        L.oracle_num_threads.restype = C.c_int
        L.oracle_n_keep.restype = i64
        L.oracle_n_keep.argtypes = [i64, dbl]
        L.oracle_block_scores.restype = None
        L.oracle_block_scores.argtypes = [vp, i64, i64, i64, i32, vp]
        L.oracle_topk_mask.restype = i64
        L.oracle_topk_mask.argtypes = [vp, i64, dbl, vp, vp]
        L.oracle_pack.restype = i64
        L.oracle_pack.argtypes = [vp, i64, i64, i64, i32, vp, vp, vp, vp, vp]
        L.oracle_unpack.restype = None
        L.oracle_unpack.argtypes = [i64, i64, i32, vp, vp, vp, vp]
        for name in ("oracle_spmm", "oracle_spmm_f32acc"):
            f = getattr(L, name)
            f.restype = None
            f.argtypes = [i64, i64, i32, vp, vp, vp, vp, i64, i64, i64, vp]
        L.oracle_act.restype = dbl
        L.oracle_act.argtypes = [i32, dbl]
        L.oracle_mlp.restype = None
        L.oracle_mlp.argtypes = [i64, i64, i32] + [vp] * 9 + [vp, i64, i64, i64, i32, vp, vp]
        L.oracle_spmm_t.restype = None
        L.oracle_spmm_t.argtypes = [i64, i64, i32, vp, vp, vp, vp, i64, i64, i64, vp]
        L.oracle_sddmm.restype = None
        L.oracle_sddmm.argtypes = [i64, i64, i32, vp, vp, vp, i64, i64, vp, i64, i64, i64, vp]
        L.oracle_generate_masks.restype = None
        L.oracle_generate_masks.argtypes = [vp, i64, vp, i64, i64, i64, i32, dbl, vp]
        L.oracle_sparsity_schedule.restype = dbl
        L.oracle_sparsity_schedule.argtypes = [i64, i64, i64, dbl, dbl]
        L.oracle_pooled_scores.restype = None
        L.oracle_pooled_scores.argtypes = [vp, i64, i64, i64, i32, vp]
        L.oracle_spmm_e5m2w.restype = None
        L.oracle_spmm_e5m2w.argtypes = [i64, i64, i32, vp, vp, vp, vp, i64, i64, i64, vp]
        L.oracle_mlp_e5m2w.restype = None
        L.oracle_mlp_e5m2w.argtypes = [i64, i64, i32] + [vp] * 9 + [vp, i64, i64, i64, i32, vp, vp]
        L.oracle_e5m2_to_f64.restype = dbl
        L.oracle_e5m2_to_f64.argtypes = [C.c_uint8]
        L.oracle_f64_to_e5m2.restype = C.c_uint8
        L.oracle_f64_to_e5m2.argtypes = [dbl]
        L.oracle_quantize_e5m2.restype = None
        L.oracle_quantize_e5m2.argtypes = [vp, i64, vp]
        L.oracle_spmm_e5m2.restype = None
        L.oracle_spmm_e5m2.argtypes = [i64, i64, i32, vp, vp, vp, vp, i64, i64, i64, vp]
        L.oracle_mlp2.restype = None
        L.oracle_mlp2.argtypes = [i64, i64, i32] + [vp] * 6 + [vp, i64, i64, i64, i32, vp, vp]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def n_keep(n_blocks: int, sparsity: float) -> int:
    return int(lib().oracle_n_keep(n_blocks, float(sparsity)))


def block_scores(W: np.ndarray, b: int) -> np.ndarray:
    W = np.ascontiguousarray(W, dtype=np.uint16)
    rows, cols = W.shape
    assert rows % b == 0 and cols % b == 0
    score = np.empty((rows // b, cols // b), dtype=np.float64)
    lib().oracle_block_scores(_p(W), cols, rows, cols, b, _p(score))
    return score


def topk_mask(score: np.ndarray, sparsity: float) -> Tuple[np.ndarray, float]:
    score = np.ascontiguousarray(score, dtype=np.float64)
    mask = np.empty(score.shape, dtype=np.uint8)
    gap = C.c_double(0.0)
    lib().oracle_topk_mask(_p(score), score.size, float(sparsity), _p(mask), C.byref(gap))
    return mask, float(gap.value)


@dataclass
class Bsr:
    rows: int
    cols: int
    b: int
    row_ptr: np.ndarray  # int32 [rows/b + 1]
    col_idx: np.ndarray  # int32 [nnz]
    vals: np.ndarray  # uint16 [nnz, b, b]
    row_order: np.ndarray  # int32 [rows/b]

    @property
    def nnz(self) -> int:
        return int(self.col_idx.size)


def pack(W: np.ndarray, b: int, mask: np.ndarray) -> Bsr:
    W = np.ascontiguousarray(W, dtype=np.uint16)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    rows, cols = W.shape
    nbr, nbc = rows // b, cols // b
    assert mask.shape == (nbr, nbc)
    nnz = int(np.count_nonzero(mask))
    row_ptr = np.empty(nbr + 1, dtype=np.int32)
    col_idx = np.empty(nnz, dtype=np.int32)
    vals = np.empty((nnz, b, b), dtype=np.uint16)
    row_order = np.empty(nbr, dtype=np.int32)
    got = lib().oracle_pack(_p(W), cols, rows, cols, b, _p(mask), _p(row_ptr), _p(col_idx), _p(vals), _p(row_order))
    assert got == nnz
    return Bsr(rows, cols, b, row_ptr, col_idx, vals, row_order)


def pack_topk(W: np.ndarray, b: int, sparsity: float) -> Tuple[Bsr, np.ndarray, float]:
    mask, gap = topk_mask(block_scores(W, b), sparsity)
    return pack(W, b, mask), mask, gap


def unpack(m: Bsr) -> np.ndarray:
    Wd = np.empty((m.rows, m.cols), dtype=np.uint16)
    lib().oracle_unpack(m.rows, m.cols, m.b, _p(m.row_ptr), _p(m.col_idx), _p(m.vals), _p(Wd))
    return Wd


def _x_strides(X: np.ndarray, layout: str) -> Tuple[int, int, int, int]:
    """X as logical K x T.  layout 'token_major': X is [T, K]; 'feature_major': X is [K, T]."""
    assert X.dtype == np.uint16 and X.ndim == 2 and X.flags.c_contiguous
    if layout == "token_major":
        T, K = X.shape
        return K, T, 1, K
    if layout == "feature_major":
        K, T = X.shape
        return K, T, T, 1
    raise ValueError(layout)


def spmm(m: Bsr, X: np.ndarray, layout: str = "token_major", f32acc: bool = False) -> np.ndarray:
    """Returns Y as fp64 [rows, T]."""
    K, T, sxk, sxt = _x_strides(X, layout)
    assert K == m.cols
    Y = np.zeros((m.rows, T), dtype=np.float64)
    fn = lib().oracle_spmm_f32acc if f32acc else lib().oracle_spmm
    fn(m.rows, m.cols, m.b, _p(m.row_ptr), _p(m.col_idx), _p(m.vals), _p(X), sxk, sxt, T, _p(Y))
    return Y


ACT = {"silu": 0, "gelu": 1, "relu": 2}


def act(name: str, g: float) -> float:
    return float(lib().oracle_act(ACT[name], float(g)))


def mlp(gate: Bsr, up: Bsr, down: Bsr, X: np.ndarray, layout: str = "token_major", activation: str = "silu",
        return_h: bool = False):
    """Returns Y as fp64 [E, T] (and H bf16 bits [I, T] if asked)."""
    K, T, sxk, sxt = _x_strides(X, layout)
    E, I, b = gate.cols, gate.rows, gate.b
    assert K == E and up.rows == I and up.cols == E and down.rows == E and down.cols == I
    assert up.b == b and down.b == b
    Y = np.zeros((E, T), dtype=np.float64)
    H = np.zeros((I, T), dtype=np.uint16) if return_h else None
    lib().oracle_mlp(E, I, b, _p(gate.row_ptr), _p(gate.col_idx), _p(gate.vals), _p(up.row_ptr), _p(up.col_idx),
                     _p(up.vals), _p(down.row_ptr), _p(down.col_idx), _p(down.vals), _p(X), sxk, sxt, T,
                     ACT[activation], _p(Y), _p(H))
    return (Y, H) if return_h else Y


def mlp2(w1: Bsr, w2: Bsr, X: np.ndarray, layout: str = "token_major", activation: str = "gelu",
         return_h: bool = False):
    """Two-matrix MLP Y = W2 * act(W1 * X) (Sec. 2.1 / Sec. 3.4.3): fp64 [E, T] (and H bf16 bits [I, T] if asked)."""
    K, T, sxk, sxt = _x_strides(X, layout)
    E, I, b = w1.cols, w1.rows, w1.b
    assert K == E and w2.rows == E and w2.cols == I and w2.b == b
    Y = np.zeros((E, T), dtype=np.float64)
    H = np.zeros((I, T), dtype=np.uint16) if return_h else None
    lib().oracle_mlp2(E, I, b, _p(w1.row_ptr), _p(w1.col_idx), _p(w1.vals), _p(w2.row_ptr), _p(w2.col_idx),
                      _p(w2.vals), _p(X), sxk, sxt, T, ACT[activation], _p(Y), _p(H))
    return (Y, H) if return_h else Y


def spmm_t(w: Bsr, dY: np.ndarray, layout: str = "token_major") -> np.ndarray:
    """Backward of Y = W~ X with respect to X: dX = W~^T dY (Sec. 3.2, Sec. 3.4), fp64 [cols, T].
    dY is [T, rows] (token_major) or [rows, T] (feature_major), bf16 bits."""
    M, T, syi, syt = _x_strides(dY, layout)
    assert M == w.rows
    dX = np.zeros((w.cols, T), dtype=np.float64)
    lib().oracle_spmm_t(w.rows, w.cols, w.b, _p(w.row_ptr), _p(w.col_idx), _p(w.vals), _p(dY), syi, syt, T, _p(dX))
    return dX


def sddmm(w: Bsr, dY: np.ndarray, X: np.ndarray, layout: str = "token_major") -> np.ndarray:
    """Backward with respect to the stored blocks: the entries of dY X^T on the kept blocks (Sec. 3.2),
    fp64 [nnz, b, b] in storage order.  Only the structure of `w` is used."""
    M, T, syi, syt = _x_strides(dY, layout)
    K, T2, sxk, sxt = _x_strides(X, layout)
    assert M == w.rows and K == w.cols and T == T2
    dv = np.zeros((w.nnz, w.b, w.b), dtype=np.float64)
    lib().oracle_sddmm(w.rows, w.cols, w.b, _p(w.row_ptr), _p(w.col_idx), _p(dY), syi, syt, _p(X), sxk, sxt, T, _p(dv))
    return dv


def generate_masks(W: np.ndarray, G: np.ndarray, b: int, sparsity: float) -> np.ndarray:
    """One mask update of blocked prune-and-grow (Sec. 3.2): uint8 [rows/b, cols/b], 1 = kept by the weight's
    own ranking, 2 = regrown (ranked high by the gradient only; stored as zeros), 0 = dropped."""
    W = np.ascontiguousarray(W, dtype=np.uint16)
    G = np.ascontiguousarray(G, dtype=np.uint16)
    assert W.shape == G.shape
    rows, cols = W.shape
    mask = np.empty((rows // b, cols // b), dtype=np.uint8)
    lib().oracle_generate_masks(_p(W), cols, _p(G), cols, rows, cols, b, float(sparsity), _p(mask))
    return mask


def sparsity_schedule(i: int, m: int, d: int, s_init: float, s_max: float) -> float:
    """Eq. (2), with the iteration held inside [0, m - d]."""
    return float(lib().oracle_sparsity_schedule(int(i), int(m), int(d), float(s_init), float(s_max)))


def pooled_scores(S: np.ndarray, b: int) -> np.ndarray:
    """2D average pooling of a sensitivity matrix over b x b blocks (Sec. 3.3): fp64 [rows/b, cols/b]."""
    S = np.ascontiguousarray(S, dtype=np.float32)
    rows, cols = S.shape
    sc = np.empty((rows // b, cols // b), dtype=np.float64)
    lib().oracle_pooled_scores(_p(S), cols, rows, cols, b, _p(sc))
    return sc


def pooled_topk_mask(S: np.ndarray, b: int, sparsity: float) -> Tuple[np.ndarray, float]:
    """Keep the blocks with the highest pooled sensitivity (same count and tie rule as the Frobenius ranking).
    Returns (uint8 mask [rows/b, cols/b], relative score gap at the keep/drop boundary)."""
    sc = pooled_scores(S, b)
    mask, gap = topk_mask(sc, sparsity)
    return mask.reshape(sc.shape), gap


def e5m2_decode(codes: np.ndarray) -> np.ndarray:
    """Exact fp64 values of E5M2 codes (any shape)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    f = lib().oracle_e5m2_to_f64
    return np.array([f(int(c)) for c in range(256)], dtype=np.float64)[codes]


def e5m2_quantize(x: np.ndarray) -> np.ndarray:
    """fp32 values -> E5M2 codes, round to nearest even, overflow to infinity (Sec. 5.2 dtype)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    lib().oracle_quantize_e5m2(_p(x), x.size, _p(out))
    return out


def spmm_e5m2(w: Bsr, vals8: np.ndarray, X8: np.ndarray, layout: str = "token_major") -> np.ndarray:
    """Y = W~ X with E5M2 block values `vals8` [nnz, b, b] on the structure of `w` and E5M2 activations: fp64 [rows, T]."""
    vals8 = np.ascontiguousarray(vals8, dtype=np.uint8)
    X8 = np.ascontiguousarray(X8, dtype=np.uint8)
    assert vals8.shape == (w.nnz, w.b, w.b) and X8.ndim == 2
    if layout == "token_major":
        T, K = X8.shape
        sxk, sxt = 1, K
    else:
        K, T = X8.shape
        sxk, sxt = T, 1
    assert K == w.cols
    Y = np.zeros((w.rows, T), dtype=np.float64)
    lib().oracle_spmm_e5m2(w.rows, w.cols, w.b, _p(w.row_ptr), _p(w.col_idx), _p(vals8), _p(X8), sxk, sxt, T, _p(Y))
    return Y


def spmm_e5m2w(w: Bsr, vals8: np.ndarray, X: np.ndarray, layout: str = "token_major") -> np.ndarray:
    """Y = W~ X with E5M2 block values `vals8` [nnz, b, b] on the structure of `w` and bf16 activations: fp64 [rows, T]."""
    vals8 = np.ascontiguousarray(vals8, dtype=np.uint8)
    assert vals8.shape == (w.nnz, w.b, w.b)
    K, T, sxk, sxt = _x_strides(X, layout)
    assert K == w.cols
    Y = np.zeros((w.rows, T), dtype=np.float64)
    lib().oracle_spmm_e5m2w(w.rows, w.cols, w.b, _p(w.row_ptr), _p(w.col_idx), _p(vals8), _p(X), sxk, sxt, T, _p(Y))
    return Y


def mlp_e5m2w(gate: Bsr, g8: np.ndarray, up: Bsr, u8: np.ndarray, down: Bsr, d8: np.ndarray, X: np.ndarray,
              layout: str = "token_major", activation: str = "silu", return_h: bool = False):
    """Eq. (1) with the three weights given as E5M2 codes on the structures of gate / up / down, bf16 activations
    and bf16 intermediate: Y fp64 [E, T] (and H bf16 bits [I, T] if asked)."""
    K, T, sxk, sxt = _x_strides(X, layout)
    E, I, b = gate.cols, gate.rows, gate.b
    assert K == E and up.rows == I and up.cols == E and down.rows == E and down.cols == I
    g8, u8, d8 = (np.ascontiguousarray(v, dtype=np.uint8) for v in (g8, u8, d8))
    assert g8.shape == (gate.nnz, b, b) and u8.shape == (up.nnz, b, b) and d8.shape == (down.nnz, b, b)
    Y = np.zeros((E, T), dtype=np.float64)
    H = np.zeros((I, T), dtype=np.uint16) if return_h else None
    lib().oracle_mlp_e5m2w(E, I, b, _p(gate.row_ptr), _p(gate.col_idx), _p(g8), _p(up.row_ptr), _p(up.col_idx), _p(u8),
                           _p(down.row_ptr), _p(down.col_idx), _p(d8), _p(X), sxk, sxt, T, ACT[activation], _p(Y), _p(H))
    return (Y, H) if return_h else Y
