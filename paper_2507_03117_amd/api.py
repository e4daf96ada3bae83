"""Thin Python binding of the C ABI declared in include/blast.h.

Argument marshalling only: torch supplies device memory and the current stream;
every step of the path runs inside libblast_hip.so.  There is no CPU fallback:
if the library is missing or fails to load, every entry point raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libblast_hip.so")

PACK_MASK, PACK_TOPK_FROBENIUS = 0, 1
TOKEN_MAJOR, FEATURE_MAJOR, COLUMN_GROUPS_64 = 0, 1, 2
F32, BF16 = 0, 1
ACT = {"silu": 0, "gelu": 1, "relu": 2}

EXPORTS = (
    "blast_strerror", "blast_n_keep", "blast_bsr_aux_bytes", "blast_bsr_pack_bound", "blast_bsr_pack", "blast_bsr_pack_enqueue",
    "blast_bsr_spmm", "blast_bsr_spmm_workspace", "blast_sparse_mlp", "blast_sparse_mlp_workspace",
    "blast_sparse_mlp_events", "blast_sparse_mlp2", "blast_sparse_mlp2_workspace", "blast_bsr_transpose", "blast_bsr_sddmm",
    "blast_generate_masks", "blast_generate_masks_workspace", "blast_sparsity_schedule",
    "blast_pooled_topk_mask", "blast_pooled_topk_mask_workspace", "blast_quantize_e5m2", "blast_quantize_e5m2_groups",
    "blast_bsr_spmm_e5m2",
    "blast_bsr_unpack", "blast_bsr_gated_spmm", "blast_bsr_joint_row_order",
    "blast_sparse_mlp_static", "blast_sparse_mlp_static_limit", "blast_sparse_mlp_status",
    "blast_sparse_mlp_handover_test", "blast_sparse_mlp_e5m2w", "blast_sparse_mlp_e5m2w_workspace",
)


class BlastError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().blast_strerror(code).decode()} (code {code})")


class BsrView(C.Structure):
    _fields_ = [
        ("rows", C.c_int64), ("cols", C.c_int64), ("b", C.c_int32), ("max_row_blocks", C.c_int32), ("nnz", C.c_int64),
        ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("vals", C.c_void_p), ("row_order", C.c_void_p),
        ("aux", C.c_void_p),
    ]


_lib = None


def lib():
    """Load libblast_hip.so (built by paper_2507_03117_amd/build.py); raise loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2507_03117_amd.build` "
                "(hipcc, gfx950).  There is no CPU fallback.")
        L = C.CDLL(LIB_PATH)
        i64, i32, dbl, vp, sz = C.c_int64, C.c_int32, C.c_double, C.c_void_p, C.c_size_t
        pv = C.POINTER(BsrView)
        L.blast_strerror.restype = C.c_char_p
        L.blast_strerror.argtypes = [C.c_int]
        L.blast_n_keep.restype = i64
        L.blast_n_keep.argtypes = [i64, dbl]
        L.blast_bsr_aux_bytes.restype = sz
        L.blast_bsr_aux_bytes.argtypes = [i64, i64, i32, i64]
        L.blast_bsr_pack_bound.restype = C.c_int
        L.blast_bsr_pack_bound.argtypes = [i64, i64, i32, i32, dbl, C.POINTER(i64), C.POINTER(sz), C.POINTER(sz)]
        L.blast_bsr_pack.restype = C.c_int
        L.blast_bsr_pack.argtypes = [vp, i64, i64, i64, i32, i32, vp, dbl, vp, vp, vp, vp, vp, sz, i64,
                                     C.POINTER(i64), C.POINTER(i32), vp, sz, vp]
        L.blast_bsr_pack_enqueue.restype = C.c_int
        L.blast_bsr_pack_enqueue.argtypes = [vp, i64, i64, i64, i32, i32, vp, dbl, vp, vp, vp, vp, vp, sz, i64,
                                             vp, vp, sz, vp]
        L.blast_bsr_spmm.restype = C.c_int
        L.blast_bsr_spmm.argtypes = [pv, vp, i64, i32, i64, vp, i64, i32, vp, sz, vp]
        L.blast_bsr_spmm_workspace.restype = C.c_int
        L.blast_bsr_spmm_workspace.argtypes = [pv, i64, C.POINTER(sz)]
        L.blast_sparse_mlp.restype = C.c_int
        L.blast_sparse_mlp.argtypes = [pv, pv, pv, vp, i64, i32, i64, i32, vp, i64, i32, vp, sz, vp]
        L.blast_sparse_mlp_status.restype = C.c_int
        L.blast_sparse_mlp_status.argtypes = [pv, i64, vp, sz, C.POINTER(i32), vp]
        L.blast_sparse_mlp_handover_test.restype = C.c_int
        L.blast_sparse_mlp_handover_test.argtypes = L.blast_sparse_mlp.argtypes + [i32, i32]
        L.blast_sparse_mlp_e5m2w.restype = C.c_int
        L.blast_sparse_mlp_e5m2w.argtypes = [pv, vp, pv, vp, pv, vp, vp, i64, i64, i32, vp, i64, i32, vp, sz, vp]
        L.blast_sparse_mlp_e5m2w_workspace.restype = C.c_int
        L.blast_sparse_mlp_e5m2w_workspace.argtypes = [pv, i64, C.POINTER(sz)]
        L.blast_sparse_mlp_static.restype = C.c_int
        L.blast_sparse_mlp_static.argtypes = [pv, pv, pv, vp, i64, i32, i64, i32, vp, i64, i32, vp]
        L.blast_sparse_mlp_static_limit.restype = sz
        L.blast_sparse_mlp_static_limit.argtypes = []
        L.blast_sparse_mlp_workspace.restype = C.c_int
        L.blast_sparse_mlp_workspace.argtypes = [pv, pv, pv, i64, C.POINTER(sz)]
        L.blast_sparse_mlp2.restype = C.c_int
        L.blast_sparse_mlp2.argtypes = [pv, pv, vp, i64, i32, i64, i32, vp, i64, i32, vp, sz, vp]
        L.blast_sparse_mlp2_workspace.restype = C.c_int
        L.blast_sparse_mlp2_workspace.argtypes = [pv, pv, i64, C.POINTER(sz)]
        L.blast_generate_masks.restype = C.c_int
        L.blast_generate_masks.argtypes = [vp, i64, vp, i64, i64, i64, i32, C.c_double, vp, vp, sz, vp]
        L.blast_generate_masks_workspace.restype = sz
        L.blast_generate_masks_workspace.argtypes = [i64, i64, i32]
        L.blast_sparsity_schedule.restype = C.c_double
        L.blast_sparsity_schedule.argtypes = [i64, i64, i64, C.c_double, C.c_double]
        L.blast_pooled_topk_mask.restype = C.c_int
        L.blast_pooled_topk_mask.argtypes = [vp, i64, i64, i64, i32, C.c_double, vp, vp, sz, vp]
        L.blast_pooled_topk_mask_workspace.restype = sz
        L.blast_pooled_topk_mask_workspace.argtypes = [i64, i64, i32]
        L.blast_quantize_e5m2.restype = C.c_int
        L.blast_quantize_e5m2.argtypes = [vp, i64, vp, vp]
        L.blast_quantize_e5m2_groups.restype = C.c_int
        L.blast_quantize_e5m2_groups.argtypes = [vp, i64, i64, i64, vp, vp]
        L.blast_bsr_spmm_e5m2.restype = C.c_int
        L.blast_bsr_spmm_e5m2.argtypes = [pv, vp, vp, i64, i32, i64, vp, i64, i32, vp]
        L.blast_bsr_unpack.restype = C.c_int
        L.blast_bsr_unpack.argtypes = [pv, vp, i64, vp]
        L.blast_bsr_transpose.restype = C.c_int
        L.blast_bsr_transpose.argtypes = [pv, vp, vp, vp, vp, vp, sz, C.POINTER(C.c_int32), vp]
        L.blast_bsr_sddmm.restype = C.c_int
        L.blast_bsr_sddmm.argtypes = [pv, vp, i64, vp, i64, i32, i64, vp, vp]
        L.blast_sparse_mlp_events.restype = C.c_int
        L.blast_sparse_mlp_events.argtypes = L.blast_sparse_mlp.argtypes + [C.POINTER(vp)]
        L.blast_bsr_joint_row_order.restype = C.c_int
        L.blast_bsr_joint_row_order.argtypes = [pv, pv, vp, vp]
        L.blast_bsr_gated_spmm.restype = C.c_int
        L.blast_bsr_gated_spmm.argtypes = [pv, pv, vp, i64, i32, i64, i32, vp, i64, vp]
        _lib = L
    return _lib


def _check(rc: int, where: str):
    if rc != 0:
        raise BlastError(rc, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def n_keep(n_blocks: int, sparsity: float) -> int:
    return int(lib().blast_n_keep(n_blocks, float(sparsity)))


@dataclass
class PackedBsr:
    """Device-resident packed matrix: tensors own the memory, `view()` is what the C ABI reads."""
    rows: int
    cols: int
    b: int
    nnz: int
    row_ptr: torch.Tensor  # int32 [rows/b + 1]
    col_idx: torch.Tensor  # int32 [cap]
    vals: torch.Tensor  # int16 (bf16 bits) [cap * b * b]
    row_order: torch.Tensor  # int32 [rows/b]
    aux: Optional[torch.Tensor]  # uint8
    max_row_blocks: int = 0  # stored blocks of the fullest block row (reported by the packer)

    def view(self) -> BsrView:
        """The C struct for this matrix; rebuilt only when an address or a scalar field has changed (a
        decode-sized call is otherwise dominated by marshalling on the host)."""
        key = (self.rows, self.cols, self.b, self.max_row_blocks, self.nnz, self.row_ptr.data_ptr(),
               self.col_idx.data_ptr(), self.vals.data_ptr(), self.row_order.data_ptr(),
               self.aux.data_ptr() if self.aux is not None else None)
        cached = self.__dict__.get("_view_cache")
        if cached is not None and cached[0] == key:
            return cached[1]
        v = BsrView(*key)
        self.__dict__["_view_cache"] = (key, v)
        return v

    def weight_bytes(self) -> int:
        return self.nnz * self.b * self.b * 2


def bsr_pack(W: torch.Tensor, b: int, *, mask: Optional[torch.Tensor] = None, sparsity: Optional[float] = None,
             nnz_cap: Optional[int] = None, with_aux: bool = True) -> PackedBsr:
    """blast_bsr_pack.  W: [rows, cols] bf16 (or int16 bit patterns) on the GPU.
    Exactly one of `mask` (uint8 [rows/b, cols/b] on the GPU) and `sparsity` selects the mode."""
    L = lib()
    assert W.is_cuda and W.dim() == 2 and W.stride(1) == 1 and W.element_size() == 2
    assert (mask is None) != (sparsity is None), "give exactly one of mask / sparsity"
    rows, cols = W.shape
    mode = PACK_MASK if mask is not None else PACK_TOPK_FROBENIUS
    s = 0.0 if sparsity is None else float(sparsity)
    cap, auxb, wsb = C.c_int64(0), C.c_size_t(0), C.c_size_t(0)
    _check(L.blast_bsr_pack_bound(rows, cols, b, mode, s, C.byref(cap), C.byref(auxb), C.byref(wsb)),
           "blast_bsr_pack_bound")
    if mask is not None:
        assert mask.is_cuda and mask.dtype == torch.uint8 and mask.is_contiguous()
    cap_v = int(cap.value) if nnz_cap is None else int(nnz_cap)
    aux_bytes = int(L.blast_bsr_aux_bytes(rows, cols, b, cap_v))
    dev = W.device
    row_ptr = torch.empty(rows // b + 1, dtype=torch.int32, device=dev)
    col_idx = torch.empty(max(cap_v, 1), dtype=torch.int32, device=dev)
    vals = torch.empty(max(cap_v, 1) * b * b, dtype=torch.int16, device=dev)
    row_order = torch.empty(max(rows // b, 1), dtype=torch.int32, device=dev)
    aux = torch.empty(max(aux_bytes, 16), dtype=torch.uint8, device=dev) if with_aux else None
    ws = torch.empty(int(wsb.value), dtype=torch.uint8, device=dev)
    nnz, heavy = C.c_int64(-1), C.c_int32(0)
    rc = L.blast_bsr_pack(_ptr(W), W.stride(0), rows, cols, b, mode, _ptr(mask), s, _ptr(row_ptr), _ptr(col_idx),
                          _ptr(vals), _ptr(row_order), _ptr(aux), aux_bytes if with_aux else 0, cap_v, C.byref(nnz),
                          C.byref(heavy), _ptr(ws), ws.numel(), _stream())
    _check(rc, "blast_bsr_pack")  # (the call has synchronised the stream: ws can go)
    return PackedBsr(rows, cols, b, int(nnz.value), row_ptr, col_idx, vals, row_order, aux, int(heavy.value))


def bsr_pack_many(Ws, b: int, *, masks=None, sparsity: Optional[float] = None, with_aux: bool = True):
    """blast_bsr_pack_enqueue for every matrix of `Ws` (same block size; `masks` a list of block masks, or one
    `sparsity` for the scoring mode): the re-packing of all the weights of a model after a mask update.  One
    allocation holds the outputs of all matrices, one scratch buffer serves them in turn, and the host
    synchronises once, at the end; the tensors of the results are views into that allocation."""
    L = lib()
    assert (masks is None) != (sparsity is None), "give exactly one of masks / sparsity"
    mode = PACK_MASK if masks is not None else PACK_TOPK_FROBENIUS
    s = 0.0 if sparsity is None else float(sparsity)
    if not Ws:
        return []
    dev = Ws[0].device
    cap, auxb, wsb = C.c_int64(0), C.c_size_t(0), C.c_size_t(0)
    total, ws_max, plans = 0, 0, []
    for W in Ws:
        assert W.is_cuda and W.dim() == 2 and W.stride(1) == 1 and W.element_size() == 2
        rows, cols = W.shape
        _check(L.blast_bsr_pack_bound(rows, cols, b, mode, s, C.byref(cap), C.byref(auxb), C.byref(wsb)),
               "blast_bsr_pack_bound")
        cap_v, aux_bytes, nbr = int(cap.value), int(auxb.value), rows // b
        ws_max = max(ws_max, int(wsb.value))
        sizes = (4 * (nbr + 1), 4 * max(nbr, 1), 4 * max(cap_v, 1), max(aux_bytes, 16) if with_aux else 0,
                 2 * max(cap_v, 1) * b * b)
        offs = []
        for nbytes in sizes:  # row_ptr, row_order, col_idx, aux, vals: each on a 256-byte boundary
            offs.append(total)
            total += (nbytes + 255) // 256 * 256
        plans.append((rows, cols, cap_v, aux_bytes, sizes, offs))
    arena = torch.empty(total, dtype=torch.uint8, device=dev)
    ws = torch.empty(ws_max, dtype=torch.uint8, device=dev)
    result = torch.empty((len(Ws), 2), dtype=torch.int32, device=dev)
    base, ws_p, res_p, stream = arena.data_ptr(), ws.data_ptr(), result.data_ptr(), _stream()
    for i, W in enumerate(Ws):
        rows, cols, cap_v, aux_bytes, sizes, (o_rp, o_ro, o_ci, o_aux, o_vals) = plans[i]
        mask = masks[i] if masks is not None else None
        if mask is not None:
            assert mask.is_cuda and mask.dtype == torch.uint8 and mask.is_contiguous()
        rc = L.blast_bsr_pack_enqueue(W.data_ptr(), W.stride(0), rows, cols, b, mode,
                                      None if mask is None else mask.data_ptr(), s, base + o_rp, base + o_ci,
                                      base + o_vals, base + o_ro, base + o_aux if with_aux else None,
                                      aux_bytes if with_aux else 0, cap_v, res_p + 8 * i, ws_p, ws_max, stream)
        _check(rc, "blast_bsr_pack_enqueue")
    # the views are made while the device works
    i32 = arena.view(torch.int32)
    out = []
    for rows, cols, cap_v, aux_bytes, sizes, (o_rp, o_ro, o_ci, o_aux, o_vals) in plans:
        nbr = rows // b
        out.append((i32[o_rp // 4:o_rp // 4 + nbr + 1], i32[o_ci // 4:o_ci // 4 + max(cap_v, 1)],
                    arena[o_vals:o_vals + sizes[4]].view(torch.int16), i32[o_ro // 4:o_ro // 4 + max(nbr, 1)],
                    arena[o_aux:o_aux + sizes[3]] if with_aux else None))
    res = result.cpu().tolist()  # synchronises: every matrix is complete, ws can go
    packed = []
    for (rows, cols, cap_v, *_), (row_ptr, col_idx, vals, row_order, aux), (nnz, heavy) in zip(plans, out, res):
        if nnz > cap_v:
            _check(-4, "blast_bsr_pack_enqueue")
        packed.append(PackedBsr(rows, cols, b, nnz, row_ptr, col_idx, vals, row_order, aux, heavy))
    return packed


def with_joint_row_order(gate: PackedBsr, up: PackedBsr) -> PackedBsr:
    """blast_bsr_joint_row_order: the same packed gate matrix (shared arrays) whose schedule accounts for
    the blocks of `up` as well.  Use the result as the `gate` argument of sparse_mlp / bsr_gated_spmm."""
    import dataclasses

    order = torch.empty_like(gate.row_order)
    vg, vu = gate.view(), up.view()
    _check(lib().blast_bsr_joint_row_order(C.byref(vg), C.byref(vu), _ptr(order), _stream()),
           "blast_bsr_joint_row_order")
    return dataclasses.replace(gate, row_order=order)


def generate_masks(W: torch.Tensor, G: torch.Tensor, b: int, sparsity: float) -> torch.Tensor:
    """blast_generate_masks: uint8 [rows/b, cols/b]; 1 = kept by the weight's ranking, 2 = regrown, 0 = dropped."""
    L = lib()
    for t in (W, G):
        assert t.is_cuda and t.dim() == 2 and t.stride(1) == 1 and t.element_size() == 2
    assert W.shape == G.shape
    rows, cols = W.shape
    mask = torch.empty((rows // b, cols // b), dtype=torch.uint8, device=W.device)
    ws = torch.empty(max(int(L.blast_generate_masks_workspace(rows, cols, b)), 16), dtype=torch.uint8, device=W.device)
    _check(L.blast_generate_masks(_ptr(W), W.stride(0), _ptr(G), G.stride(0), rows, cols, b, float(sparsity),
                                  _ptr(mask), _ptr(ws), ws.numel(), _stream()), "blast_generate_masks")
    torch.cuda.current_stream().synchronize()  # ws is released on return
    return mask


def pooled_topk_mask(S: torch.Tensor, b: int, sparsity: float) -> torch.Tensor:
    """blast_pooled_topk_mask: keep the blocks with the highest mean sensitivity; uint8 [rows/b, cols/b]."""
    L = lib()
    assert S.is_cuda and S.dim() == 2 and S.stride(1) == 1 and S.dtype == torch.float32
    rows, cols = S.shape
    mask = torch.empty((rows // b, cols // b), dtype=torch.uint8, device=S.device)
    ws = torch.empty(max(int(L.blast_pooled_topk_mask_workspace(rows, cols, b)), 16), dtype=torch.uint8, device=S.device)
    _check(L.blast_pooled_topk_mask(_ptr(S), S.stride(0), rows, cols, b, float(sparsity), _ptr(mask), _ptr(ws),
                                    ws.numel(), _stream()), "blast_pooled_topk_mask")
    torch.cuda.current_stream().synchronize()  # ws is released on return
    return mask


def sparsity_schedule(i: int, m: int, d: int, s_init: float, s_max: float) -> float:
    """blast_sparsity_schedule: Eq. (2)."""
    return float(lib().blast_sparsity_schedule(int(i), int(m), int(d), float(s_init), float(s_max)))


def bsr_unpack(W: PackedBsr, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """blast_bsr_unpack: the dense pruned weight, bf16 [rows, cols], zeros outside the stored blocks."""
    D = out if out is not None else torch.empty((W.rows, W.cols), dtype=torch.bfloat16, device=W.row_ptr.device)
    assert D.is_cuda and D.dim() == 2 and D.stride(1) == 1 and D.element_size() == 2 and D.shape == (W.rows, W.cols)
    v = W.view()
    _check(lib().blast_bsr_unpack(C.byref(v), _ptr(D), D.stride(0), _stream()), "blast_bsr_unpack")
    return D


def quantize_e5m2(x: torch.Tensor) -> torch.Tensor:
    """blast_quantize_e5m2: bf16 (or int16 bit patterns) tensor -> uint8 E5M2 codes of the same shape."""
    assert x.is_cuda and x.is_contiguous() and x.element_size() == 2
    out = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    _check(lib().blast_quantize_e5m2(_ptr(x), x.numel(), _ptr(out), _stream()), "blast_quantize_e5m2")
    return out


def quantize_e5m2_groups(x: torch.Tensor) -> torch.Tensor:
    """blast_quantize_e5m2_groups: token-major bf16 [T, K] -> uint8 E5M2 codes in column groups, [K/64, T, 64]."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.element_size() == 2 and x.shape[1] % 64 == 0
    T, K = x.shape
    out = torch.empty((K // 64, T, 64), dtype=torch.uint8, device=x.device)
    _check(lib().blast_quantize_e5m2_groups(_ptr(x), x.stride(0), T, K, _ptr(out), _stream()),
           "blast_quantize_e5m2_groups")
    return out


def bsr_spmm_e5m2(W: PackedBsr, vals8: torch.Tensor, X8: torch.Tensor, *, layout: int = TOKEN_MAJOR,
                  out_dtype: torch.dtype = torch.float32, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """blast_bsr_spmm_e5m2: Y = W * X with E5M2 block values `vals8` (quantize_e5m2(W.vals)) and E5M2 activations
    (token-major, feature-major, or the [K/64, T, 64] tensor of quantize_e5m2_groups with layout=COLUMN_GROUPS_64)."""
    assert X8.is_cuda and X8.dtype == torch.uint8
    assert vals8.dtype == torch.uint8 and vals8.numel() >= W.nnz * W.b * W.b
    if layout == COLUMN_GROUPS_64:
        assert X8.dim() == 3 and X8.is_contiguous() and X8.shape[2] == 64
        T, K = X8.shape[1], X8.shape[0] * 64
    else:
        assert X8.dim() == 2 and X8.stride(1) == 1
        T, K = X8.shape if layout == TOKEN_MAJOR else (X8.shape[1], X8.shape[0])
    assert K == W.cols
    Y = out if out is not None else _alloc_out(W.rows, T, TOKEN_MAJOR if layout == COLUMN_GROUPS_64 else layout,
                                               out_dtype, X8.device)
    v = W.view()
    _check(lib().blast_bsr_spmm_e5m2(C.byref(v), _ptr(vals8), _ptr(X8), X8.stride(-2), layout, T, _ptr(Y), Y.stride(0),
                                     BF16 if Y.dtype == torch.bfloat16 else F32, _stream()), "blast_bsr_spmm_e5m2")
    return Y


def bsr_transpose(W: PackedBsr) -> PackedBsr:
    """blast_bsr_transpose: the packed W~^T; bsr_spmm on it computes dX = W~^T dY."""
    L = lib()
    assert W.aux is not None, "pack with with_aux=True: the transpose reads the column-grouped index"
    b, dev = W.b, W.row_ptr.device
    n = max(W.nnz, 1)
    row_ptr = torch.empty(W.cols // b + 1, dtype=torch.int32, device=dev)
    col_idx = torch.empty(n, dtype=torch.int32, device=dev)
    vals = torch.empty(n * b * b, dtype=torch.int16, device=dev)
    row_order = torch.empty(max(W.cols // b, 1), dtype=torch.int32, device=dev)
    aux_bytes = int(L.blast_bsr_aux_bytes(W.cols, W.rows, b, W.nnz))
    aux = torch.empty(max(aux_bytes, 16), dtype=torch.uint8, device=dev)
    heavy = C.c_int32(0)
    v = W.view()
    _check(L.blast_bsr_transpose(C.byref(v), _ptr(row_ptr), _ptr(col_idx), _ptr(vals), _ptr(row_order), _ptr(aux),
                                 aux_bytes, C.byref(heavy), _stream()), "blast_bsr_transpose")
    return PackedBsr(W.cols, W.rows, b, W.nnz, row_ptr, col_idx, vals, row_order, aux, int(heavy.value))


def bsr_sddmm(W: PackedBsr, dY: torch.Tensor, X: torch.Tensor, *, layout: int = TOKEN_MAJOR,
              out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """blast_bsr_sddmm: gradient of the stored blocks, fp32 [nnz, b, b] (entries of dY X^T on kept blocks)."""
    L = lib()
    T, M, ldy = _layout_dims(dY, layout)
    T2, K, ldx = _layout_dims(X, layout)
    assert M == W.rows and K == W.cols and T == T2
    dv = out if out is not None else torch.empty((W.nnz, W.b, W.b), dtype=torch.float32, device=X.device)
    assert dv.dtype == torch.float32 and dv.is_contiguous() and dv.numel() == W.nnz * W.b * W.b
    v = W.view()
    _check(L.blast_bsr_sddmm(C.byref(v), _ptr(dY), ldy, _ptr(X), ldx, layout, T, _ptr(dv), _stream()), "blast_bsr_sddmm")
    return dv


def _layout_dims(X: torch.Tensor, layout: int):
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1 and X.element_size() == 2
    if layout == TOKEN_MAJOR:
        return X.shape[0], X.shape[1], X.stride(0)  # T, K, ld
    return X.shape[1], X.shape[0], X.stride(0)


def _alloc_out(rows: int, T: int, layout: int, out_dtype: torch.dtype, dev) -> torch.Tensor:
    shape = (T, rows) if layout == TOKEN_MAJOR else (rows, T)
    return torch.empty(shape, dtype=out_dtype, device=dev)


def bsr_spmm(W: PackedBsr, X: torch.Tensor, *, layout: int = TOKEN_MAJOR, out_dtype: torch.dtype = torch.float32,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """blast_bsr_spmm: Y = W * X.  X is [T, cols] (TOKEN_MAJOR) or [cols, T] (FEATURE_MAJOR), bf16."""
    L = lib()
    T, K, ldx = _layout_dims(X, layout)
    assert K == W.cols
    Y = out if out is not None else _alloc_out(W.rows, T, layout, out_dtype, X.device)
    v = W.view()
    wsb = C.c_size_t(0)
    _check(L.blast_bsr_spmm_workspace(C.byref(v), T, C.byref(wsb)), "blast_bsr_spmm_workspace")
    ws = torch.empty(int(wsb.value), dtype=torch.uint8, device=X.device) if wsb.value else None
    _check(L.blast_bsr_spmm(C.byref(v), _ptr(X), ldx, layout, T, _ptr(Y), Y.stride(0),
                            BF16 if Y.dtype == torch.bfloat16 else F32, _ptr(ws), int(wsb.value), _stream()),
           "blast_bsr_spmm")
    return Y


def mlp_workspace_bytes(gate: PackedBsr, up: PackedBsr, down: PackedBsr, T: int) -> int:
    vg, vu, vd = gate.view(), up.view(), down.view()
    wsb = C.c_size_t(0)
    _check(lib().blast_sparse_mlp_workspace(C.byref(vg), C.byref(vu), C.byref(vd), T, C.byref(wsb)),
           "blast_sparse_mlp_workspace")
    return int(wsb.value)


def sparse_mlp(gate: PackedBsr, up: PackedBsr, down: PackedBsr, X: torch.Tensor, *, layout: int = TOKEN_MAJOR,
               act: str = "silu", out_dtype: torch.dtype = torch.float32, out: Optional[torch.Tensor] = None,
               ws: Optional[torch.Tensor] = None, events=None) -> torch.Tensor:
    """blast_sparse_mlp: Y = Wdown * (act(Wgate * X) (.) (Wup * X)).
    `events`: optional ctypes array of 3 hipEvent_t -> blast_sparse_mlp_events."""
    L = lib()
    T, K, ldx = _layout_dims(X, layout)
    assert K == gate.cols
    Y = out if out is not None else _alloc_out(down.rows, T, layout, out_dtype, X.device)
    vg, vu, vd = gate.view(), up.view(), down.view()
    if ws is None:
        ws = torch.empty(max(mlp_workspace_bytes(gate, up, down, T), 256), dtype=torch.uint8, device=X.device)
    args = (C.byref(vg), C.byref(vu), C.byref(vd), _ptr(X), ldx, layout, T, ACT[act], _ptr(Y), Y.stride(0),
            BF16 if Y.dtype == torch.bfloat16 else F32, _ptr(ws), ws.numel(), _stream())
    if events is None:
        _check(L.blast_sparse_mlp(*args), "blast_sparse_mlp")
    else:
        _check(L.blast_sparse_mlp_events(*args, events), "blast_sparse_mlp_events")
    return Y


def sparse_mlp_e5m2w(gate: PackedBsr, gate8: torch.Tensor, up: PackedBsr, up8: torch.Tensor, down: PackedBsr,
                     down8: torch.Tensor, X: torch.Tensor, *, act: str = "silu", out_dtype: torch.dtype = torch.float32,
                     out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """blast_sparse_mlp_e5m2w: the gated MLP with E5M2 block values (quantize_e5m2 of each matrix's vals),
    token-major bf16 activations."""
    L = lib()
    T, K, ldx = _layout_dims(X, TOKEN_MAJOR)
    assert K == gate.cols
    for v8, m in ((gate8, gate), (up8, up), (down8, down)):
        assert v8.is_cuda and v8.dtype == torch.uint8 and v8.numel() >= m.nnz * m.b * m.b
    Y = out if out is not None else _alloc_out(down.rows, T, TOKEN_MAJOR, out_dtype, X.device)
    vg, vu, vd = gate.view(), up.view(), down.view()
    if ws is None:
        wsb = C.c_size_t(0)
        _check(L.blast_sparse_mlp_e5m2w_workspace(C.byref(vg), T, C.byref(wsb)), "blast_sparse_mlp_e5m2w_workspace")
        ws = torch.empty(max(int(wsb.value), 256), dtype=torch.uint8, device=X.device)
    _check(L.blast_sparse_mlp_e5m2w(C.byref(vg), _ptr(gate8), C.byref(vu), _ptr(up8), C.byref(vd), _ptr(down8), _ptr(X),
                                    ldx, T, ACT[act], _ptr(Y), Y.stride(0), BF16 if Y.dtype == torch.bfloat16 else F32,
                                    _ptr(ws), ws.numel(), _stream()), "blast_sparse_mlp_e5m2w")
    return Y


def sparse_mlp_status(gate: PackedBsr, T: int, ws: Optional[torch.Tensor]) -> int:
    """blast_sparse_mlp_status: 0 = every in-kernel wait of the single-launch form ended normally; ws=None asks
    about the library's own scratch (sparse_mlp_static).  Waits for the current stream."""
    vg = gate.view()
    st = C.c_int32(-1)
    _check(lib().blast_sparse_mlp_status(C.byref(vg), T, _ptr(ws), ws.numel() if ws is not None else 0, C.byref(st),
                                         _stream()), "blast_sparse_mlp_status")
    return int(st.value)


def sparse_mlp_static(gate: PackedBsr, up: PackedBsr, down: PackedBsr, X: torch.Tensor, out: torch.Tensor, *,
                      layout: int = TOKEN_MAJOR, act: str = "silu") -> torch.Tensor:
    """blast_sparse_mlp_static: blast_sparse_mlp with the scratch in the library's own device array; the
    caller passes the output tensor, nothing is allocated on the way."""
    T, K, ldx = _layout_dims(X, layout)
    assert K == gate.cols
    vg, vu, vd = gate.view(), up.view(), down.view()
    _check(lib().blast_sparse_mlp_static(C.byref(vg), C.byref(vu), C.byref(vd), _ptr(X), ldx, layout, T, ACT[act],
                                         _ptr(out), out.stride(0), BF16 if out.dtype == torch.bfloat16 else F32,
                                         _stream()), "blast_sparse_mlp_static")
    return out


class PreparedCall:
    """A C-ABI call with its arguments marshalled once: calling it costs one foreign call.  For loops that
    repeat a launch with the same buffers (decode steps, benchmarks), where argument conversion on the host
    would otherwise take longer than the kernels.  Holds references to every tensor it points into."""

    __slots__ = ("_fn", "_args", "_where", "_keep")

    def __init__(self, fn, where, args, keep):
        self._fn, self._where, self._args, self._keep = fn, where, args, keep

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != 0:
            raise BlastError(rc, self._where)


def prepare_sparse_mlp(gate: PackedBsr, up: PackedBsr, down: PackedBsr, X: torch.Tensor, out: torch.Tensor,
                       ws: torch.Tensor, *, layout: int = TOKEN_MAJOR, act: str = "silu", events=None) -> PreparedCall:
    """blast_sparse_mlp (or blast_sparse_mlp_events) on the current stream with fixed buffers, as a PreparedCall."""
    L = lib()
    T, K, ldx = _layout_dims(X, layout)
    assert K == gate.cols
    vg, vu, vd = gate.view(), up.view(), down.view()
    args = [C.byref(vg), C.byref(vu), C.byref(vd), _ptr(X), C.c_int64(ldx), C.c_int32(layout), C.c_int64(T),
            C.c_int32(ACT[act]), _ptr(out), C.c_int64(out.stride(0)),
            C.c_int32(BF16 if out.dtype == torch.bfloat16 else F32), _ptr(ws), C.c_size_t(ws.numel()), _stream()]
    keep = (vg, vu, vd, gate, up, down, X, out, ws, events)
    if events is None:
        return PreparedCall(L.blast_sparse_mlp, "blast_sparse_mlp", tuple(args), keep)
    return PreparedCall(L.blast_sparse_mlp_events, "blast_sparse_mlp_events", tuple(args + [events]), keep)


def mlp2_workspace_bytes(w1: PackedBsr, w2: PackedBsr, T: int) -> int:
    v1, v2 = w1.view(), w2.view()
    wsb = C.c_size_t(0)
    _check(lib().blast_sparse_mlp2_workspace(C.byref(v1), C.byref(v2), T, C.byref(wsb)), "blast_sparse_mlp2_workspace")
    return int(wsb.value)


def sparse_mlp2(w1: PackedBsr, w2: PackedBsr, X: torch.Tensor, *, layout: int = TOKEN_MAJOR, act: str = "gelu",
                out_dtype: torch.dtype = torch.float32, out: Optional[torch.Tensor] = None,
                ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """blast_sparse_mlp2: Y = W2 * act(W1 * X)."""
    L = lib()
    T, K, ldx = _layout_dims(X, layout)
    assert K == w1.cols
    Y = out if out is not None else _alloc_out(w2.rows, T, layout, out_dtype, X.device)
    v1, v2 = w1.view(), w2.view()
    if ws is None:
        ws = torch.empty(max(mlp2_workspace_bytes(w1, w2, T), 256), dtype=torch.uint8, device=X.device)
    _check(L.blast_sparse_mlp2(C.byref(v1), C.byref(v2), _ptr(X), ldx, layout, T, ACT[act], _ptr(Y), Y.stride(0),
                               BF16 if Y.dtype == torch.bfloat16 else F32, _ptr(ws), ws.numel(), _stream()),
           "blast_sparse_mlp2")
    return Y


def bsr_gated_spmm(gate: PackedBsr, up: PackedBsr, X: torch.Tensor, *, layout: int = TOKEN_MAJOR, act: str = "silu",
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """blast_bsr_gated_spmm: H = act(Wgate * X) (.) (Wup * X), bf16, same layout as X."""
    L = lib()
    T, K, ldx = _layout_dims(X, layout)
    assert K == gate.cols
    H = out if out is not None else _alloc_out(gate.rows, T, layout, torch.bfloat16, X.device)
    vg, vu = gate.view(), up.view()
    _check(L.blast_bsr_gated_spmm(C.byref(vg), C.byref(vu), _ptr(X), ldx, layout, T, ACT[act], _ptr(H), H.stride(0),
                                  _stream()), "blast_bsr_gated_spmm")
    return H
