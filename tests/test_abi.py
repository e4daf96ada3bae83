"""Host-side checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

from oracle import oracle as orc
from paper_2507_03117_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    txt = open(os.path.join(ROOT, "include", "blast.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(blast_[a-z0-9_]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    L = api.lib()
    syms = declared_symbols()
    assert set(syms) == set(api.EXPORTS)
    for s in syms:
        assert hasattr(L, s), s


def test_strerror_texts():
    L = api.lib()
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        t = L.blast_strerror(code)
        assert t and len(t) > 1
        seen.add(t)
    assert len(seen) == 8


@pytest.mark.parametrize("n,s", [(4096, 0.9), (6144, 0.7), (6144, 0.8), (6144, 0.9), (6144, 0.95), (3584, 0.95),
                                 (53248, 0.95), (10, 0.0), (10, 1.0), (7, 0.5), (3, 0.34), (12345, 0.3333)])
def test_n_keep_matches_oracle(n, s):
    assert api.n_keep(n, s) == orc.n_keep(n, s)


def test_n_keep_rejects_bad_sparsity():
    assert api.n_keep(10, -0.1) == -1 and api.n_keep(10, 1.5) == -1 and api.n_keep(-1, 0.5) == -1


def test_pack_bound_and_errors():
    L = api.lib()
    cap, auxb, wsb = C.c_int64(0), C.c_size_t(0), C.c_size_t(0)
    assert L.blast_bsr_pack_bound(8192, 2048, 64, api.PACK_TOPK_FROBENIUS, 0.9, C.byref(cap), C.byref(auxb), C.byref(wsb)) == 0
    assert cap.value == 409 and auxb.value >= 4 * (32 + 1 + 2 * 409) + 12 * (128 + 4096 // 16) and wsb.value >= 9 * 4096
    assert L.blast_bsr_pack_bound(8192, 2048, 64, api.PACK_MASK, 0.0, C.byref(cap), None, None) == 0
    assert cap.value == 4096
    assert L.blast_bsr_pack_bound(8192, 2050, 64, 0, 0.0, None, None, None) == -2  # shape
    assert L.blast_bsr_pack_bound(8192, 2048, 48, 0, 0.0, None, None, None) == -3  # block
    assert L.blast_bsr_pack_bound(8192, 2048, 64, 7, 0.0, None, None, None) == -1  # mode
    assert L.blast_bsr_pack_bound(8192, 2048, 64, 1, 1.5, None, None, None) == -1  # sparsity
    assert L.blast_bsr_aux_bytes(8192, 2048, 64, 4096) >= 4 * (32 + 1 + 2 * 4096)


def test_pack_argument_errors_return_before_any_launch():
    """blast_bsr_pack and blast_bsr_pack_enqueue check every argument before they touch the GPU."""
    L = api.lib()
    nnz, heavy = C.c_int64(0), C.c_int32(0)
    buf = (C.c_int64 * 8)()  # (stands in for device pointers: no call below gets as far as using them)
    p = C.cast(buf, C.c_void_p)
    common = (p, 128, 128, 128, 64, api.PACK_MASK, p, 0.0, p, p, p, p, None, 0, 4)
    assert L.blast_bsr_pack(*common, None, C.byref(heavy), p, 1 << 20, None) == -1  # nnz_out missing
    assert L.blast_bsr_pack(*common, C.byref(nnz), C.byref(heavy), None, 0, None) == -5  # no workspace
    assert L.blast_bsr_pack(p, 128, 130, 128, 64, 0, p, 0.0, p, p, p, p, None, 0, 4, C.byref(nnz), None, p, 1 << 20,
                            None) == -2  # rows not a multiple of b
    assert L.blast_bsr_pack(p, 64, 128, 128, 64, 0, p, 0.0, p, p, p, p, None, 0, 4, C.byref(nnz), None, p, 1 << 20,
                            None) == -1  # row pitch shorter than a row
    assert L.blast_bsr_pack(p, 128, 128, 128, 64, 0, None, 0.0, p, p, p, p, None, 0, 4, C.byref(nnz), None, p, 1 << 20,
                            None) == -1  # mask mode without a mask
    assert L.blast_bsr_pack(p, 128, 128, 128, 64, 1, None, 1.5, p, p, p, p, None, 0, 4, C.byref(nnz), None, p, 1 << 20,
                            None) == -1  # sparsity out of range
    assert L.blast_bsr_pack_enqueue(*common, None, p, 1 << 20, None) == -1  # result missing
    assert L.blast_bsr_pack_enqueue(*common, C.c_void_p(p.value + 4), p, 1 << 20, None) == -1  # result misaligned
    assert L.blast_bsr_pack_enqueue(*common, p, None, 0, None) == -5  # no workspace
    assert L.blast_bsr_pack_enqueue(p, 128, 128, 128, 48, 0, p, 0.0, p, p, p, p, None, 0, 4, p, p, 1 << 20, None) == -3
    assert L.blast_bsr_pack_enqueue(p, 128, 128, 128, 64, 0, p, 0.0, p, p, p, p, p, 8, 4, p, p, 1 << 20, None) == -5  # aux too small


def test_spmm_and_mlp_argument_errors_return_before_any_launch():
    L = api.lib()
    v = api.BsrView(128, 128, 64, 0, 0, None, None, None, None, None)
    # null row_ptr
    assert L.blast_bsr_spmm(C.byref(v), None, 128, 0, 4, None, 128, 0, None, 0, None) == -1
    assert L.blast_bsr_spmm(None, None, 128, 0, 4, None, 128, 0, None, 0, None) == -1
    dummy = (C.c_int32 * 4)()
    v.row_ptr = C.cast(dummy, C.c_void_p)
    assert L.blast_bsr_spmm(C.byref(v), None, 128, 0, 4, None, 128, 0, None, 0, None) == -1  # X null
    assert L.blast_bsr_spmm(C.byref(v), None, 128, 5, 0, None, 128, 0, None, 0, None) == -1  # layout enum
    assert L.blast_bsr_spmm(C.byref(v), None, 128, 0, -1, None, 128, 0, None, 0, None) == -1  # T < 0
    assert L.blast_bsr_spmm(C.byref(v), None, 128, 0, 0, None, 128, 0, None, 0, None) == 0  # T == 0 is a no-op
    bad = api.BsrView(100, 128, 64, 0, 0, v.row_ptr, None, None, None, None)
    assert L.blast_bsr_spmm(C.byref(bad), None, 128, 0, 4, None, 128, 0, None, 0, None) == -2
    bad = api.BsrView(96, 96, 48, 0, 0, v.row_ptr, None, None, None, None)
    assert L.blast_bsr_spmm(C.byref(bad), None, 128, 0, 4, None, 128, 0, None, 0, None) == -3
    # MLP: inconsistent shapes
    g = api.BsrView(256, 128, 64, 0, 0, v.row_ptr, None, None, None, None)
    d_ok = api.BsrView(128, 256, 64, 0, 0, v.row_ptr, None, None, None, None)
    d_bad = api.BsrView(128, 128, 64, 0, 0, v.row_ptr, None, None, None, None)
    assert L.blast_sparse_mlp(C.byref(g), C.byref(g), C.byref(d_bad), None, 128, 0, 4, 0, None, 128, 0, None, 0, None) == -2
    assert L.blast_sparse_mlp(C.byref(g), C.byref(g), C.byref(d_ok), None, 128, 0, 4, 9, None, 128, 0, None, 0, None) == -1
    assert L.blast_sparse_mlp(C.byref(g), None, C.byref(d_ok), None, 128, 0, 4, 0, None, 128, 0, None, 0, None) == -1
    ws = C.c_size_t(0)
    assert L.blast_sparse_mlp_workspace(C.byref(g), C.byref(g), C.byref(d_ok), 16, C.byref(ws)) == 0
    assert ws.value >= 16 * 256 * 2
    # two-matrix MLP: same checks
    assert L.blast_sparse_mlp2(C.byref(g), C.byref(d_bad), None, 128, 0, 4, 1, None, 128, 0, None, 0, None) == -2
    assert L.blast_sparse_mlp2(C.byref(g), C.byref(d_ok), None, 128, 0, 4, 9, None, 128, 0, None, 0, None) == -1
    assert L.blast_sparse_mlp2(C.byref(g), None, None, 128, 0, 4, 1, None, 128, 0, None, 0, None) == -1
    assert L.blast_sparse_mlp2(C.byref(g), C.byref(d_ok), None, 128, 0, 0, 1, None, 128, 0, None, 0, None) == 0  # T == 0
    ws2 = C.c_size_t(0)
    assert L.blast_sparse_mlp2_workspace(C.byref(g), C.byref(d_ok), 16, C.byref(ws2)) == 0
    assert ws2.value == ws.value
    # backward entry points
    assert L.blast_bsr_transpose(None, None, None, None, None, None, 0, None, None) == -1
    assert L.blast_bsr_transpose(C.byref(g), None, None, None, None, None, 0, None, None) == -5  # no aux on the input
    assert L.blast_bsr_sddmm(None, None, 128, None, 128, 0, 4, None, None) == -1
    assert L.blast_bsr_sddmm(C.byref(g), None, 128, None, 128, 0, 4, None, None) == 0  # nnz == 0: nothing to do
    g1 = api.BsrView(256, 128, 64, 0, 1, v.row_ptr, v.row_ptr, None, None, None)
    assert L.blast_bsr_sddmm(C.byref(g1), None, 256, None, 128, 0, 4, None, None) == -1  # dvals null
    assert L.blast_bsr_sddmm(C.byref(g1), None, 256, None, 128, 7, 4, None, None) == -1  # layout enum
    bad48 = api.BsrView(96, 96, 48, 0, 1, v.row_ptr, v.row_ptr, None, None, None)
    assert L.blast_bsr_sddmm(C.byref(bad48), None, 96, None, 96, 0, 4, None, None) == -3
    # mask update: shape / argument checks, and the schedule (host arithmetic, runs without a GPU)
    assert L.blast_generate_masks(None, 128, None, 128, 128, 128, 64, 0.5, None, None, 0, None) == -1
    assert L.blast_generate_masks(None, 128, None, 128, 100, 128, 64, 0.5, None, None, 0, None) == -2
    assert L.blast_generate_masks(None, 128, None, 128, 128, 128, 64, 1.5, None, None, 0, None) == -1
    assert L.blast_generate_masks_workspace(128, 128, 64) >= 4 * 8 + 2 * 4
    assert L.blast_sparsity_schedule(0, 9000, 1000, 0.1, 0.8) == pytest.approx(0.1, abs=1e-15)
    assert L.blast_sparsity_schedule(8000, 9000, 1000, 0.1, 0.8) == 0.8
    assert L.blast_sparsity_schedule(9000, 9000, 1000, 0.1, 0.8) == 0.8
    assert L.blast_sparsity_schedule(4000, 9000, 1000, 0.1, 0.8) == pytest.approx(0.8 - 0.7 / 8, abs=1e-15)
    assert L.blast_pooled_topk_mask(None, 128, 128, 128, 64, 0.5, None, None, 0, None) == -1
    assert L.blast_pooled_topk_mask(None, 128, 128, 100, 64, 0.5, None, None, 0, None) == -2
    assert L.blast_pooled_topk_mask_workspace(128, 128, 64) >= 4 * 8
    assert L.blast_bsr_unpack(None, None, 128, None) == -1
    assert L.blast_bsr_unpack(C.byref(g), None, 128, None) == -1  # W null
    assert L.blast_bsr_unpack(C.byref(bad48), None, 96, None) == -3
    # E5M2 entry points
    assert L.blast_quantize_e5m2(None, -1, None, None) == -1
    assert L.blast_quantize_e5m2(None, 0, None, None) == 0
    assert L.blast_quantize_e5m2(None, 8, None, None) == -1
    assert L.blast_quantize_e5m2_groups(None, 128, 4, 100, None, None) == -1  # K not a multiple of 64
    assert L.blast_quantize_e5m2_groups(None, 128, 0, 128, None, None) == 0
    assert L.blast_quantize_e5m2_groups(None, 128, 4, 128, None, None) == -1   # null pointers
    assert L.blast_bsr_spmm_e5m2(C.byref(g), None, None, 128, 3, 4, None, 256, 0, None) == -1  # layout enum
    assert L.blast_bsr_spmm_e5m2(None, None, None, 128, 0, 4, None, 128, 0, None) == -1
    assert L.blast_bsr_spmm_e5m2(C.byref(g), None, None, 128, 0, 4, None, 256, 0, None) == -1  # Y null
    assert L.blast_bsr_spmm_e5m2(C.byref(g), None, None, 128, 0, 0, None, 256, 0, None) == 0   # T == 0
    assert L.blast_bsr_spmm_e5m2(C.byref(bad48), None, None, 96, 0, 4, None, 96, 0, None) == -3
    # pack: null outputs / bad ld are rejected up front
    nnz = C.c_int64(0)
    assert L.blast_bsr_pack(None, 128, 128, 128, 64, 0, None, 0.0, None, None, None, None, None, 0, 4, C.byref(nnz), None, None, 0, None) == -1
