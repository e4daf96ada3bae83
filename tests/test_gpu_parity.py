"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Index arrays bit-exact; outputs within
rel-Frobenius <= 1e-3 and max-abs <= 1e-2 * RMS (tests/helpers.py)."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2507_03117_amd import synth
from tests.helpers import bits_of, check_close, long_row_case, long_scratch_bytes, mask_dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available()
    from paper_2507_03117_amd import api as _api

    _api.lib()
    return _api


def pack_both(api, W, b, mask=None, sparsity=None):
    """Pack on the device and with the oracle; assert bit-exact structure and values."""
    if mask is not None:
        ref = orc.pack(W, b, mask)
        dev = api.bsr_pack(to_dev(W), b, mask=mask_dev(mask))
    else:
        ref, ref_mask, gap = orc.pack_topk(W, b, sparsity)
        assert gap > 1e-9, "selection hangs on rounding: reseed"
        dev = api.bsr_pack(to_dev(W), b, sparsity=sparsity)
    assert dev.nnz == ref.nnz
    assert np.array_equal(dev.row_ptr.cpu().numpy(), ref.row_ptr)
    assert np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)
    assert np.array_equal(bits_of(dev.vals)[: ref.nnz * b * b].reshape(ref.nnz, b, b), ref.vals)
    if ref.row_order.size:
        assert np.array_equal(dev.row_order.cpu().numpy()[: ref.row_order.size], ref.row_order)
    return dev, ref


CHUNK = 16  # blocks per chunk of the packer's chunk plan (decode kernels)
WIDE_CHUNK = 64  # ... of its second plan (streaming kernels)


def check_aux(dev, ref):
    """aux = two chunk plans (rows in schedule order cut into chunks of <= 16 and of <= 64 blocks), the dense
    numbering of the rows that the first plan cuts and the index of their first chunk, then the column-grouped index (the same blocks by column,
    then ascending row)."""
    nbr, nbc = ref.rows // ref.b, ref.cols // ref.b
    aux = dev.aux.cpu().numpy()
    a16 = lambda x: (x + 15) // 16 * 16
    cnt = np.diff(ref.row_ptr)
    off = 0
    for chunk in (CHUNK, WIDE_CHUNK):
        cap = nbr + (nbr * nbc) // chunk + 1
        hdr = aux[off: off + 16].view(np.int32)
        off += 16
        chunk_row = aux[off: off + 4 * cap].view(np.int32)
        off += a16(4 * cap)
        chunk_kb = aux[off: off + 4 * cap].view(np.int32)
        off += a16(4 * cap)
        chunk_ke = aux[off: off + 4 * cap].view(np.int32)
        off += a16(4 * cap)
        # expected plan, written from the definition
        exp = []
        for r in ref.row_order:
            kb, ke = int(ref.row_ptr[r]), int(ref.row_ptr[r + 1])
            nch = max(1, -(-(ke - kb) // chunk))
            for j in range(nch):
                exp.append((int(r), nch > 1, kb + j * chunk, min(kb + (j + 1) * chunk, ke)))
        assert hdr[0] == len(exp) and hdr[1] == (int(cnt.max()) if cnt.size else 0) == dev.max_row_blocks and hdr[2] == chunk
        n_split = sum(1 for e in exp if e[1])
        assert hdr[3] == n_split and all(e[1] for e in exp[:n_split])  # the cut rows' chunks head the plan
        n = len(exp)
        assert [(int(c) & 0x7FFFFFFF, int(c) < 0, int(a), int(b_)) for c, a, b_ in
                zip(chunk_row[:n], chunk_kb[:n], chunk_ke[:n])] == exp
    row_slot = aux[off: off + 4 * nbr].view(np.int32)
    off += a16(4 * nbr)
    exp_slot = np.full(nbr, -1, dtype=np.int32)
    for rank, r in enumerate(ref.row_order):
        if cnt[r] > CHUNK:
            exp_slot[r] = rank
    assert np.array_equal(row_slot, exp_slot)
    row_chunk0 = aux[off: off + 4 * nbr].view(np.int32)
    off += a16(4 * nbr)
    exp_chunk0, at = np.full(nbr, -1, dtype=np.int32), 0
    for r in ref.row_order:
        if cnt[r] > CHUNK:
            exp_chunk0[r] = at
        at += max(1, -(-int(cnt[r]) // CHUNK))
    assert np.array_equal(row_chunk0, exp_chunk0)
    col_ptr = aux[off: off + 4 * (nbc + 1)].view(np.int32)
    off += a16(4 * (nbc + 1))
    csc_row = aux[off: off + 4 * ref.nnz].view(np.int32)
    off += a16(4 * ref.nnz)
    csc_blk = aux[off: off + 4 * ref.nnz].view(np.int32)
    rows_of_blk = np.repeat(np.arange(nbr), np.diff(ref.row_ptr))
    order = np.lexsort((rows_of_blk, ref.col_idx))  # by column, then row
    assert np.array_equal(col_ptr, np.concatenate([[0], np.cumsum(np.bincount(ref.col_idx, minlength=nbc))]))
    assert np.array_equal(csc_blk, order.astype(np.int32))
    assert np.array_equal(csc_row, rows_of_blk[order].astype(np.int32))


# ------------------------------------------------------------------ packing
@pytest.mark.parametrize("b", [16, 32, 64, 128])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_pack_mask_mode(api, b, sparsity):
    rng = np.random.default_rng(100 + b)
    nbr, nbc = 7, 11
    W = synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.02)
    mask = synth.uniform_mask(rng, nbr, nbc, sparsity)
    if 0 < sparsity < 1:
        mask[3, :] = 0
        mask[5, :] = 1
    dev, ref = pack_both(api, W, b, mask=mask)
    check_aux(dev, ref)


@pytest.mark.parametrize("b,rows,cols,sparsity", [(16, 256, 512, 0.7), (32, 1024, 4096, 0.9), (64, 2048, 1024, 0.95),
                                                  (128, 1024, 2048, 0.8), (64, 512, 512, 0.0), (64, 512, 512, 1.0)])
def test_pack_topk_mode(api, b, rows, cols, sparsity):
    rng = np.random.default_rng(200 + b)
    W = synth.gauss_bf16(rng, (rows, cols), 0.02)
    dev, ref = pack_both(api, W, b, sparsity=sparsity)
    assert ref.nnz == orc.n_keep((rows // b) * (cols // b), sparsity)
    check_aux(dev, ref)


def test_pack_topk_ties_and_zero_blocks(api):
    # all-zero blocks tie at score 0 and duplicated blocks tie exactly: lower linear index wins
    rng = np.random.default_rng(7)
    b, nbr, nbc = 32, 6, 8
    W = synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.02)
    Wv = W.reshape(nbr, b, nbc, b)
    Wv[0, :, 2:7, :] = 0
    Wv[4, :, :, :] = 0
    Wv[2, :, 1, :] = Wv[1, :, 5, :]
    Wv[5, :, 6, :] = Wv[1, :, 5, :]
    for s in (0.1, 0.5, 0.8, 0.9):
        ref_mask, _ = orc.topk_mask(orc.block_scores(W, b), s)
        ref = orc.pack(W, b, ref_mask)
        dev = api.bsr_pack(to_dev(W), b, sparsity=s)
        assert dev.nnz == ref.nnz
        assert np.array_equal(dev.row_ptr.cpu().numpy(), ref.row_ptr)
        assert np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)


@pytest.mark.parametrize("sparsity", [0.5, 0.9, 0.999])
def test_pack_topk_many_blocks(api, sparsity):
    """26624 blocks: the selection walks global memory until the keys that share the selected prefix fit in LDS
    (4096), collects them and finishes there."""
    rng = np.random.default_rng(210)
    b, rows, cols = 16, 2048, 3328
    W = synth.gauss_bf16(rng, (rows, cols), 0.02)
    dev, ref = pack_both(api, W, b, sparsity=sparsity)
    assert ref.nnz == orc.n_keep((rows // b) * (cols // b), sparsity)
    check_aux(dev, ref)


@pytest.mark.parametrize("sparsity", [0.3, 0.75])
def test_pack_topk_many_blocks_with_massive_ties(api, sparsity):
    """26624 blocks with only three distinct scores: the tied keys never fit in LDS, every pass runs over global
    memory, and the threshold is a tie that the index order has to cut (lower linear index wins)."""
    rng = np.random.default_rng(211)
    b, nbr, nbc = 16, 128, 208
    proto = synth.gauss_bf16(rng, (3, b, b), 0.02)
    which = rng.integers(0, 3, size=(nbr, nbc))
    W = np.ascontiguousarray(proto[which].transpose(0, 2, 1, 3).reshape(nbr * b, nbc * b))
    ref_mask, _ = orc.topk_mask(orc.block_scores(W, b), sparsity)
    ref = orc.pack(W, b, ref_mask)
    dev = api.bsr_pack(to_dev(W), b, sparsity=sparsity)
    assert dev.nnz == ref.nnz
    assert np.array_equal(dev.row_ptr.cpu().numpy(), ref.row_ptr)
    assert np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)
    assert np.array_equal(bits_of(dev.vals)[: ref.nnz * b * b].reshape(ref.nnz, b, b), ref.vals)


def test_pack_strided_weight_and_capacity_error(api):
    import torch

    rng = np.random.default_rng(8)
    b = 32
    Wfull = synth.gauss_bf16(rng, (128, 256 + 64), 0.02)
    W = Wfull[:, :256]
    mask = synth.uniform_mask(rng, 4, 8, 0.5)
    ref = orc.pack(np.ascontiguousarray(W), b, mask)
    dev = api.bsr_pack(to_dev(Wfull)[:, :256], b, mask=mask_dev(mask))  # ldw = 320
    assert np.array_equal(bits_of(dev.vals)[: ref.nnz * b * b].reshape(ref.nnz, b, b), ref.vals)
    with pytest.raises(api.BlastError) as ei:
        api.bsr_pack(to_dev(np.ascontiguousarray(W)), b, mask=mask_dev(mask), nnz_cap=ref.nnz - 1)
    assert ei.value.code == -4
    torch.cuda.synchronize()


def _assert_packed_equal(dev, ref, b):
    assert dev.nnz == ref.nnz
    assert np.array_equal(dev.row_ptr.cpu().numpy(), ref.row_ptr)
    assert np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)
    assert np.array_equal(bits_of(dev.vals)[: ref.nnz * b * b].reshape(ref.nnz, b, b), ref.vals)
    assert np.array_equal(dev.row_order.cpu().numpy()[: ref.row_order.size], ref.row_order)
    assert dev.max_row_blocks == int(np.diff(ref.row_ptr).max())
    check_aux(dev, ref)


@pytest.mark.parametrize("nbr,nbc", [(64, 128), (1, 8192), (8192, 1), (1024, 8), (3, 1024), (65, 128), (2, 1100),
                                     (1025, 4)])
def test_pack_single_workgroup_limits(api, nbr, nbc):
    """Up to 8192 blocks with at most 1024 block rows and columns one workgroup writes every index array; the cases
    sit on both sides of each of the three limits."""
    rng = np.random.default_rng(220 + nbr)
    b = 16
    W = synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.02)
    dev, ref = pack_both(api, W, b, sparsity=0.9)
    _assert_packed_equal(dev, ref, b)
    mask = synth.uniform_mask(rng, nbr, nbc, 0.8)
    dev, ref = pack_both(api, W, b, mask=mask)
    _assert_packed_equal(dev, ref, b)


@pytest.mark.parametrize("sparsity", [0.3, 0.75, 0.97])
def test_pack_single_workgroup_massive_ties(api, sparsity):
    """6400 blocks with three distinct scores: the threshold is a tie that the index order cuts."""
    rng = np.random.default_rng(212)
    b, nbr, nbc = 16, 64, 100
    proto = synth.gauss_bf16(rng, (3, b, b), 0.02)
    which = rng.integers(0, 3, size=(nbr, nbc))
    W = np.ascontiguousarray(proto[which].transpose(0, 2, 1, 3).reshape(nbr * b, nbc * b))
    ref_mask, _ = orc.topk_mask(orc.block_scores(W, b), sparsity)
    ref = orc.pack(W, b, ref_mask)
    dev = api.bsr_pack(to_dev(W), b, sparsity=sparsity)
    _assert_packed_equal(dev, ref, b)


def test_pack_random_shapes(api):
    """Forty seeded random block grids on both sides of the single-workgroup limits, random sparsities, both
    modes: every index array against the oracle."""
    rng = np.random.default_rng(240)
    b = 16
    done = 0
    while done < 40:
        nbr = int(rng.integers(1, 1300)) if rng.random() < 0.3 else int(rng.integers(1, 140))
        nbc = int(rng.integers(1, 1300)) if rng.random() < 0.3 else int(rng.integers(1, 140))
        if nbr * nbc > 20000:
            continue
        done += 1
        s = float(rng.choice([0.0, 0.37, 0.5, 0.8, 0.93, 0.99, 1.0]))
        W = synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.02)
        mask = synth.uniform_mask(rng, nbr, nbc, s)
        dev, ref = pack_both(api, W, b, mask=mask)
        _assert_packed_equal(dev, ref, b)
        ref_t, _, gap = orc.pack_topk(W, b, s)
        if gap > 1e-9:
            _assert_packed_equal(api.bsr_pack(to_dev(W), b, sparsity=s), ref_t, b)


def test_pack_many_matches_single_calls(api):
    """blast_bsr_pack_enqueue: three matrices of different shapes packed back to back with one shared scratch
    buffer and one synchronisation, in both modes; one of them takes the many-launch path."""
    rng = np.random.default_rng(230)
    b = 32
    shapes = [(128 * b, 32 * b), (32 * b, 128 * b), (96 * b, 100 * b)]
    Ws = [synth.gauss_bf16(rng, sh, 0.02) for sh in shapes]
    devs = api.bsr_pack_many([to_dev(W) for W in Ws], b, sparsity=0.9)
    for W, dev in zip(Ws, devs):
        ref, _, gap = orc.pack_topk(W, b, 0.9)
        assert gap > 1e-9
        _assert_packed_equal(dev, ref, b)
    masks = [synth.uniform_mask(rng, sh[0] // b, sh[1] // b, 0.85) for sh in shapes]
    devs = api.bsr_pack_many([to_dev(W) for W in Ws], b, masks=[mask_dev(m) for m in masks])
    for W, m, dev in zip(Ws, masks, devs):
        _assert_packed_equal(dev, orc.pack(W, b, m), b)


@pytest.mark.parametrize("shape", [(128, 32), (170, 100)])
def test_pack_enqueue_replays_from_a_graph(api, shape):
    """blast_bsr_pack_enqueue only enqueues kernels, so the re-packing of a weight whose values change (the mask
    update of every step_size iterations) can be recorded once and replayed: three replays on three different
    weights, with eager work in between, each against the oracle.  Both the single-workgroup path and the
    many-launch path."""
    import ctypes as C

    import torch

    rng = np.random.default_rng(250 + shape[0])
    b, (nbr, nbc), s = 32, shape, 0.85
    L = api.lib()
    cap, auxb, wsb = C.c_int64(0), C.c_size_t(0), C.c_size_t(0)
    assert L.blast_bsr_pack_bound(nbr * b, nbc * b, b, api.PACK_TOPK_FROBENIUS, s, C.byref(cap), C.byref(auxb),
                                  C.byref(wsb)) == 0
    dev = "cuda:0"
    W = torch.zeros((nbr * b, nbc * b), dtype=torch.bfloat16, device=dev)
    row_ptr = torch.empty(nbr + 1, dtype=torch.int32, device=dev)
    col_idx = torch.empty(cap.value, dtype=torch.int32, device=dev)
    vals = torch.empty(cap.value * b * b, dtype=torch.int16, device=dev)
    row_order = torch.empty(nbr, dtype=torch.int32, device=dev)
    aux = torch.empty(auxb.value, dtype=torch.uint8, device=dev)
    ws = torch.empty(wsb.value, dtype=torch.uint8, device=dev)
    result = torch.zeros(2, dtype=torch.int32, device=dev)

    def enqueue():
        rc = L.blast_bsr_pack_enqueue(W.data_ptr(), W.stride(0), nbr * b, nbc * b, b, api.PACK_TOPK_FROBENIUS, None, s,
                                      row_ptr.data_ptr(), col_idx.data_ptr(), vals.data_ptr(), row_order.data_ptr(),
                                      aux.data_ptr(), auxb.value, cap.value, result.data_ptr(), ws.data_ptr(),
                                      wsb.value, C.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()  # (warm-up outside the capture)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    for rep in range(3):
        w = synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.02)
        ref, _, gap = orc.pack_topk(w, b, s)
        assert gap > 1e-9
        W.copy_(to_dev(w))
        row_ptr.fill_(-1)
        col_idx.fill_(-1)
        result.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        assert result.cpu().tolist() == [ref.nnz, int(np.diff(ref.row_ptr).max())]
        packed = api.PackedBsr(nbr * b, nbc * b, b, ref.nnz, row_ptr, col_idx, vals, row_order, aux,
                               int(np.diff(ref.row_ptr).max()))
        _assert_packed_equal(packed, ref, b)


# ------------------------------------------------------------------ SpMM
@pytest.mark.parametrize("b", [16, 32, 64, 128])
@pytest.mark.parametrize("T", [1, 3, 17, 64, 100, 300])
def test_spmm_small_shapes(api, b, T):
    import torch

    nbr, nbc = 5, 6
    w, mask, x = synth.small_case(1000 + b + T, nbr * b, nbc * b, b, 0.5, T, empty_rows=(1,), full_rows=(3,))
    dev, ref = pack_both(api, w, b, mask=mask)
    y_or = orc.spmm(ref, x)  # [rows, T]
    y = api.bsr_spmm(dev, to_dev(x))  # [T, rows] fp32
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    check_close(yh.T, y_or, f"spmm b={b} T={T}")
    assert not yh[:, b:2 * b].any()  # empty block row is written as exact zeros


@pytest.mark.parametrize("b", [64, 128])
@pytest.mark.parametrize("T", [4, 5, 8, 9, 16])
def test_spmm_token_counts_around_the_small_activation_tiles(api, b, T):
    """The decode kernel copies activation tiles of 4, 8 or 16 token rows depending on T and b: every
    boundary, on both sides, with distinct values in every token row."""
    import torch

    w, mask, x = synth.small_case(1500 + b + T, 6 * b, 7 * b, b, 0.45, T, empty_rows=(2,), full_rows=(4,))
    dev, ref = pack_both(api, w, b, mask=mask)
    y = api.bsr_spmm(dev, to_dev(x))
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, orc.spmm(ref, x), f"spmm b={b} T={T}")


@pytest.mark.parametrize("b,T", [(32, 5), (64, 70), (128, 33)])
def test_spmm_feature_major_and_bf16_out(api, b, T):
    import torch

    w, mask, x = synth.small_case(2000 + b, 4 * b, 3 * b, b, 0.4, T)
    dev, ref = pack_both(api, w, b, mask=mask)
    y_or = orc.spmm(ref, x)
    xf = np.ascontiguousarray(x.T)  # [K, T]
    y = api.bsr_spmm(dev, to_dev(xf), layout=api.FEATURE_MAJOR)  # [rows, T]
    torch.cuda.synchronize()
    check_close(y.cpu().numpy(), y_or, "feature-major")
    # bf16 output: the fp32 accumulator rounded to nearest even -> within one bf16 ulp of the rounded oracle
    yb = api.bsr_spmm(dev, to_dev(x), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    got = synth.bf16_bits_to_f32(bits_of(yb)).astype(np.float64).T
    want = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(y_or.astype(np.float32))).astype(np.float64)
    ulp = np.maximum(np.abs(want), 1e-30) * 2.0 ** -7
    assert (np.abs(got - want) <= ulp).all()


@pytest.mark.parametrize("T", [262143, 262145])
def test_spmm_token_counts_on_both_sides_of_the_32_bit_offset_limit(api, T):
    """The streaming kernel addresses the activations of one block column with 32-bit byte offsets: with 8192
    features a token row is 16 KiB, so 262143 tokens are the most one launch takes and 262145 are cut into two
    token ranges.  Token rows repeat with a period (4099) that no power-of-two wrap maps onto itself."""
    import torch

    b, rows, cols, period = 64, 128, 8192, 4099
    rng = np.random.default_rng(1700)
    w = synth.gauss_bf16(rng, (rows, cols), 0.05)
    mask = synth.uniform_mask(rng, rows // b, cols // b, 0.9)
    mask[0, -1] = 1  # the last block column, where the offsets are largest
    base = synth.gauss_bf16(rng, (period, cols), 1.0)
    dev, ref = pack_both(api, w, b, mask=mask)
    idx = torch.arange(T, device="cuda:0") % period
    x = to_dev(base).index_select(0, idx)  # [T, cols] bf16, 4.3 GB
    y = api.bsr_spmm(dev, x)
    torch.cuda.synchronize()
    sample = np.array([0, 1, 255, 256, 4098, 4099, 131071, 131072, 131073, T - 257, T - 256, T - 2, T - 1])
    got = y[torch.from_numpy(sample).to("cuda:0")].cpu().numpy()
    want = orc.spmm(ref, base[sample % period])  # [rows, n]
    check_close(got.T, want, f"spmm T={T}")
    # equal token rows give equal output rows wherever they sit (an output element's sum does not depend on
    # its place in a tile): every row against the one a period earlier, over the whole output
    assert torch.equal(y[period:], y[:-period])
    del x, y
    torch.cuda.empty_cache()


def test_spmm_unaligned_token_major_uses_slow_loads(api):
    import torch

    b, T = 32, 9
    w, mask, x = synth.small_case(31, 3 * b, 4 * b, b, 0.3, T)
    dev, ref = pack_both(api, w, b, mask=mask)
    xpad = np.zeros((T, 4 * b + 3), dtype=np.uint16)
    xpad[:, : 4 * b] = x
    xd = to_dev(xpad)[:, : 4 * b]  # ldx = 131: not a multiple of 8
    y = api.bsr_spmm(dev, xd)
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, orc.spmm(ref, x), "unaligned ldx")


def test_spmm_dense_and_empty_matrix(api):
    import torch

    b, T = 64, 40
    w, _, x = synth.small_case(32, 3 * b, 2 * b, b, 0.0, T)
    dev, ref = pack_both(api, w, b, sparsity=0.0)
    y = api.bsr_spmm(dev, to_dev(x))
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, orc.spmm(ref, x), "dense")
    dev0, ref0 = pack_both(api, w, b, sparsity=1.0)
    y0 = api.bsr_spmm(dev0, to_dev(x), out=torch.full((T, 3 * b), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    assert not y0.cpu().numpy().any()


@pytest.mark.parametrize("b", [32, 64, 128])
@pytest.mark.parametrize("T", [1, 40, 256, 257, 600])
def test_spmm_strided_operands(api, b, T):
    """Activations and outputs that are column slices of wider buffers (ld > width); what lies beside the
    output columns must stay untouched.  Covers the tile boundaries of the kernel choice (256 / 257 tokens)."""
    import torch

    nbr, nbc = 4, 6
    w, mask, x = synth.small_case(5000 + b + T, nbr * b, nbc * b, b, 0.5, T, empty_rows=(2,))
    dev, ref = pack_both(api, w, b, mask=mask)
    y_or = orc.spmm(ref, x)
    xw = torch.full((T, nbc * b + 64), 7.0, dtype=torch.bfloat16, device="cuda:0")
    xw[:, 32:32 + nbc * b] = to_dev(x).view(torch.bfloat16)
    yw = torch.full((T, nbr * b + 40), -3.0, dtype=torch.float32, device="cuda:0")
    y = api.bsr_spmm(dev, xw[:, 32:32 + nbc * b], out=yw[:, 8:8 + nbr * b])
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, y_or, f"strided b={b} T={T}")
    yh = yw.cpu().numpy()
    assert (yh[:, :8] == -3.0).all() and (yh[:, 8 + nbr * b:] == -3.0).all()


@pytest.mark.parametrize("b,nbc,T", [(32, 70, 300), (64, 40, 520), (128, 36, 200), (64, 72, 300),
                                     (32, 70, 9), (32, 70, 40), (64, 72, 1), (64, 72, 7), (64, 72, 16), (64, 72, 100), (128, 66, 3), (128, 66, 20),
                                     # rows long enough for the decode kernel to take the chunk plan as well
                                     (32, 300, 5), (64, 272, 2), (64, 272, 9), (64, 272, 33), (128, 260, 3), (128, 260, 20),
                                     # many tokens: the streaming kernels take the rows in chunks of 64 blocks
                                     (32, 300, 300), (64, 272, 300), (128, 200, 600), (128, 129, 1030)])
def test_spmm_heavy_rows_are_chunked(api, b, nbc, T):
    """Rows with more than 16 stored blocks are cut into chunks that add their partial sums atomically (at
    decode token counts only when a row is more than 256 blocks long; at many tokens in chunks of 64)."""
    import torch

    rng = np.random.default_rng(900 + b)
    nbr = 6
    mask = synth.uniform_mask(rng, nbr, nbc, 0.9)
    mask[0, :] = 1          # a full row: several chunks
    mask[2, : nbc // 2] = 1  # a second heavy row
    mask[4, :] = 0          # an empty row
    w = synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.02)
    x = synth.gauss_bf16(rng, (T, nbc * b), 1.0)
    dev, ref = pack_both(api, w, b, mask=mask)
    check_aux(dev, ref)
    assert dev.max_row_blocks == nbc
    y_or = orc.spmm(ref, x)
    for _ in range(2):  # the output buffer starts poisoned both times
        y = api.bsr_spmm(dev, to_dev(x), out=torch.full((T, nbr * b), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, y_or, f"chunked b={b}")
    assert not y.cpu().numpy()[:, 4 * b:5 * b].any()
    # bf16 output takes the unsplit path and still agrees
    yb = api.bsr_spmm(dev, to_dev(x), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    got = synth.bf16_bits_to_f32(bits_of(yb)).astype(np.float64).T
    assert np.abs(got - y_or).max() <= 2.0 ** -7 * np.abs(y_or).max()


def test_spmm_config1_linear(api):
    import torch

    wl = synth.WORKLOADS["linear_1024x4096_b32_s90"]
    lin = synth.make_linear(wl)
    x = synth.make_x(wl, 64)
    dev, ref = pack_both(api, lin.W, wl.b, mask=lin.mask)
    assert ref.nnz == 409
    y = api.bsr_spmm(dev, to_dev(x))
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, orc.spmm(ref, x), "config 1")
    # the literal "4096 x 64" feature-major reading of the same configuration
    yf = api.bsr_spmm(dev, to_dev(np.ascontiguousarray(x.T)), layout=api.FEATURE_MAJOR)
    torch.cuda.synchronize()
    check_close(yf.cpu().numpy(), orc.spmm(ref, x), "config 1 feature-major")


# ------------------------------------------------------------------ fused MLP
def _mlp_case(api, seed, E, I, b, sparsity, T, act="silu", layout="token_major", poison=True):
    import torch

    rng = np.random.default_rng(seed)
    g, u, d = (synth.gauss_bf16(rng, s, 0.05) for s in ((I, E), (I, E), (E, I)))
    mg, mu = (synth.uniform_mask(rng, I // b, E // b, sparsity) for _ in range(2))
    md = synth.uniform_mask(rng, E // b, I // b, sparsity)
    if I // b > 2:
        mg[1, :] = 0  # empty gate block row -> zero H rows
        md[:, 2] = 0  # H rows nobody consumes
    if E // b > 1:
        md[1, :] = 0  # empty down block row -> zero Y rows
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    dg, rg = pack_both(api, g, b, mask=mg)
    du, ru = pack_both(api, u, b, mask=mu)
    dd, rd = pack_both(api, d, b, mask=md)
    y_or = orc.mlp(rg, ru, rd, x, activation=act)
    if layout == "token_major":
        out = torch.full((T, E), float("nan"), device="cuda:0") if poison else None
        y = api.sparse_mlp(dg, du, dd, to_dev(x), act=act, out=out).cpu().numpy().T
    else:
        y = api.sparse_mlp(dg, du, dd, to_dev(np.ascontiguousarray(x.T)), act=act, layout=api.FEATURE_MAJOR).cpu().numpy()
    torch.cuda.synchronize()
    check_close(y, y_or, f"mlp E={E} I={I} b={b} T={T} {act} {layout}")
    if E // b > 1:
        assert not y[b:2 * b].any()


@pytest.mark.parametrize("b", [16, 32, 64, 128])
@pytest.mark.parametrize("T", [1, 5, 16, 17, 32, 33, 130, 300])
def test_mlp_small(api, b, T):
    _mlp_case(api, 3000 + b + T, 4 * b, 6 * b, b, 0.5, T)


@pytest.mark.parametrize("b,T", [(64, 1), (64, 8), (64, 16), (64, 29), (64, 50), (64, 64), (64, 65),
                                 (128, 1), (128, 4), (128, 9), (128, 16), (128, 21), (128, 32)])
def test_mlp_one_launch_with_many_blocks_per_wave(api, b, T):
    """Rows of 14-28 stored blocks in both products of the single-launch form: every wave walks several blocks,
    so its ring (b = 64) or its two register sets (b = 128) go round more than once."""
    _mlp_case(api, 3050 + b + T, 20 * b, 24 * b, b, 0.3, T)


@pytest.mark.parametrize("act", ["silu", "gelu", "relu"])
def test_mlp_activations_and_layouts(api, act):
    _mlp_case(api, 3100, 256, 512, 64, 0.6, 37, act=act)
    _mlp_case(api, 3101, 256, 512, 64, 0.6, 37, act=act, layout="feature_major")


def test_mlp_dense_and_all_pruned(api):
    _mlp_case(api, 3200, 128, 256, 64, 0.0, 20)
    _mlp_case(api, 3201, 128, 256, 64, 1.0, 20)


def test_joint_row_order(api):
    import torch

    rng = np.random.default_rng(77)
    b, nbr, nbc = 32, 40, 12
    g, u = (synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.05) for _ in range(2))
    mg, mu = (synth.uniform_mask(rng, nbr, nbc, 0.6) for _ in range(2))
    mg[3, :] = 0
    mu[3, :] = 0
    dg, rg = pack_both(api, g, b, mask=mg)
    du, ru = pack_both(api, u, b, mask=mu)
    gj = api.with_joint_row_order(dg, du)
    torch.cuda.synchronize()
    cnt = np.diff(rg.row_ptr) + np.diff(ru.row_ptr)
    assert np.array_equal(gj.row_order.cpu().numpy(), np.argsort(-cnt, kind="stable"))
    # results do not depend on the schedule
    x = synth.gauss_bf16(rng, (300, nbc * b), 1.0)
    h1 = api.bsr_gated_spmm(dg, du, to_dev(x))
    h2 = api.bsr_gated_spmm(gj, du, to_dev(x))
    torch.cuda.synchronize()
    assert torch.equal(h1.view(torch.int16), h2.view(torch.int16))


@pytest.mark.parametrize("b,T", [(64, 1), (64, 16), (64, 29), (64, 60), (128, 3), (128, 16), (128, 27)])
def test_mlp_one_launch_reuses_workspace(api, b, T):
    """The single-launch form hands H over inside the kernel through the caller's workspace: calls that
    reuse one workspace with different activations must each see their own H (no stale slots or lines)."""
    import torch

    rng = np.random.default_rng(7000 + b + T)
    E, I = 4 * b, 6 * b
    g, u, d = (synth.gauss_bf16(rng, s, 0.05) for s in ((I, E), (I, E), (E, I)))
    mg, mu, md = (synth.uniform_mask(rng, r // b, c // b, 0.5) for r, c in ((I, E), (I, E), (E, I)))
    dg, rg = pack_both(api, g, b, mask=mg)
    du, ru = pack_both(api, u, b, mask=mu)
    dd, rd = pack_both(api, d, b, mask=md)
    ws = torch.full((max(api.mlp_workspace_bytes(dg, du, dd, T), 256),), 0xA5, dtype=torch.uint8, device="cuda:0")
    for rep in range(4):
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        y = api.sparse_mlp(dg, du, dd, to_dev(x), ws=ws, out=torch.full((T, E), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.mlp(rg, ru, rd, x), f"one launch b={b} T={T} call {rep}")


@pytest.mark.parametrize("b,T", [(128, 40), (128, 100), (64, 200)])
def test_mlp_with_a_gated_row_long_enough_to_stay_in_the_decode_kernel(api, b, T):
    """Beyond 64 tokens the gated product normally streams; a block row that is full in both matrices keeps it
    in the decode kernel, several token groups per unit (the streaming kernel would walk that row in one
    workgroup)."""
    import torch

    E, I = (48 * b, 4 * b) if b == 128 else (180 * b, 4 * b)
    rng = np.random.default_rng(3400 + b + T)
    g, u = (synth.gauss_bf16(rng, (I, E), 0.02) for _ in range(2))
    d = synth.gauss_bf16(rng, (E, I), 0.05)
    mg, mu = (synth.uniform_mask(rng, I // b, E // b, 0.9) for _ in range(2))
    mg[2, :] = 1
    mu[2, :] = 1  # the full joint row
    md = synth.uniform_mask(rng, E // b, I // b, 0.25)
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    (dg, rg), (du, ru), (dd, rd) = (pack_both(api, w, b, mask=m) for w, m in ((g, mg), (u, mu), (d, md)))
    assert dg.max_row_blocks + du.max_row_blocks == 2 * (E // b)
    y = api.sparse_mlp(dg, du, dd, to_dev(x))
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, orc.mlp(rg, ru, rd, x), f"long gated row b={b} T={T}")


@pytest.mark.parametrize("T", [3, 40, 300])
def test_mlp_from_two_host_threads_on_two_streams(api, T):
    """Calls on distinct streams from distinct host threads, each with its own output and workspace, may
    overlap on the GPU (the single-launch form at T = 3 included: its slots live in the call's workspace)."""
    import threading

    import torch

    b, E, I = 64, 256, 512
    cases = []
    for seed in (3300, 3301):
        rng = np.random.default_rng(seed + T)
        g, u, d = (synth.gauss_bf16(rng, s, 0.05) for s in ((I, E), (I, E), (E, I)))
        mg, mu = (synth.uniform_mask(rng, I // b, E // b, 0.5) for _ in range(2))
        md = synth.uniform_mask(rng, E // b, I // b, 0.5)
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        packs = [pack_both(api, w, b, mask=m) for w, m in ((g, mg), (u, mu), (d, md))]
        (dg, rg), (du, ru), (dd, rd) = packs
        cases.append(dict(dev=(dg, du, dd), x=to_dev(x), want=orc.mlp(rg, ru, rd, x),
                          ws=torch.empty(max(api.mlp_workspace_bytes(dg, du, dd, T), 256), dtype=torch.uint8, device="cuda:0"),
                          out=torch.empty((T, E), dtype=torch.float32, device="cuda:0"), got=[], err=None))
    torch.cuda.synchronize()

    def worker(c):
        try:
            st = torch.cuda.Stream()  # default priority
            with torch.cuda.stream(st):
                for _ in range(20):
                    c["out"].fill_(float("nan"))
                    api.sparse_mlp(*c["dev"], c["x"], out=c["out"], ws=c["ws"])
                    c["got"].append(c["out"].clone())
            st.synchronize()
        except Exception as e:  # surfaced in the main thread
            c["err"] = e

    threads = [threading.Thread(target=worker, args=(c,)) for c in cases]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for k, c in enumerate(cases):
        assert c["err"] is None, c["err"]
        assert len(c["got"]) == 20
        for y in c["got"]:
            check_close(y.cpu().numpy().T, c["want"], f"thread {k} T={T}")


@pytest.mark.parametrize("T", [8, 300])
def test_mlp_under_graph_capture(api, T):
    """The call records into a graph (no allocation, no synchronisation, no per-launch host state that a
    replay would repeat) and every replay, with new activations, matches the oracle."""
    import torch

    rng = np.random.default_rng(7100 + T)
    b, E, I = 64, 256, 384
    g, u, d = (synth.gauss_bf16(rng, s, 0.05) for s in ((I, E), (I, E), (E, I)))
    mg, mu, md = (synth.uniform_mask(rng, r // b, c // b, 0.5) for r, c in ((I, E), (I, E), (E, I)))
    dg, rg = pack_both(api, g, b, mask=mg)
    du, ru = pack_both(api, u, b, mask=mu)
    dd, rd = pack_both(api, d, b, mask=md)
    ws = torch.empty(max(api.mlp_workspace_bytes(dg, du, dd, T), 256), dtype=torch.uint8, device="cuda:0")
    xs = to_dev(synth.gauss_bf16(rng, (T, E), 1.0))
    y = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        api.sparse_mlp(dg, du, dd, xs, out=y, ws=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.sparse_mlp(dg, du, dd, xs, out=y, ws=ws)
    for rep in range(3):
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        xs.copy_(to_dev(x))
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.mlp(rg, ru, rd, x), f"graph replay {rep} T={T}")


def test_mlp_repeatable(api):
    import torch

    wl = synth.WORKLOADS["llama1b_b64_s90"]
    rng = np.random.default_rng(5)
    E, I, b, T = 512, 1024, 64, 48
    g, u, d = (synth.gauss_bf16(rng, s, 0.03) for s in ((I, E), (I, E), (E, I)))
    x = to_dev(synth.gauss_bf16(rng, (T, E), 1.0))
    dg = api.bsr_pack(to_dev(g), b, sparsity=0.8)
    du = api.bsr_pack(to_dev(u), b, sparsity=0.8)
    dd = api.bsr_pack(to_dev(d), b, sparsity=0.8)
    y1 = api.sparse_mlp(dg, du, dd, x).clone()
    for _ in range(3):
        y2 = api.sparse_mlp(dg, du, dd, x)
        torch.cuda.synchronize()
        check_close(y2.cpu().numpy(), y1.cpu().numpy().astype(np.float64), "repeat")
    assert wl.b == 64


# ------------------------------------------------------------------ two-matrix MLP  Y = W2 act(W1 X)
def _mlp2_case(api, seed, E, I, b, sparsity, T, act="gelu", layout="token_major", out_dtype="f32", scale=0.05):
    import torch

    rng = np.random.default_rng(seed)
    w1, w2 = (synth.gauss_bf16(rng, s, scale) for s in ((I, E), (E, I)))
    m1 = synth.uniform_mask(rng, I // b, E // b, sparsity)
    m2 = synth.uniform_mask(rng, E // b, I // b, sparsity)
    if I // b > 2:
        m1[1, :] = 0  # empty W1 block row -> zero H rows (act(0) = 0)
        m2[:, 2] = 0  # H rows nobody consumes
    if E // b > 1:
        m2[1, :] = 0  # empty W2 block row -> zero Y rows
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    d1, r1 = pack_both(api, w1, b, mask=m1)
    d2, r2 = pack_both(api, w2, b, mask=m2)
    y_or = orc.mlp2(r1, r2, x, activation=act)
    tdt = torch.float32 if out_dtype == "f32" else torch.bfloat16
    if layout == "token_major":
        out = torch.full((T, E), float("nan"), device="cuda:0", dtype=tdt)
        y = api.sparse_mlp2(d1, d2, to_dev(x), act=act, out=out).float().cpu().numpy().T
    else:
        y = api.sparse_mlp2(d1, d2, to_dev(np.ascontiguousarray(x.T)), act=act, layout=api.FEATURE_MAJOR,
                            out_dtype=tdt).float().cpu().numpy()
    torch.cuda.synchronize()
    what = f"mlp2 E={E} I={I} b={b} T={T} {act} {layout} {out_dtype}"
    if out_dtype == "f32":
        check_close(y, y_or, what)
    else:
        # one more rounding of Y to bf16: half an ulp (2^-9 relative) per element
        assert np.isfinite(y).all(), what
        assert np.all(np.abs(y - y_or) <= 2.0 ** -8 * np.abs(y_or) + 1e-2 * np.sqrt((y_or ** 2).mean())), what
        assert np.linalg.norm(y - y_or) <= 4e-3 * np.linalg.norm(y_or), what
    if E // b > 1:
        assert not y[b:2 * b].any()


@pytest.mark.parametrize("b", [16, 32, 64, 128])
@pytest.mark.parametrize("T", [1, 5, 16, 17, 32, 33, 130, 300])
def test_mlp2_small(api, b, T):
    _mlp2_case(api, 8000 + b + T, 4 * b, 6 * b, b, 0.5, T)


@pytest.mark.parametrize("act", ["silu", "gelu", "relu"])
@pytest.mark.parametrize("T", [7, 37, 280])
def test_mlp2_activations_and_layouts(api, act, T):
    # weights scaled so that pre-activations spread over [-3, 3]: both tails of each function are exercised
    _mlp2_case(api, 8100 + T, 256, 512, 64, 0.6, T, act=act, scale=0.12)
    _mlp2_case(api, 8101 + T, 256, 512, 64, 0.6, T, act=act, layout="feature_major", scale=0.12)
    _mlp2_case(api, 8102 + T, 256, 512, 32, 0.6, T, act=act, out_dtype="bf16", scale=0.12)


def test_mlp2_dense_and_all_pruned(api):
    _mlp2_case(api, 8200, 128, 256, 64, 0.0, 20)
    _mlp2_case(api, 8201, 128, 256, 64, 1.0, 20)
    _mlp2_case(api, 8202, 256, 512, 128, 0.0, 300)


@pytest.mark.parametrize("b,T", [(64, 1), (64, 16), (64, 29), (128, 3), (128, 16)])
def test_mlp2_one_launch_reuses_workspace(api, b, T):
    """Single-launch form of the two-matrix MLP: repeated calls on one workspace, and interleaved with the
    three-matrix form on the same workspace, each see their own H."""
    import torch

    rng = np.random.default_rng(8300 + b + T)
    E, I = 4 * b, 6 * b
    w1, wu, w2 = (synth.gauss_bf16(rng, s, 0.08) for s in ((I, E), (I, E), (E, I)))
    m1, mu, m2 = (synth.uniform_mask(rng, r // b, c // b, 0.5) for r, c in ((I, E), (I, E), (E, I)))
    d1, r1 = pack_both(api, w1, b, mask=m1)
    du, ru = pack_both(api, wu, b, mask=mu)
    d2, r2 = pack_both(api, w2, b, mask=m2)
    assert api.mlp2_workspace_bytes(d1, d2, T) == api.mlp_workspace_bytes(d1, du, d2, T)
    ws = torch.full((max(api.mlp2_workspace_bytes(d1, d2, T), 256),), 0x5A, dtype=torch.uint8, device="cuda:0")
    for rep in range(4):
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        y = api.sparse_mlp2(d1, d2, to_dev(x), ws=ws, out=torch.full((T, E), float("nan"), device="cuda:0"))
        y3 = api.sparse_mlp(d1, du, d2, to_dev(x), ws=ws, out=torch.full((T, E), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.mlp2(r1, r2, x), f"mlp2 one launch b={b} T={T} call {rep}")
        check_close(y3.cpu().numpy().T, orc.mlp(r1, ru, r2, x), f"mlp after mlp2 b={b} T={T} call {rep}")


@pytest.mark.parametrize("T", [8, 300])
def test_mlp2_under_graph_capture(api, T):
    import torch

    rng = np.random.default_rng(8400 + T)
    b, E, I = 64, 256, 384
    w1, w2 = (synth.gauss_bf16(rng, s, 0.08) for s in ((I, E), (E, I)))
    m1, m2 = (synth.uniform_mask(rng, r // b, c // b, 0.5) for r, c in ((I, E), (E, I)))
    d1, r1 = pack_both(api, w1, b, mask=m1)
    d2, r2 = pack_both(api, w2, b, mask=m2)
    ws = torch.empty(max(api.mlp2_workspace_bytes(d1, d2, T), 256), dtype=torch.uint8, device="cuda:0")
    xs = to_dev(synth.gauss_bf16(rng, (T, E), 1.0))
    y = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        api.sparse_mlp2(d1, d2, xs, out=y, ws=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.sparse_mlp2(d1, d2, xs, out=y, ws=ws)
    for rep in range(3):
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        xs.copy_(to_dev(x))
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.mlp2(r1, r2, x), f"mlp2 graph replay {rep} T={T}")


def test_mlp2_topk_packed_gpt2_shape(api):
    """E = 768, I = 3072 (a GPT-2-small MLP block, one of the models of Sec. 4), packed on the device by block norm at 90 %."""
    import torch

    rng = np.random.default_rng(8500)
    E, I, b = 768, 3072, 64
    w1, w2 = (synth.gauss_bf16(rng, s, 0.04) for s in ((I, E), (E, I)))
    d1, r1 = pack_both(api, w1, b, sparsity=0.9)
    d2, r2 = pack_both(api, w2, b, sparsity=0.9)
    for T in (4, 100, 513):
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        y = api.sparse_mlp2(d1, d2, to_dev(x))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.mlp2(r1, r2, x), f"mlp2 gpt2 shape T={T}")


@pytest.mark.parametrize("T", [1, 20, 32, 40, 300, 700])
def test_mlp_decode_with_a_very_long_down_row(api, T):
    """A row of W_down long enough for the chunk plans: its output rows are cleared on the side by the gate/up
    launch (decode kernel: extra workgroups; streaming kernel, many tokens: every workgroup before its own
    work) or by a launch of their own (in between), into a poisoned Y."""
    import torch

    rng = np.random.default_rng(8600 + T)
    b, E, nbi = 64, 256, 272
    I = nbi * b
    g, u, d = (synth.gauss_bf16(rng, s, 0.02) for s in ((I, E), (I, E), (E, I)))
    mg, mu = (synth.uniform_mask(rng, nbi, E // b, 0.5) for _ in range(2))
    md = synth.uniform_mask(rng, E // b, nbi, 0.9)
    md[0, :] = 1   # 272 blocks: cut into 17 chunks
    md[2, :] = 0   # an empty row beside it
    dg, rg = pack_both(api, g, b, mask=mg)
    du, ru = pack_both(api, u, b, mask=mu)
    dd, rd = pack_both(api, d, b, mask=md)
    assert dd.max_row_blocks == nbi
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    want = orc.mlp(rg, ru, rd, x)
    for _ in range(2):
        y = api.sparse_mlp(dg, du, dd, to_dev(x), out=torch.full((T, E), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, want, f"mlp long down row T={T}")
    assert not y.cpu().numpy()[:, 2 * b:3 * b].any()


@pytest.mark.parametrize("b,T", [(32, 100), (64, 65), (64, 200), (64, 700), (128, 129), (128, 300)])
def test_mlp_with_long_gate_and_up_rows(api, b, T):
    """Beyond the decode kernels' token counts the cut rows of a skewed gated product are summed chunk by chunk
    into scratch and finished by a launch of their own; the workspace query asks for that scratch exactly there.
    No atomics: two calls give the same bits."""
    import torch

    rng = np.random.default_rng(8800 + b + T)
    E, I, (g, u, d), (mg, mu, md) = long_row_case(rng, b)
    dg, rg = pack_both(api, g, b, mask=mg)
    du, ru = pack_both(api, u, b, mask=mu)
    dd, rd = pack_both(api, d, b, mask=md)
    dgj = api.with_joint_row_order(dg, du)
    a256 = lambda n: -(-n // 256) * 256
    for gate in (dg, dgj):
        small = api.mlp_workspace_bytes(gate, du, dd, 64)   # decode range: no scratch
        want_ws = small - a256(64 * I * 2) + a256(T * I * 2) + long_scratch_bytes((dg, du), b, T)
        assert api.mlp_workspace_bytes(gate, du, dd, T) == want_ws and want_ws > small
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    want = orc.mlp(rg, ru, rd, x)
    seen = []
    for gate in (dg, dgj, dgj):
        y = api.sparse_mlp(gate, du, dd, to_dev(x), out=torch.full((T, E), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, want, f"mlp long gate/up rows b={b} T={T}")
        seen.append(y)
    assert torch.equal(seen[1], seen[2])
    # without the scratch (a workspace sized for the plain path) the same call takes the plain path
    ws = torch.empty(a256(T * I * 2) + small - a256(64 * I * 2), dtype=torch.uint8, device="cuda:0")
    y = api.sparse_mlp(dgj, du, dd, to_dev(x), out=torch.full((T, E), float("nan"), device="cuda:0"), ws=ws)
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, want, f"mlp long gate/up rows, plain workspace b={b} T={T}")


def test_mlp_with_long_rows_graph_replay(api):
    """The launches of the long-row path (product, finish) recorded once and replayed on new inputs."""
    import torch

    rng = np.random.default_rng(8900)
    b, T = 64, 150
    E, I, (g, u, d), (mg, mu, md) = long_row_case(rng, b)
    dg, rg = pack_both(api, g, b, mask=mg)
    du, ru = pack_both(api, u, b, mask=mu)
    dd, rd = pack_both(api, d, b, mask=md)
    dg = api.with_joint_row_order(dg, du)
    xs = torch.zeros((T, E), dtype=torch.bfloat16, device="cuda:0")
    y = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(api.mlp_workspace_bytes(dg, du, dd, T), dtype=torch.uint8, device="cuda:0")
    api.sparse_mlp(dg, du, dd, xs, out=y, ws=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.sparse_mlp(dg, du, dd, xs, out=y, ws=ws)
    for rep in range(3):
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        xs.copy_(to_dev(x))
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.mlp(rg, ru, rd, x), f"mlp long rows graph replay {rep}")


@pytest.mark.parametrize("T", [3, 20])
def test_mlp2_decode_with_a_very_long_second_row(api, T):
    """Two-matrix form of the case above: the first product (with its activation) carries the side workgroups
    that clear the rows the chunked second product accumulates into."""
    import torch

    rng = np.random.default_rng(8700 + T)
    b, E, nbi = 64, 256, 272
    I = nbi * b
    w1, w2 = (synth.gauss_bf16(rng, s, 0.03) for s in ((I, E), (E, I)))
    m1 = synth.uniform_mask(rng, nbi, E // b, 0.5)
    m2 = synth.uniform_mask(rng, E // b, nbi, 0.9)
    m2[1, :] = 1
    m2[3, :] = 0
    d1, r1 = pack_both(api, w1, b, mask=m1)
    d2, r2 = pack_both(api, w2, b, mask=m2)
    assert d2.max_row_blocks == nbi
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    want = orc.mlp2(r1, r2, x, activation="gelu")
    for _ in range(2):
        y = api.sparse_mlp2(d1, d2, to_dev(x), act="gelu", out=torch.full((T, E), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, want, f"mlp2 long second row T={T}")
    assert not y.cpu().numpy()[:, 3 * b:4 * b].any()
