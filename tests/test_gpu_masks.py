"""GPU parity of the blocked prune-and-grow mask update (Sec. 3.2) and of packing its result: byte-exact masks,
bit-exact packed arrays, regrown blocks stored as zeros."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2507_03117_amd import synth
from tests.helpers import bits_of, check_close, mask_dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available()
    from paper_2507_03117_amd import api as _api

    _api.lib()
    return _api


def _gaps_ok(A, b, s):
    """The selection must not hang on the rounding of a score sum (device tree order vs oracle row order)."""
    _, gap = orc.topk_mask(orc.block_scores(A, b), s)
    return gap > 1e-9


@pytest.mark.parametrize("b,rows,cols,s", [(16, 256, 512, 0.7), (32, 1024, 2048, 0.9), (64, 2048, 1024, 0.5),
                                           (128, 1024, 1536, 0.8), (64, 512, 512, 0.0), (64, 512, 512, 1.0)])
def test_generate_masks_matches_oracle(api, b, rows, cols, s):
    import torch

    rng = np.random.default_rng(9700 + b + rows)
    W, G = synth.gauss_bf16(rng, (rows, cols), 0.02), synth.gauss_bf16(rng, (rows, cols), 1e-3)
    assert _gaps_ok(W, b, s) and _gaps_ok(G, b, s), "selection hangs on rounding: reseed"
    m = api.generate_masks(to_dev(W), to_dev(G), b, s)
    torch.cuda.synchronize()
    want = orc.generate_masks(W, G, b, s)
    assert np.array_equal(m.cpu().numpy(), want)
    if 0.0 < s < 1.0:
        assert (want == 2).any() and (want == 1).any() and (want == 0).any()


def test_generate_masks_and_pooled_selection_beyond_one_workgroup(api):
    """26624 blocks: more than one workgroup selects from (8192), so the mask update runs its two selections side
    by side over global memory and merges them in a launch of its own, and the pooled selection takes the same
    select."""
    import torch

    rng = np.random.default_rng(9750)
    b, rows, cols, s = 16, 2048, 3328, 0.9
    W, G = synth.gauss_bf16(rng, (rows, cols), 0.02), synth.gauss_bf16(rng, (rows, cols), 1e-3)
    assert _gaps_ok(W, b, s) and _gaps_ok(G, b, s), "selection hangs on rounding: reseed"
    m = api.generate_masks(to_dev(W), to_dev(G), b, s)
    torch.cuda.synchronize()
    want = orc.generate_masks(W, G, b, s)
    assert np.array_equal(m.cpu().numpy(), want)
    assert (want == 2).any() and (want == 1).any() and (want == 0).any()
    S = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    want, gap = orc.pooled_topk_mask(S, b, s)
    assert gap > 1e-9, "selection hangs on rounding: reseed"
    m = api.pooled_topk_mask(torch.from_numpy(S).to("cuda:0"), b, s)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy(), want)


def test_generate_masks_ties_and_equal_gradient(api):
    import torch

    rng = np.random.default_rng(9800)
    b, nbr, nbc = 32, 8, 8
    # duplicated blocks give exactly equal scores on both sides: the index tie-break decides
    blk = synth.gauss_bf16(rng, (4, b, b), 1.0)
    pick = rng.integers(0, 4, size=(nbr, nbc))
    W = blk[pick].transpose(0, 2, 1, 3).reshape(nbr * b, nbc * b)
    G = blk[(pick + 1) % 4].transpose(0, 2, 1, 3).reshape(nbr * b, nbc * b)
    for s in (0.3, 0.5, 0.77):
        m = api.generate_masks(to_dev(W), to_dev(G), b, s)
        torch.cuda.synchronize()
        assert np.array_equal(m.cpu().numpy(), orc.generate_masks(W, G, b, s)), s
    m = api.generate_masks(to_dev(W), to_dev(W), b, 0.5)
    torch.cuda.synchronize()
    assert not (m.cpu().numpy() == 2).any()


def test_pack_with_regrown_blocks_and_one_training_round(api):
    """generate_masks -> pack -> product: the packed W_new has the union structure, zeros in the regrown blocks,
    and multiplies like the weight pruned to S(W) alone (regrown blocks do not change the current transform)."""
    import torch

    rng = np.random.default_rng(9900)
    b, rows, cols, T = 64, 1024, 768, 70
    s = api.sparsity_schedule(4000, 9000, 1000, 0.1, 0.8)
    assert s == orc.sparsity_schedule(4000, 9000, 1000, 0.1, 0.8)
    W, G = synth.gauss_bf16(rng, (rows, cols), 0.02), synth.gauss_bf16(rng, (rows, cols), 1e-3)
    assert _gaps_ok(W, b, s) and _gaps_ok(G, b, s)
    m = api.generate_masks(to_dev(W), to_dev(G), b, s)
    dev = api.bsr_pack(to_dev(W), b, mask=m)
    torch.cuda.synchronize()
    want_mask = orc.generate_masks(W, G, b, s)
    ref = orc.pack(W, b, want_mask)
    assert dev.nnz == ref.nnz == int((want_mask != 0).sum())
    assert np.array_equal(dev.row_ptr.cpu().numpy(), ref.row_ptr)
    assert np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)
    assert np.array_equal(bits_of(dev.vals)[: ref.nnz * b * b].reshape(ref.nnz, b, b), ref.vals)
    assert np.array_equal(dev.row_order.cpu().numpy(), ref.row_order)
    rr = np.repeat(np.arange(rows // b), np.diff(ref.row_ptr))
    grown = want_mask[rr, ref.col_idx] == 2
    assert grown.any() and not ref.vals[grown].any() and ref.vals[~grown].any()
    x = synth.gauss_bf16(rng, (T, cols), 1.0)
    y = api.bsr_spmm(dev, to_dev(x))
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, orc.spmm(orc.pack(W, b, (want_mask == 1).astype(np.uint8)), x), "product after regrowth")
    # the regrown blocks do receive a gradient (that is how they come alive in the following iterations)
    dY = synth.gauss_bf16(rng, (T, rows), 1.0)
    dv = api.bsr_sddmm(dev, to_dev(dY), to_dev(x))
    torch.cuda.synchronize()
    dv_or = orc.sddmm(ref, dY, x)
    check_close(dv.cpu().numpy().reshape(1, -1), dv_or.reshape(1, -1), "gradient of W_new")
    assert np.abs(dv.cpu().numpy()[grown]).max() > 0


@pytest.mark.parametrize("b,rows,cols,s", [(16, 256, 512, 0.7), (32, 1024, 2048, 0.9), (64, 2048, 1024, 0.5),
                                           (128, 1024, 1536, 0.8), (64, 512, 512, 0.0), (64, 512, 512, 1.0)])
def test_pooled_topk_mask_matches_oracle(api, b, rows, cols, s):
    """Sec. 3.3: block scores by average pooling of a sensitivity matrix (either sign), then the top blocks."""
    import torch

    rng = np.random.default_rng(9950 + b + rows)
    S = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)  # block means of either sign
    want, gap = orc.pooled_topk_mask(S, b, s)
    assert gap > 1e-9, "selection hangs on rounding: reseed"
    m = api.pooled_topk_mask(torch.from_numpy(S).to("cuda:0"), b, s)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy(), want)
    if 0.0 < s < 1.0:
        sc = orc.pooled_scores(S, b)
        assert (sc[want == 1] < 0).any() or (sc[want == 0] < 0).any()  # negative scores took part in the ranking


def test_pooled_topk_mask_ties_and_pack(api):
    import torch

    b, nbr, nbc = 32, 6, 10
    rng = np.random.default_rng(9960)
    # every block constant, values drawn from three levels (one negative, and a zero level): many exact ties
    levels = np.array([-0.5, 0.0, 0.25], dtype=np.float32)
    S = np.kron(levels[rng.integers(0, 3, size=(nbr, nbc))], np.ones((b, b), dtype=np.float32)).astype(np.float32)
    for s in (0.2, 0.5, 0.8):
        want, _ = orc.pooled_topk_mask(S, b, s)
        m = api.pooled_topk_mask(torch.from_numpy(S).to("cuda:0"), b, s)
        torch.cuda.synchronize()
        assert np.array_equal(m.cpu().numpy(), want), s
    # the mask drives the packer like any other
    W = synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.05)
    dev = api.bsr_pack(to_dev(W), b, mask=m)
    ref = orc.pack(W, b, want)
    torch.cuda.synchronize()
    assert dev.nnz == ref.nnz and np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)


@pytest.mark.parametrize("b", [16, 32, 64, 128])
def test_unpack_is_the_inverse_of_pack(api, b):
    """prune_weights(): the dense pruned weight equals W (.) mask bit for bit, regrown blocks are zero, and a
    strided, poisoned destination is fully overwritten."""
    import torch

    rng = np.random.default_rng(9970 + b)
    rows, cols = 6 * b, 5 * b
    W = synth.gauss_bf16(rng, (rows, cols), 0.05)
    mask = synth.uniform_mask(rng, rows // b, cols // b, 0.6)
    mask[1, :] = 0
    mask[2, 3] = 2  # a regrown block
    dev = api.bsr_pack(to_dev(W), b, mask=mask_dev(mask))
    ref = orc.pack(W, b, mask)
    big = torch.full((rows, cols + 8), -1, dtype=torch.int16, device="cuda:0")
    out = api.bsr_unpack(dev, out=big.view(torch.bfloat16)[:, :cols])
    torch.cuda.synchronize()
    got = bits_of(out)
    assert np.array_equal(got, orc.unpack(ref))
    keep = np.kron((mask == 1).astype(np.uint16), np.ones((b, b), dtype=np.uint16))
    assert np.array_equal(got, W * keep)
    assert np.all(big.cpu().numpy()[:, cols:] == -1)  # nothing written past the row width
