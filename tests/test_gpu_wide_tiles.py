"""GPU parity of the prefill kernel's 256-token x 128-row tiles (eight-wave workgroups, b = 128) and of its two
schedules: token tiles pinned to an XCD, and block rows pinned to an XCD with the rows dealt to groups of
workgroups by accumulated work.  The shapes are the smallest that reach those code paths: the wide tile needs
twice as many (block row, 256-token tile) pairs as the chip has compute units, the row-pinned schedule an
activation slab of more than 6 MiB per XCD (12800 features here), a token-tile count that divides 32, and - for
the work-balanced dealing - at most 8 groups per XCD and 64 rows per XCD."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2507_03117_amd import synth
from tests.helpers import check_close, mask_dev, stratified_tokens, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available()
    from paper_2507_03117_amd import api as _api

    _api.lib()
    return _api


def _sparse_weight(rng, mask, b, std=0.02):
    """Gaussian values on the kept blocks only (mask-mode packing never reads a dropped block)."""
    nbr, nbc = mask.shape
    w = np.zeros((nbr * b, nbc * b), dtype=np.uint16)
    rr, cc = np.nonzero(mask)
    w.reshape(nbr, b, nbc, b)[rr, :, cc, :] = synth.gauss_bf16(rng, (rr.size, b, b), std)
    return w


def _skewed_mask(rng, nbr, nbc, sparsity):
    mask = synth.uniform_mask(rng, nbr, nbc, sparsity)
    mask[3, :] = 1                      # a full row
    mask[nbr // 2, : nbc // 3] = 1      # a heavy row
    mask[5, :] = 0                      # empty rows
    mask[nbr - 1, :] = 0
    return mask


def _pack(api, w, b, mask):
    dev = api.bsr_pack(to_dev(w), b, mask=mask_dev(mask))
    ref = orc.pack(w, b, mask)
    assert dev.nnz == ref.nnz and np.array_equal(dev.row_ptr.cpu().numpy(), ref.row_ptr)
    assert np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)
    assert np.array_equal(dev.row_order.cpu().numpy()[: ref.row_order.size], ref.row_order)
    return dev, ref


# (block rows, block columns, tokens): what the case reaches
SPMM_CASES = [
    (110, 6, 1290),   # wide tile, token tiles pinned, ragged last tile (6 tiles: 32 % 6 != 0)
    (130, 100, 1024),  # row-pinned: 4 tiles, 8 groups per XCD, 17 rows per XCD, every other octet mirrored
    (130, 100, 1000),  # the same with a ragged last tile
    (75, 100, 2048),  # row-pinned: 8 tiles, 4 groups; 75 rows: the last octet is partial
    (40, 100, 4096),  # row-pinned: 16 tiles, 2 groups
    (260, 100, 512),  # row-pinned: 2 tiles, 16 groups per XCD: rows dealt round-robin
    (72, 100, 2304),  # 9 tiles do not divide 32: falls back to pinned token tiles
]


@pytest.mark.parametrize("nbr,nbc,T", SPMM_CASES)
def test_spmm_wide_tiles(api, nbr, nbc, T):
    import torch

    b = 128
    rng = np.random.default_rng(4000 + nbr + nbc + T)
    mask = _skewed_mask(rng, nbr, nbc, 0.93 if nbc > 8 else 0.5)
    w = _sparse_weight(rng, mask, b)
    x = synth.gauss_bf16(rng, (T, nbc * b), 1.0)
    dev, ref = _pack(api, w, b, mask)
    sel = stratified_tokens(T, 24)
    y_or = orc.spmm(ref, np.ascontiguousarray(x[sel]))
    xd = to_dev(x)
    # fp32 output: rows long enough are cut into chunks that add into cleared rows; poisoned output
    y = api.bsr_spmm(dev, xd, out=torch.full((T, nbr * b), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert np.isfinite(yh).all()
    fro, mx = check_close(yh[sel].T, y_or, f"wide spmm f32 {nbr}x{nbc} T={T}")
    assert not yh[:, 5 * b:6 * b].any() and not yh[:, (nbr - 1) * b:].any()
    # bf16 output: never chunked (whole rows in one workgroup)
    yb = api.bsr_spmm(dev, xd, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    got = yb.float().cpu().numpy()[sel].astype(np.float64).T
    assert np.abs(got - y_or).max() <= 2.0 ** -7 * np.abs(y_or).max()
    print(f"wide spmm {nbr}x{nbc} T={T}: rel_fro={fro:.2e} max_abs/rms={mx:.2e} on {sel.size} tokens")


@pytest.mark.parametrize("nbi,nbe,T", [(130, 100, 1024), (75, 100, 2048), (110, 6, 1290), (260, 100, 512)])
def test_mlp_wide_tiles(api, nbi, nbe, T):
    """Gated product and down projection on the wide tile: I = nbi * 128, E = nbe * 128."""
    import torch

    b = 128
    rng = np.random.default_rng(4100 + nbi + nbe + T)
    sp = 0.93 if nbe > 8 else 0.5
    mg, mu = _skewed_mask(rng, nbi, nbe, sp), _skewed_mask(rng, nbi, nbe, sp)
    mu[3, :] = synth.uniform_mask(rng, 1, nbe, sp)[0]  # the full gate row meets an ordinary up row
    mu[7, :] = 1
    md = synth.uniform_mask(rng, nbe, nbi, sp)
    md[1, :] = 1
    md[2, :] = 0
    g, u, d = _sparse_weight(rng, mg, b), _sparse_weight(rng, mu, b), _sparse_weight(rng, md, b, 0.05)
    x = synth.gauss_bf16(rng, (T, nbe * b), 1.0)
    (dg, rg), (du, ru), (dd, rd) = _pack(api, g, b, mg), _pack(api, u, b, mu), _pack(api, d, b, md)
    dg = api.with_joint_row_order(dg, du)
    sel = stratified_tokens(T, 16)
    y_or = orc.mlp(rg, ru, rd, np.ascontiguousarray(x[sel]))
    y = api.sparse_mlp(dg, du, dd, to_dev(x), out=torch.full((T, nbe * b), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert np.isfinite(yh).all()
    fro, mx = check_close(yh[sel].T, y_or, f"wide mlp I={nbi * b} E={nbe * b} T={T}")
    assert not yh[:, 2 * b:3 * b].any()
    print(f"wide mlp {nbi}x{nbe} T={T}: rel_fro={fro:.2e} max_abs/rms={mx:.2e} on {sel.size} tokens")
