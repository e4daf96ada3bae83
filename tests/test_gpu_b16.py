"""16 x 16 blocks: the kernel that multiplies pairs of stored blocks on the 32-deep matrix instruction
(csrc/kern_b16.h) against the oracle - odd and even block counts per row, every token-tile boundary, both output
types, strided and unaligned outputs, the gated and the activated form, and the 1B-shaped layer at full size."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2507_03117_amd import synth
from tests.helpers import bits_of, check_close, mask_dev, stratified_tokens, to_dev

pytestmark = pytest.mark.gpu

B = 16


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available()
    from paper_2507_03117_amd import api as _api

    _api.lib()
    return _api


def _rows_with_counts(rng, counts, nbc):
    mask = np.zeros((len(counts), nbc), dtype=np.uint8)
    for r, c in enumerate(counts):
        mask[r, rng.choice(nbc, size=c, replace=False)] = 1
    return mask


def _pack(api, w, mask):
    dev = api.bsr_pack(to_dev(w), B, mask=mask_dev(mask))
    ref = orc.pack(w, B, mask)
    assert np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)
    return dev, ref


@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 31, 32, 33, 48, 63, 64, 65, 127, 129, 300])
def test_spmm_every_block_count_and_tile_edge(api, T):
    """Block rows holding 0 ... 9 and all 12 blocks (odd counts end in half a pair), token counts on both sides of
    every tile size the launcher picks (16, 32, 64 tokens per wave)."""
    import torch

    rng = np.random.default_rng(1600 + T)
    counts = [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 1, 0, 2]
    nbc = 12
    mask = _rows_with_counts(rng, counts, nbc)
    w = synth.gauss_bf16(rng, (len(counts) * B, nbc * B), 0.02)
    x = synth.gauss_bf16(rng, (T, nbc * B), 1.0)
    dev, ref = _pack(api, w, mask)
    y_or = orc.spmm(ref, x)
    y = api.bsr_spmm(dev, to_dev(x), out=torch.full((T, len(counts) * B), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    check_close(yh.T, y_or, f"b=16 spmm T={T}")
    assert not yh[:, :B].any() and not yh[:, 12 * B:13 * B].any()  # empty block rows: exact zeros
    yb = api.bsr_spmm(dev, to_dev(x), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    got = synth.bf16_bits_to_f32(bits_of(yb)).astype(np.float64).T
    want = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(y_or.astype(np.float32))).astype(np.float64)
    # the fp32 accumulator rounded to nearest even: within one bf16 ulp of the rounded oracle
    assert np.all(np.abs(got - want) <= np.maximum(np.abs(want), 1e-30) * 2.0 ** -7 + 1e-12)


@pytest.mark.parametrize("T", [1, 7, 16])
@pytest.mark.parametrize("gated", [False, True])
def test_long_rows_at_decode_token_counts(api, T, gated):
    """Rows of 30-80 blocks at up to 16 tokens: sixteen waves deal a row's pairs (some get none, one gets the
    odd last block) and their partial sums are added in LDS."""
    import torch

    rng = np.random.default_rng(1650 + T)
    counts = [80, 33, 47, 0, 61]
    nbc = 80
    w = synth.gauss_bf16(rng, (len(counts) * B, nbc * B), 0.02)
    x = synth.gauss_bf16(rng, (T, nbc * B), 1.0)
    dev, ref = _pack(api, w, _rows_with_counts(rng, counts, nbc))
    if not gated:
        y = api.bsr_spmm(dev, to_dev(x), out=torch.full((T, len(counts) * B), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.spmm(ref, x), f"b=16 long rows T={T}")
        return
    w2 = synth.gauss_bf16(rng, (len(counts) * B, nbc * B), 0.02)
    dev2, ref2 = _pack(api, w2, _rows_with_counts(rng, counts[::-1], nbc))
    h = api.bsr_gated_spmm(dev, dev2, to_dev(x))
    torch.cuda.synchronize()
    rd = orc.pack(synth.gauss_bf16(rng, (nbc * B, len(counts) * B), 0.05), B,
                  synth.uniform_mask(rng, nbc, len(counts), 0.5))
    _, h_or = orc.mlp(ref, ref2, rd, x, return_h=True)
    got = synth.bf16_bits_to_f32(bits_of(h)).astype(np.float64).T
    want = synth.bf16_bits_to_f32(h_or).astype(np.float64)
    assert (np.abs(got - want) <= np.abs(want) * 2.0 ** -7 + 1e-5 * np.sqrt((want ** 2).mean())).all()


@pytest.mark.parametrize("T", [5, 40, 130])
def test_spmm_strided_and_unaligned_operands(api, T):
    """Outputs whose row pitch or address rules out the 16-byte stores take the element-wise stores of the same
    kernel; activations whose rows are not 16-byte aligned take the generic tile kernel."""
    import torch

    rng = np.random.default_rng(1700 + T)
    nbr, nbc = 6, 9
    mask = synth.uniform_mask(rng, nbr, nbc, 0.5)
    w = synth.gauss_bf16(rng, (nbr * B, nbc * B), 0.02)
    x = synth.gauss_bf16(rng, (T, nbc * B), 1.0)
    dev, ref = _pack(api, w, mask)
    y_or = orc.spmm(ref, x)
    big = torch.full((T, nbr * B + 6), float("nan"), device="cuda:0")
    for out in (big[:, :nbr * B], big[:, 1:nbr * B + 1], big[:, 4:nbr * B + 4]):  # pitch 102 floats; offsets 0, 4, 16 bytes
        big.fill_(float("nan"))
        api.bsr_spmm(dev, to_dev(x), out=out)
        torch.cuda.synchronize()
        check_close(out.cpu().numpy().T, y_or, f"b=16 strided out T={T}")
    xp = torch.zeros((T, nbc * B + 4), dtype=torch.int16, device="cuda:0")
    xs = xp[:, 2:nbc * B + 2]  # rows start 4 bytes off a 16-byte boundary, pitch 148 elements
    xs.copy_(to_dev(x).view(torch.int16))
    y = api.bsr_spmm(dev, xs)
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, y_or, f"b=16 unaligned X T={T}")


@pytest.mark.parametrize("T", [1, 16, 33, 100])
@pytest.mark.parametrize("act", ["silu", "gelu", "relu"])
def test_gated_product_matches_the_oracles_intermediate(api, T, act):
    """H = act(G) * U in bf16: bit patterns against the oracle's H (one bf16 ulp where the fp32 sums differ in
    their last bits)."""
    import torch

    rng = np.random.default_rng(1800 + T)
    E, I = 8 * B, 11 * B
    g, u = (synth.gauss_bf16(rng, (I, E), 0.05) for _ in range(2))
    mg, mu = (synth.uniform_mask(rng, I // B, E // B, 0.4) for _ in range(2))
    mg[2, :] = 0
    mu[5, :] = 0
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    dg, rg = _pack(api, g, mg)
    du, ru = _pack(api, u, mu)
    h = api.bsr_gated_spmm(dg, du, to_dev(x), act=act)
    torch.cuda.synchronize()
    rd = orc.pack(synth.gauss_bf16(rng, (E, I), 0.05), B, synth.uniform_mask(rng, E // B, I // B, 0.5))
    _, h_or = orc.mlp(rg, ru, rd, x, activation=act, return_h=True)  # bf16 bits [I, T]
    got = synth.bf16_bits_to_f32(bits_of(h)).astype(np.float64).T
    want = synth.bf16_bits_to_f32(h_or).astype(np.float64)
    diff = np.abs(got - want)
    # one bf16 ulp, plus the fp32-vs-fp64 accumulation error of G and U where h is nearly cancelled
    assert (diff <= np.abs(want) * 2.0 ** -7 + 1e-5 * np.sqrt((want ** 2).mean())).all()
    assert (diff > 0).mean() < 0.03
    assert not got[2 * B:3 * B].any() and not got[5 * B:6 * B].any()


def test_mlp_random_shapes(api):
    """Twenty seeded random 16-wide-block MLPs (random sizes, sparsities, token counts, activations): Y against the
    oracle.  Token counts from 33 on go through the regrouped activations, and once more with a workspace that
    has no room for them."""
    import torch

    rng = np.random.default_rng(1900)
    for case in range(20):
        E, I = int(rng.integers(1, 24)) * B, int(rng.integers(1, 40)) * B
        T = int(rng.choice([1, 3, 16, 17, 32, 33, 64, 65, 100, 257]))
        s = float(rng.choice([0.0, 0.3, 0.7, 0.9]))
        act = str(rng.choice(["silu", "gelu", "relu"]))
        g, u, d = (synth.gauss_bf16(rng, sh, 0.05) for sh in ((I, E), (I, E), (E, I)))
        mg, mu = (synth.uniform_mask(rng, I // B, E // B, s) for _ in range(2))
        md = synth.uniform_mask(rng, E // B, I // B, s)
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        (dg, rg), (du, ru), (dd, rd) = _pack(api, g, mg), _pack(api, u, mu), _pack(api, d, md)
        y_or = orc.mlp(rg, ru, rd, x, activation=act)
        y = api.sparse_mlp(dg, du, dd, to_dev(x), act=act, out=torch.full((T, E), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, y_or, f"b=16 mlp case {case}: E={E} I={I} T={T} s={s} {act}")
        if T >= 33:  # a workspace without room for the regrouped X: the same kernels on the token-major tensor
            small = api.mlp_workspace_bytes(dg, du, dd, T) - (2 * E * T + 255) // 256 * 256
            yb = api.sparse_mlp(dg, du, dd, to_dev(x), act=act,
                                ws=torch.empty(small, dtype=torch.uint8, device="cuda:0"))
            torch.cuda.synchronize()
            check_close(yb.cpu().numpy().T, y_or, f"b=16 mlp case {case}, small workspace")


@pytest.mark.parametrize("T", [1, 16, 128, 2048])
def test_llama1b_b16_mlp(api, T):
    """The 1B-shaped layer with 16 x 16 blocks at 90 %: 6553 blocks per matrix, about 13 per block row."""
    import torch

    wl = synth.WORKLOADS["llama1b_b16_s90"]
    inp = synth.make_mlp(wl)
    packs = []
    for l in (inp.gate, inp.up, inp.down):
        dev = api.bsr_pack(to_dev(l.W), B, mask=mask_dev(l.mask))
        ref = orc.pack(l.W, B, l.mask)
        assert dev.nnz == ref.nnz == 6553
        assert np.array_equal(dev.row_ptr.cpu().numpy(), ref.row_ptr)
        assert np.array_equal(dev.col_idx.cpu().numpy()[: ref.nnz], ref.col_idx)
        packs.append((dev, ref))
    (dg, rg), (du, ru), (dd, rd) = packs
    x = synth.make_x(wl, T)
    y = api.sparse_mlp(dg, du, dd, to_dev(x), out=torch.full((T, wl.hidden), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    sel = np.arange(T) if T <= 64 else stratified_tokens(T, 64)
    y_or = orc.mlp(rg, ru, rd, np.ascontiguousarray(x[sel]))
    y_h = y.cpu().numpy()
    assert np.isfinite(y_h).all()
    fro, mx = check_close(y_h[sel].T, y_or, f"llama1b_b16_s90 T={T}")
    print(f"llama1b_b16_s90 T={T}: rel_fro={fro:.2e} max_abs/rms={mx:.2e} on {sel.size} tokens")
