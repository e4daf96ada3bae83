"""GPU parity of the E5M2 path (Sec. 5.2): the quantiser is bit-exact against the oracle's, the product matches
the oracle's fp64 product of the same E5M2 codes within the tolerances of the 16-bit path."""
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


def _f32(bits):
    return synth.bf16_bits_to_f32(bits)


def test_quantize_every_bf16_pattern(api):
    """All 65536 bf16 bit patterns: normals, subnormal targets, ties, overflow, infinities, NaN."""
    import torch

    allbits = np.arange(65536, dtype=np.uint16)
    got = api.quantize_e5m2(to_dev(allbits)).cpu().numpy()
    want = orc.e5m2_quantize(_f32(allbits))
    nan = np.isnan(_f32(allbits))
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7C) == 0x7C) and np.all((got[nan] & 0x03) != 0)  # NaN stays NaN
    torch.cuda.synchronize()
    # a source that is only 2-byte aligned and a length that is no multiple of 8: same codes
    part = api.quantize_e5m2(to_dev(allbits)[5:65531]).cpu().numpy()
    assert np.array_equal(part, got[5:65531])
    tail = api.quantize_e5m2(to_dev(allbits)[:1003]).cpu().numpy()
    assert np.array_equal(tail, got[:1003])


def _case(api, rng, M, K, b, sparsity, T, w_std=0.05):
    W = synth.gauss_bf16(rng, (M, K), w_std)
    mask = synth.uniform_mask(rng, M // b, K // b, sparsity)
    if M // b > 2:
        mask[1, :] = 0
    dev = api.bsr_pack(to_dev(W), b, mask=mask_dev(mask))
    ref = orc.pack(W, b, mask)
    x = synth.gauss_bf16(rng, (T, K), 1.0)
    vals8 = api.quantize_e5m2(dev.vals[: max(dev.nnz, 1) * b * b].contiguous())
    x8 = api.quantize_e5m2(to_dev(x))
    v8_or = orc.e5m2_quantize(_f32(ref.vals))
    x8_or = orc.e5m2_quantize(_f32(x))
    assert np.array_equal(vals8.cpu().numpy()[: ref.nnz * b * b].reshape(ref.nnz, b, b), v8_or)
    assert np.array_equal(x8.cpu().numpy(), x8_or)
    return dev, ref, vals8, x8, v8_or, x8_or


@pytest.mark.parametrize("b", [16, 32, 64, 128])
@pytest.mark.parametrize("T", [1, 5, 64, 65, 128, 129, 300, 600])
def test_spmm_e5m2_small(api, b, T):
    import torch

    rng = np.random.default_rng(9990 + b + T)
    M, K = 6 * b, 4 * b
    dev, ref, vals8, x8, v8_or, x8_or = _case(api, rng, M, K, b, 0.5, T)
    y = api.bsr_spmm_e5m2(dev, vals8, x8, out=torch.full((T, M), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, orc.spmm_e5m2(ref, v8_or, x8_or), f"e5m2 b={b} T={T}")
    assert not y.cpu().numpy()[:, b:2 * b].any()


@pytest.mark.parametrize("b", [64, 128])
@pytest.mark.parametrize("T", [1, 5, 65, 129, 300])
def test_spmm_e5m2_column_groups(api, b, T):
    """Activations quantised into column groups of 64 features: the codes are the token-major ones, permuted
    (bit for bit), and the product equals the oracle's on the plain codes; also from a strided bf16 source, with
    bf16 output, and with rows long enough for the chunk plan."""
    import torch

    rng = np.random.default_rng(9700 + b + T)
    M, K = 3 * b, 80 * 64
    W = synth.gauss_bf16(rng, (M, K), 0.05)
    mask = synth.uniform_mask(rng, M // b, K // b, 0.6)
    mask[1, :] = 0
    mask[2, :] = 1  # a full row: 80 or 40 blocks
    dev = api.bsr_pack(to_dev(W), b, mask=mask_dev(mask))
    ref = orc.pack(W, b, mask)
    x = synth.gauss_bf16(rng, (T, K), 1.0)
    vals8 = api.quantize_e5m2(dev.vals[: dev.nnz * b * b].contiguous())
    v8_or = orc.e5m2_quantize(_f32(ref.vals))
    x8_or = orc.e5m2_quantize(_f32(x))
    xg = api.quantize_e5m2_groups(to_dev(x))
    assert xg.shape == (K // 64, T, 64)
    assert np.array_equal(xg.cpu().numpy(), x8_or.reshape(T, K // 64, 64).transpose(1, 0, 2))
    # the same from a source with a row pitch
    wide = torch.zeros((T, K + 24), dtype=torch.bfloat16, device="cuda:0")
    wide[:, :K] = to_dev(x)
    assert torch.equal(api.quantize_e5m2_groups(wide[:, :K]), xg)
    want = orc.spmm_e5m2(ref, v8_or, x8_or)
    y = api.bsr_spmm_e5m2(dev, vals8, xg, layout=api.COLUMN_GROUPS_64, out=torch.full((T, M), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, want, f"e5m2 column groups b={b} T={T}")
    assert not y.cpu().numpy()[:, b:2 * b].any()
    # token-major codes give the same sums in the same order
    y_tm = api.bsr_spmm_e5m2(dev, vals8, api.quantize_e5m2(to_dev(x)))
    if T > 128:  # (with few tokens and long rows the token-major call adds chunks atomically, in any order)
        assert torch.equal(y, y_tm)
    yb = api.bsr_spmm_e5m2(dev, vals8, xg, layout=api.COLUMN_GROUPS_64, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    got = synth.bf16_bits_to_f32(bits_of(yb)).astype(np.float64).T
    # one bf16 ulp of the value, plus the fp32 accumulation error of 5120 terms where the sum is near zero
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -7 + 1e-4 * np.sqrt((want ** 2).mean()))


def test_spmm_e5m2_column_groups_rejects_small_blocks(api):
    import torch

    rng = np.random.default_rng(5)
    W = synth.gauss_bf16(rng, (64, 128), 0.05)
    dev = api.bsr_pack(to_dev(W), 32, sparsity=0.5)
    vals8 = api.quantize_e5m2(dev.vals[: dev.nnz * 32 * 32].contiguous())
    xg = api.quantize_e5m2_groups(to_dev(synth.gauss_bf16(rng, (4, 128), 1.0)))
    with pytest.raises(api.BlastError):
        api.bsr_spmm_e5m2(dev, vals8, xg, layout=api.COLUMN_GROUPS_64)
    torch.cuda.synchronize()


def test_spmm_e5m2_layouts_bf16_out_and_unaligned(api):
    import torch

    rng = np.random.default_rng(9995)
    b, M, K, T = 64, 256, 192, 70
    dev, ref, vals8, x8, v8_or, x8_or = _case(api, rng, M, K, b, 0.4, T)
    want = orc.spmm_e5m2(ref, v8_or, x8_or)
    yf = api.bsr_spmm_e5m2(dev, vals8, x8.t().contiguous(), layout=api.FEATURE_MAJOR)
    torch.cuda.synchronize()
    check_close(yf.cpu().numpy(), want, "e5m2 feature-major")
    yb = api.bsr_spmm_e5m2(dev, vals8, x8, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ybf = yb.float().cpu().numpy().T
    assert np.all(np.abs(ybf - want) <= 2.0 ** -8 * np.abs(want) + 1e-2 * np.sqrt((want ** 2).mean()))
    # a row pitch that is not a multiple of 16 bytes: plain kernel
    big = torch.zeros((T, K + 5), dtype=torch.uint8, device="cuda:0")
    big[:, :K] = x8
    yu = api.bsr_spmm_e5m2(dev, vals8, big[:, :K])
    torch.cuda.synchronize()
    check_close(yu.cpu().numpy().T, want, "e5m2 unaligned")
    # a pitch larger than the width, still aligned: tuned kernel
    big2 = torch.zeros((T, K + 64), dtype=torch.uint8, device="cuda:0")
    big2[:, :K] = x8
    ys = api.bsr_spmm_e5m2(dev, vals8, big2[:, :K])
    torch.cuda.synchronize()
    check_close(ys.cpu().numpy().T, want, "e5m2 strided")


def test_spmm_e5m2_exact_on_representable_data_and_dense_empty(api):
    """Operands that are exact in E5M2 with integer-valued products: the device must match the oracle exactly,
    whatever the order of the additions (covers the four-wave split and its reduction)."""
    import torch

    rng = np.random.default_rng(9996)
    b, M, K = 64, 256, 1024
    Wv = rng.choice([-2.0, -1.0, 0.0, 1.0, 2.0, 3.0], size=(M, K)).astype(np.float32)
    W = synth.f32_to_bf16_bits(Wv)
    for sparsity in (0.0, 0.7, 1.0):
        mask = synth.uniform_mask(rng, M // b, K // b, sparsity)
        dev = api.bsr_pack(to_dev(W), b, mask=mask_dev(mask))
        ref = orc.pack(W, b, mask)
        vals8 = api.quantize_e5m2(dev.vals[: max(dev.nnz, 1) * b * b].contiguous())
        for T in (3, 100, 400):
            x = synth.f32_to_bf16_bits(rng.choice([-1.0, 0.0, 1.0, 2.0], size=(T, K)).astype(np.float32))
            y = api.bsr_spmm_e5m2(dev, vals8, api.quantize_e5m2(to_dev(x)))
            torch.cuda.synchronize()
            want = orc.spmm_e5m2(ref, orc.e5m2_quantize(_f32(ref.vals)), orc.e5m2_quantize(_f32(x)))
            assert np.array_equal(y.cpu().numpy().T.astype(np.float64), want), (sparsity, T)


def test_spmm_e5m2_llama1b_gate_full_size(api):
    import torch

    wl = synth.WORKLOADS["llama1b_b64_s90"]
    lin = synth.make_mlp(wl).gate
    b = wl.b
    dev = api.bsr_pack(to_dev(lin.W), b, mask=mask_dev(lin.mask))
    ref = orc.pack(lin.W, b, lin.mask)
    vals8 = api.quantize_e5m2(dev.vals[: dev.nnz * b * b].contiguous())
    v8_or = orc.e5m2_quantize(_f32(ref.vals))
    assert np.array_equal(vals8.cpu().numpy().reshape(ref.nnz, b, b), v8_or)
    for T in (1, 16, 2048):
        x = synth.make_x(wl, T)
        x8 = api.quantize_e5m2(to_dev(x))
        y = api.bsr_spmm_e5m2(dev, vals8, x8)
        torch.cuda.synchronize()
        sel = np.arange(T) if T <= 64 else np.unique(np.concatenate(([0, T - 1], np.random.default_rng(T).choice(T, 46, replace=False))))
        want = orc.spmm_e5m2(ref, v8_or, orc.e5m2_quantize(_f32(x[sel])))
        check_close(y.cpu().numpy()[sel].T, want, f"e5m2 1B gate T={T}")
        yg = api.bsr_spmm_e5m2(dev, vals8, api.quantize_e5m2_groups(to_dev(x)), layout=api.COLUMN_GROUPS_64)
        torch.cuda.synchronize()
        check_close(yg.cpu().numpy()[sel].T, want, f"e5m2 1B gate, column groups, T={T}")


@pytest.mark.parametrize("b,nbc,T", [(64, 80, 1), (64, 80, 20), (64, 80, 100), (128, 70, 5), (128, 70, 128), (64, 80, 300)])
def test_spmm_e5m2_heavy_rows(api, b, nbc, T):
    """Rows much longer than a chunk: with few tokens and fp32 output the chunks of a row add atomically into
    cleared rows (poisoned output, two calls in a row); bf16 output and many tokens take the unsplit forms."""
    import torch

    rng = np.random.default_rng(9997 + b + T)
    nbr = 6
    mask = synth.uniform_mask(rng, nbr, nbc, 0.9)
    mask[0, :] = 1
    mask[2, : (3 * nbc) // 4] = 1
    mask[4, :] = 0
    W = synth.gauss_bf16(rng, (nbr * b, nbc * b), 0.05)
    dev = api.bsr_pack(to_dev(W), b, mask=mask_dev(mask))
    ref = orc.pack(W, b, mask)
    assert dev.max_row_blocks == nbc
    x = synth.gauss_bf16(rng, (T, nbc * b), 1.0)
    vals8 = api.quantize_e5m2(dev.vals[: dev.nnz * b * b].contiguous())
    x8 = api.quantize_e5m2(to_dev(x))
    want = orc.spmm_e5m2(ref, orc.e5m2_quantize(_f32(ref.vals)), orc.e5m2_quantize(_f32(x)))
    for _ in range(2):
        y = api.bsr_spmm_e5m2(dev, vals8, x8, out=torch.full((T, nbr * b), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, want, f"e5m2 heavy rows b={b} T={T}")
    assert not y.cpu().numpy()[:, 4 * b:5 * b].any()
    yb = api.bsr_spmm_e5m2(dev, vals8, x8, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert np.abs(yb.float().cpu().numpy().T - want).max() <= 2.0 ** -7 * np.abs(want).max()


# ---- E5M2 weights, bf16 activations: the decode form of the gated MLP ----

def _w8_layer(api, rng, E, I, b, sparsity, masks=None):
    Ws = [synth.gauss_bf16(rng, s, 0.05) for s in ((I, E), (I, E), (E, I))]
    if masks is None:
        masks = [synth.uniform_mask(rng, r // b, c // b, sparsity) for r, c in ((I, E), (I, E), (E, I))]
        if I // b > 2:
            masks[0][1, :] = 0   # an empty gate row: zero rows of H
            masks[2][:, 2] = 0   # rows of H nobody reads
        if E // b > 1:
            masks[2][1, :] = 0   # an empty row of the down projection
    dev = [api.bsr_pack(to_dev(w), b, mask=mask_dev(m)) for w, m in zip(Ws, masks)]
    ref = [orc.pack(w, b, m) for w, m in zip(Ws, masks)]
    dev8 = [api.quantize_e5m2(d.vals[: max(d.nnz, 1) * b * b].contiguous()) for d in dev]
    ref8 = [orc.e5m2_quantize(_f32(r.vals)) for r in ref]
    for d8, r8, r in zip(dev8, ref8, ref):
        assert np.array_equal(d8.cpu().numpy()[: r.nnz * b * b].reshape(r.nnz, b, b), r8)
    return dev, dev8, ref, ref8


@pytest.mark.parametrize("b", [64, 128])
@pytest.mark.parametrize("T", [1, 4, 5, 8, 9, 16, 17, 32, 33, 70])
def test_mlp_with_e5m2_weights_small(api, b, T):
    import torch

    rng = np.random.default_rng(5200 + b + T)
    E, I = 4 * b, 6 * b
    dev, dev8, ref, ref8 = _w8_layer(api, rng, E, I, b, 0.5)
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    y_or = orc.mlp_e5m2w(ref[0], ref8[0], ref[1], ref8[1], ref[2], ref8[2], x)
    y = api.sparse_mlp_e5m2w(dev[0], dev8[0], dev[1], dev8[1], dev[2], dev8[2], to_dev(x),
                             out=torch.full((T, E), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    check_close(yh.T, y_or, f"E5M2-weight mlp b={b} T={T}")
    assert not yh[:, b:2 * b].any()
    # bf16 output and another activation
    yb = api.sparse_mlp_e5m2w(dev[0], dev8[0], dev[1], dev8[1], dev[2], dev8[2], to_dev(x), act="gelu",
                              out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    yg = orc.mlp_e5m2w(ref[0], ref8[0], ref[1], ref8[1], ref[2], ref8[2], x, activation="gelu")
    assert np.abs(yb.float().cpu().numpy().T - yg).max() <= 2.0 ** -7 * np.abs(yg).max() + 1e-6


def test_e5m2_weight_conversion_covers_every_code(api):
    """A block whose 4096 values run through all 256 codes that are finite (subnormals included): the widening to
    bf16 inside the kernel is exact, so an identity-like activation picks every code out unchanged."""
    import torch

    b, T = 64, 64
    codes = np.array([c for c in range(256) if (c & 0x7C) != 0x7C], dtype=np.uint8)  # finite codes
    vals = np.resize(codes, b * b).reshape(1, b, b)
    dec = orc.e5m2_decode(vals.ravel()).reshape(b, b)
    # gate = up = down structure: one stored block at (0, 0) of a 64 x 64 matrix; X = identity picks columns
    mask = np.ones((1, 1), dtype=np.uint8)
    W = synth.f32_to_bf16_bits(dec.astype(np.float32))  # exact: every E5M2 value is a bf16 value
    dev = api.bsr_pack(to_dev(W), b, mask=mask_dev(mask))
    ref = orc.pack(W, b, mask)
    d8 = api.quantize_e5m2(dev.vals[: b * b].contiguous())
    assert np.array_equal(d8.cpu().numpy().reshape(1, b, b), vals)
    x = synth.f32_to_bf16_bits(np.eye(b, dtype=np.float32))
    y = api.sparse_mlp_e5m2w(dev, d8, dev, d8, dev, d8, to_dev(x), act="relu")
    torch.cuda.synchronize()
    check_close(y.cpu().numpy().T, orc.mlp_e5m2w(ref, vals, ref, vals, ref, vals, x, activation="relu"), "all codes")


@pytest.mark.parametrize("name,T", [("llama1b_b64_s90", 1), ("llama1b_b64_s90", 16), ("llama8b_b128_s95", 1),
                                    ("llama8b_b128_s95", 32)])
def test_mlp_with_e5m2_weights_at_decode_configs(api, name, T):
    import torch

    wl = synth.WORKLOADS[name]
    inp = synth.make_mlp(wl)
    rng = np.random.default_rng(5300 + T)
    dev = [api.bsr_pack(to_dev(l.W), wl.b, mask=mask_dev(l.mask)) for l in (inp.gate, inp.up, inp.down)]
    ref = [orc.pack(l.W, wl.b, l.mask) for l in (inp.gate, inp.up, inp.down)]
    dev8 = [api.quantize_e5m2(d.vals[: d.nnz * wl.b * wl.b].contiguous()) for d in dev]
    ref8 = [orc.e5m2_quantize(_f32(r.vals)) for r in ref]
    x = synth.make_x(wl, T)
    y = api.sparse_mlp_e5m2w(dev[0], dev8[0], dev[1], dev8[1], dev[2], dev8[2], to_dev(x),
                             out=torch.full((T, wl.hidden), float("nan"), device="cuda:0"))
    torch.cuda.synchronize()
    fro, mx = check_close(y.cpu().numpy().T, orc.mlp_e5m2w(ref[0], ref8[0], ref[1], ref8[1], ref[2], ref8[2], x),
                          f"{name} E5M2 weights T={T}")
    print(f"{name} E5M2 weights T={T}: rel_fro={fro:.2e} max_abs/rms={mx:.2e}")


def test_e5m2_weight_mlp_argument_errors(api):
    import ctypes as C

    L = api.lib()
    v = api.BsrView(64, 64, 32, 0, 0, None, None, None, None, None)
    dummy = (C.c_int32 * 4)()
    v.row_ptr = C.cast(dummy, C.c_void_p)
    # b = 32 is not served by this call
    assert L.blast_sparse_mlp_e5m2w(C.byref(v), None, C.byref(v), None, C.byref(v), None, None, 64, 0, 0, None, 64, 0,
                                    None, 0, None) == -3
    wsb = C.c_size_t(0)
    v64 = api.BsrView(128, 128, 64, 0, 0, v.row_ptr, None, None, None, None)
    assert L.blast_sparse_mlp_e5m2w_workspace(C.byref(v64), 16, C.byref(wsb)) == 0 and wsb.value == 16 * 128 * 2
    assert L.blast_sparse_mlp_e5m2w(C.byref(v64), None, None, None, C.byref(v64), None, None, 128, 4, 0, None, 128, 0,
                                    None, 0, None) == -1  # no up matrix


@pytest.mark.parametrize("b,nbi,T", [(64, 272, 1), (64, 272, 20), (128, 260, 5), (128, 260, 40)])
def test_mlp_with_e5m2_weights_and_a_very_long_down_row(api, b, nbi, T):
    """A row of W_down long enough for the chunk plan: its chunks add into rows cleared by a launch of their own
    (fp32 output, poisoned Y); the bf16 output of the same layer takes whole rows."""
    import torch

    rng = np.random.default_rng(5400 + b + T)
    E, I = 4 * b, nbi * b
    mg, mu = (synth.uniform_mask(rng, nbi, E // b, 0.5) for _ in range(2))
    md = synth.uniform_mask(rng, E // b, nbi, 0.9)
    md[0, :] = 1   # nbi blocks: cut into chunks of 16
    md[2, :] = 0   # an empty row beside it
    dev, dev8, ref, ref8 = _w8_layer(api, rng, E, I, b, 0.0, masks=[mg, mu, md])
    assert dev[2].max_row_blocks == nbi
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    want = orc.mlp_e5m2w(ref[0], ref8[0], ref[1], ref8[1], ref[2], ref8[2], x)
    for _ in range(2):
        y = api.sparse_mlp_e5m2w(dev[0], dev8[0], dev[1], dev8[1], dev[2], dev8[2], to_dev(x),
                                 out=torch.full((T, E), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, want, f"E5M2-weight mlp, long down row b={b} T={T}")
    assert not y.cpu().numpy()[:, 2 * b:3 * b].any()
    yb = api.sparse_mlp_e5m2w(dev[0], dev8[0], dev[1], dev8[1], dev[2], dev8[2], to_dev(x), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert np.abs(yb.float().cpu().numpy().T - want).max() <= 2.0 ** -7 * np.abs(want).max() + 1e-6
