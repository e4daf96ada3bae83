"""Pins for the CPU oracle: every check compares the oracle with something that
is NOT the oracle (a library routine, a closed form, an exact brute force in
rational arithmetic, an invariant of the mathematics).  No GPU needed."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import oracle as orc
from paper_2507_03117_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f64(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def expand(mask, b):
    return np.kron(mask, np.ones((b, b), dtype=mask.dtype))


# ---------------------------------------------------------------- drop counts (ceil reading)
@pytest.mark.parametrize("n,s,keep", [
    (4096, 0.90, 409), (6144, 0.70, 1843), (6144, 0.80, 1228), (6144, 0.90, 614), (6144, 0.95, 307),
    (3584, 0.95, 179), (53248, 0.95, 2662), (10, 0.0, 10), (10, 1.0, 0), (7, 0.5, 3), (3, 0.34, 1),
])
def test_n_keep_table(n, s, keep):
    # closed form: n_keep = n - ceil(s*n) with s in exact basis points
    assert orc.n_keep(n, s) == keep
    assert keep == n - math.ceil(Fraction(round(s * 10000), 10000) * n)
    assert synth.n_zero_blocks(n, s) == n - keep


# ---------------------------------------------------------------- block scores
def test_scores_closed_forms():
    b = 4
    W = np.zeros((8, 12), dtype=np.float32)
    W[:4, :4] = 1.0  # score b*b
    W[:4, 4:8] = np.arange(16).reshape(4, 4)  # sum k^2 = 1240
    W[4:, 8:] = -0.5  # 16 * 0.25
    W[4, 0] = 3.0  # single entry
    s = orc.block_scores(synth.f32_to_bf16_bits(W), b)
    assert s.tolist() == [[16.0, 1240.0, 0.0], [9.0, 0.0, 4.0]]


def test_scores_match_numpy_and_expectation():
    rng = np.random.default_rng(1)
    Wb = synth.gauss_bf16(rng, (256, 384), 0.02)
    b = 32
    s = orc.block_scores(Wb, b)
    ref = (f64(Wb) ** 2).reshape(8, b, 12, b).sum(axis=(1, 3))
    np.testing.assert_allclose(s, ref, rtol=1e-13)
    # E[score] = b^2 * sigma^2
    assert abs(s.mean() / (b * b * 0.02 ** 2) - 1.0) < 0.03


# ---------------------------------------------------------------- top-k selection
def test_topk_equals_python_full_sort_and_threshold_property():
    rng = np.random.default_rng(2)
    score = rng.random((16, 24))
    score[3, 5] = score[7, 7] = score[0, 1]  # exact ties
    for s in (0.0, 0.3, 0.5, 0.9, 0.95, 1.0):
        mask, gap = orc.topk_mask(score, s)
        n = score.size
        keep = n - math.ceil(Fraction(round(s * 10000), 10000) * n)
        assert int(mask.sum()) == keep
        flat = score.ravel()
        order = sorted(range(n), key=lambda i: (-flat[i], i))
        ref = np.zeros(n, dtype=np.uint8)
        ref[order[:keep]] = 1
        assert np.array_equal(mask.ravel(), ref)
        if 0 < keep < n:
            assert flat[mask.ravel() == 1].min() >= flat[mask.ravel() == 0].max()


def test_topk_tie_break_prefers_lower_index():
    score = np.zeros((2, 4))  # all tied (e.g. all-zero blocks)
    mask, _ = orc.topk_mask(score, 0.5)
    assert mask.ravel().tolist() == [1, 1, 1, 1, 0, 0, 0, 0]
    score = np.array([[1.0, 5.0, 1.0, 1.0]])
    mask, _ = orc.topk_mask(score, 0.5)
    assert mask.ravel().tolist() == [1, 1, 0, 0]


def test_topk_gap_reported():
    score = np.array([[4.0, 3.0, 2.0, 1.0]])
    _, gap = orc.topk_mask(score, 0.5)
    assert gap == pytest.approx((3.0 - 2.0) / 3.0)


# ---------------------------------------------------------------- packing
@pytest.mark.parametrize("b", [1, 2, 16, 32])
def test_pack_roundtrip_and_scipy_indices(b):
    rng = np.random.default_rng(10 + b)
    rows, cols = 8 * b, 12 * b
    Wb = synth.gauss_bf16(rng, (rows, cols), 0.02)
    Wb[Wb == 0] = 0x3C00  # no exact zeros, so scipy's structure equals the mask
    Wb[Wb == 0x8000] = 0x3C00
    mask = synth.uniform_mask(rng, 8, 12, 0.7)
    mask[2, :] = 0  # an empty block row
    m = orc.pack(Wb, b, mask)
    # invariants
    assert m.row_ptr[0] == 0 and m.row_ptr[-1] == m.nnz == int(mask.sum())
    assert np.all(np.diff(m.row_ptr) >= 0)
    for r in range(8):
        c = m.col_idx[m.row_ptr[r]:m.row_ptr[r + 1]]
        assert np.all(np.diff(c) > 0) and np.all(c < 12) and np.all(c >= 0)
        assert np.array_equal(c, np.nonzero(mask[r])[0])
    # round trip bit-for-bit
    Wm = Wb * expand(mask, b).astype(np.uint16)
    assert np.array_equal(orc.unpack(m), Wm)
    # library routine
    dense = f64(Wm)
    if b == 1:
        ref = sp.csr_matrix(dense)
    else:
        ref = sp.bsr_matrix(dense, blocksize=(b, b))
    ref.sort_indices()
    assert np.array_equal(ref.indptr, m.row_ptr)
    assert np.array_equal(ref.indices, m.col_idx)
    if b > 1:
        assert np.array_equal(ref.data, f64(m.vals))  # blocks row-major, same order
    # schedule: stable sort by count, descending
    cnt = np.diff(m.row_ptr)
    assert np.array_equal(m.row_order, np.argsort(-cnt, kind="stable"))
    assert cnt[m.row_order[-1]] == 0


def test_pack_keeps_all_zero_block():
    b = 2
    W = np.zeros((4, 4), dtype=np.uint16)
    mask = np.array([[1, 0], [0, 1]], dtype=np.uint8)
    m = orc.pack(W, b, mask)
    assert m.nnz == 2 and m.col_idx.tolist() == [0, 1] and m.row_ptr.tolist() == [0, 1, 2]


def test_full_and_empty_masks():
    rng = np.random.default_rng(3)
    b = 4
    Wb = synth.gauss_bf16(rng, (16, 8), 0.02)
    Xb = synth.gauss_bf16(rng, (5, 8), 1.0)
    full, _, _ = orc.pack_topk(Wb, b, 0.0)
    assert full.nnz == 8 and np.array_equal(orc.unpack(full), Wb)
    Y = orc.spmm(full, Xb)
    np.testing.assert_allclose(Y, f64(Wb) @ f64(Xb).T, rtol=1e-12, atol=1e-300)
    empty, _, _ = orc.pack_topk(Wb, b, 1.0)
    assert empty.nnz == 0 and not empty.row_ptr.any()
    assert not orc.spmm(empty, Xb).any()


# ---------------------------------------------------------------- SpMM
def test_spmm_dense_case_equals_numpy_both_layouts():
    rng = np.random.default_rng(4)
    b = 16
    Wb = synth.gauss_bf16(rng, (64, 96), 0.02)
    Xb = synth.gauss_bf16(rng, (7, 96), 1.0)  # token-major [T, K]
    mask = synth.uniform_mask(rng, 4, 6, 0.5)
    m = orc.pack(Wb, b, mask)
    ref = (f64(Wb) * expand(mask, b)) @ f64(Xb).T
    np.testing.assert_allclose(orc.spmm(m, Xb, "token_major"), ref, rtol=1e-12, atol=1e-15)
    Xf = np.ascontiguousarray(Xb.T)  # feature-major [K, T]
    np.testing.assert_allclose(orc.spmm(m, Xf, "feature_major"), ref, rtol=1e-12, atol=1e-15)


def _brute_spmm(Wi, mask, b, Xi):
    """Exact rational evaluation, written independently (pure Python)."""
    M, K = len(Wi), len(Wi[0])
    T = len(Xi[0])
    Y = [[Fraction(0)] * T for _ in range(M)]
    for i in range(M):
        for k in range(K):
            if mask[i // b][k // b]:
                for t in range(T):
                    Y[i][t] += Fraction(Wi[i][k]) * Fraction(Xi[k][t])
    return Y


@pytest.mark.parametrize("M,K,b,T,seed", [(2, 2, 1, 1, 0), (4, 6, 2, 3, 1), (8, 4, 4, 2, 2), (6, 8, 2, 1, 3), (8, 8, 4, 3, 4)])
def test_spmm_brute_force_exact(M, K, b, T, seed):
    rng = np.random.default_rng(seed)
    Wi = rng.integers(-8, 9, size=(M, K))  # small integers are exact in bf16
    Xi = rng.integers(-8, 9, size=(K, T))
    mask = (rng.random((M // b, K // b)) < 0.6).astype(np.uint8)
    m = orc.pack(synth.f32_to_bf16_bits(Wi.astype(np.float32)), b, mask)
    Xf = synth.f32_to_bf16_bits(Xi.astype(np.float32))  # feature-major [K, T]
    Y = orc.spmm(m, Xf, "feature_major")
    ref = _brute_spmm(Wi.tolist(), mask.tolist(), b, Xi.tolist())
    for i in range(M):
        for t in range(T):
            assert Fraction(Y[i, t]) == ref[i][t]


def test_token_independence_bitwise():
    w, mask, x = synth.small_case(5, 64, 96, 16, 0.6, 9)
    m = orc.pack(w, 16, mask)
    full = orc.spmm(m, x)
    cols = [7, 0, 3]
    sub = orc.spmm(m, np.ascontiguousarray(x[cols]))
    assert np.array_equal(full[:, cols], sub)


def test_transpose_symmetry():
    # Sec. 3.4.1: Y = XW and Y = WX are the same kernel mirrored.
    w, mask, x = synth.small_case(6, 48, 80, 16, 0.5, 5)
    m = orc.pack(w, 16, mask)
    Y = orc.spmm(m, x)  # [rows, T]
    Wt = (f64(w) * expand(mask, 16)).T  # paper's orientation: in x out
    np.testing.assert_allclose(Y.T, f64(x) @ Wt, rtol=1e-12, atol=1e-15)
    # BSR(W) <-> BCSC(W^T): scipy's BSC-like view via transpose
    csc = sp.bsr_matrix(Wt.T, blocksize=(16, 16))
    csc.sort_indices()
    assert np.array_equal(csc.indptr, m.row_ptr) and np.array_equal(csc.indices, m.col_idx)


def test_linearity_identity_permutation():
    rng = np.random.default_rng(7)
    b = 8
    w, mask, x1 = synth.small_case(7, 32, 48, b, 0.5, 4)
    x2 = synth.gauss_bf16(rng, x1.shape, 1.0)
    m = orc.pack(w, b, mask)
    # linearity in X needs exactly representable sums: use x2 := 2 * x1 (exact in bf16) and a zero
    x_twice = synth.f32_to_bf16_bits(2.0 * synth.bf16_bits_to_f32(x1))
    np.testing.assert_allclose(orc.spmm(m, x_twice), 2.0 * orc.spmm(m, x1), rtol=1e-15)
    # additivity in W over disjoint masks
    mask_a = mask.copy()
    mask_a[:, ::2] = 0
    mask_b = mask - mask_a
    ya = orc.spmm(orc.pack(w, b, mask_a), x2)
    yb = orc.spmm(orc.pack(w, b, mask_b), x2)
    np.testing.assert_allclose(ya + yb, orc.spmm(m, x2), rtol=1e-12, atol=1e-15)
    # block-diagonal identity copies X
    n = 32
    eye = synth.f32_to_bf16_bits(np.eye(n, dtype=np.float32))
    xe = synth.gauss_bf16(rng, (5, n), 1.0)
    me = orc.pack(eye, b, np.eye(n // b, dtype=np.uint8))
    assert np.array_equal(orc.spmm(me, xe), f64(xe).T)
    # permuting block columns of W with the matching row blocks of X leaves Y unchanged
    perm = rng.permutation(48 // b)
    idx = (perm[:, None] * b + np.arange(b)[None, :]).ravel()
    mp = orc.pack(np.ascontiguousarray(w[:, idx]), b, np.ascontiguousarray(mask[:, perm]))
    np.testing.assert_allclose(orc.spmm(mp, np.ascontiguousarray(x2[:, idx])), orc.spmm(m, x2), rtol=1e-12, atol=1e-15)


def test_spmm_statistics_config1_shape():
    # RMS(Y) ~ sigma_w * sqrt(b * mean blocks per row) for unit-variance X
    wl = synth.WORKLOADS["linear_1024x4096_b32_s90"]
    lin = synth.make_linear(wl)
    x = synth.make_x(wl, 8)
    m = orc.pack(lin.W, wl.b, lin.mask)
    assert m.nnz == 409
    Y = orc.spmm(m, x)
    rms = math.sqrt(float((Y ** 2).mean()))
    assert abs(rms / (0.02 * math.sqrt(32 * 409 / 32)) - 1.0) < 0.05


def test_f32_accumulation_bound():
    w, mask, x = synth.small_case(8, 128, 1024, 32, 0.5, 6)
    m = orc.pack(w, 32, mask)
    y64 = orc.spmm(m, x)
    y32 = orc.spmm(m, x, f32acc=True)
    rel = np.linalg.norm(y32 - y64) / np.linalg.norm(y64)
    assert 0 < rel < 1e-5


# ---------------------------------------------------------------- activations and the MLP
def test_activation_golden_values():
    for line in open(os.path.join(GOLDEN, "activation_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, x, v = line.split()
        assert orc.act(name, float(x)) == pytest.approx(float(v), rel=1e-14, abs=1e-300)
    # global minimum of SiLU
    xs = np.linspace(-3, 0, 30001)
    vals = np.array([orc.act("silu", float(t)) for t in xs])
    assert abs(xs[vals.argmin()] + 1.27846) < 2e-4 and abs(vals.min() + 0.27846) < 1e-5


def _np_mlp(wg, wu, wd, xb, act):
    X = f64(xb).T  # [E, T]
    G, U = wg @ X, wu @ X
    if act == "silu":
        a = G / (1.0 + np.exp(-G))
    elif act == "gelu":
        a = 0.5 * G * (1.0 + np.vectorize(math.erf)(G / math.sqrt(2.0)))
    else:
        a = np.maximum(G, 0.0)
    H = f64(synth.f32_to_bf16_bits((a * U).astype(np.float32)))
    return wd @ H, H


@pytest.mark.parametrize("act", ["silu", "gelu", "relu"])
def test_mlp_equals_numpy_dense_formula(act):
    rng = np.random.default_rng(11)
    E, I, b, T = 64, 128, 16, 6
    g, u, d = (synth.gauss_bf16(rng, s, 0.2) for s in ((I, E), (I, E), (E, I)))
    mg, mu, md = (synth.uniform_mask(rng, *s, 0.5) for s in ((I // b, E // b), (I // b, E // b), (E // b, I // b)))
    mg[1, :] = 0  # empty gate row -> H row zero
    xb = synth.gauss_bf16(rng, (T, E), 1.0)
    pg, pu, pd = orc.pack(g, b, mg), orc.pack(u, b, mu), orc.pack(d, b, md)
    Y, H = orc.mlp(pg, pu, pd, xb, activation=act, return_h=True)
    Yref, Href = _np_mlp(f64(g) * expand(mg, b), f64(u) * expand(mu, b), f64(d) * expand(md, b), xb, act)
    # H may differ from numpy's only where exp/erf differ in the last ulp before rounding: allow none here
    assert np.array_equal(f64(H), Href)
    np.testing.assert_allclose(Y, Yref, rtol=1e-12, atol=1e-15)
    assert not f64(H)[b:2 * b].any()
    # feature-major input gives the same result
    Y2 = orc.mlp(pg, pu, pd, np.ascontiguousarray(xb.T), layout="feature_major", activation=act)
    assert np.array_equal(Y, Y2)


def test_mlp_special_cases():
    rng = np.random.default_rng(12)
    n, b, T = 32, 8, 5
    eye = synth.f32_to_bf16_bits(np.eye(n, dtype=np.float32))
    diag = np.eye(n // b, dtype=np.uint8)
    pe = orc.pack(eye, b, diag)
    xb = synth.gauss_bf16(rng, (T, n), 1.0)
    x = f64(xb).T
    # identity weights: Y = bf16(silu(x) * x)
    Y = orc.mlp(pe, pe, pe, xb)
    ref = f64(synth.f32_to_bf16_bits((x / (1 + np.exp(-x)) * x).astype(np.float32)))
    assert np.array_equal(Y, ref)
    # zero gate or zero X => zero output
    zero = orc.pack(np.zeros((n, n), dtype=np.uint16), b, diag)
    assert not orc.mlp(zero, pe, pe, xb).any()
    assert not orc.mlp(pe, pe, pe, np.zeros_like(xb)).any()


def test_h_rounding_is_nearest_even():
    # identity MLP turns H = bf16(silu(x) * x) into the output, so the rounding is observable.
    # relu: H = bf16(x * x); choose x with x*x exactly half-way between two bf16 values.
    n, b = 8, 8
    eye = synth.f32_to_bf16_bits(np.eye(n, dtype=np.float32))
    pe = orc.pack(eye, b, np.ones((1, 1), dtype=np.uint8))
    # x = 1 + 2^-4 -> x^2 = 1 + 2^-3 + 2^-8 : tie between 1+2^-3 (even mantissa 0x10) and 1+2^-3+2^-7 -> even wins
    # x = 1 + 2^-4 + 2^-5 -> x^2 = 1 + 2^-3 + 2^-4 + 2^-8*(1 + 2 + ... ) computed exactly below
    xs = np.array([1 + 2 ** -4, 1 + 3 * 2 ** -5, 1.5, 1 + 2 ** -7], dtype=np.float32)
    xb = np.zeros((1, n), dtype=np.uint16)
    xb[0, :4] = synth.f32_to_bf16_bits(xs)
    Y = orc.mlp(pe, pe, pe, xb, activation="relu")[:, 0]
    for j, xv in enumerate(xs.tolist()):
        sq = Fraction(xv) ** 2
        ulp = Fraction(2) ** (math.floor(math.log2(sq)) - 7)
        lo = (sq // ulp) * ulp
        hi = lo + ulp
        if sq - lo < hi - sq:
            want = lo
        elif sq - lo > hi - sq:
            want = hi
        else:
            want = lo if (lo / ulp) % 2 == 0 else hi
        assert Fraction(Y[j]) == want, (j, xv)


# ---- two-matrix MLP  Y = W2 act(W1 X)  (Sec. 2.1, Sec. 3.4.3) ----

def _np_act(G, act):
    if act == "silu":
        return G / (1.0 + np.exp(-G))
    if act == "gelu":
        return 0.5 * G * (1.0 + np.vectorize(math.erf)(G / math.sqrt(2.0)))
    return np.maximum(G, 0.0)


@pytest.mark.parametrize("act", ["gelu", "relu", "silu"])
def test_mlp2_equals_numpy_dense_formula(act):
    rng = np.random.default_rng(21)
    E, I, b, T = 48, 96, 16, 7
    w1, w2 = (synth.gauss_bf16(rng, s, 0.25) for s in ((I, E), (E, I)))
    m1, m2 = (synth.uniform_mask(rng, *s, 0.5) for s in ((I // b, E // b), (E // b, I // b)))
    m1[2, :] = 0  # empty W1 row: act(0) = 0 for all three functions -> H rows zero
    xb = synth.gauss_bf16(rng, (T, E), 1.0)
    p1, p2 = orc.pack(w1, b, m1), orc.pack(w2, b, m2)
    Y, H = orc.mlp2(p1, p2, xb, activation=act, return_h=True)
    X = f64(xb).T
    G = (f64(w1) * expand(m1, b)) @ X
    Href = f64(synth.f32_to_bf16_bits(_np_act(G, act).astype(np.float32)))
    assert np.array_equal(f64(H), Href)
    np.testing.assert_allclose(Y, (f64(w2) * expand(m2, b)) @ Href, rtol=1e-12, atol=1e-15)
    assert not f64(H)[2 * b:3 * b].any()
    Y2 = orc.mlp2(p1, p2, np.ascontiguousarray(xb.T), layout="feature_major", activation=act)
    assert np.array_equal(Y, Y2)


def test_mlp2_special_cases():
    rng = np.random.default_rng(22)
    n, b, T = 32, 8, 5
    eye = synth.f32_to_bf16_bits(np.eye(n, dtype=np.float32))
    diag = np.eye(n // b, dtype=np.uint8)
    pe = orc.pack(eye, b, diag)
    xb = synth.gauss_bf16(rng, (T, n), 1.0)
    x = f64(xb).T
    # identity weights, relu: Y = max(x, 0) exactly (bf16 in, bf16 out)
    assert np.array_equal(orc.mlp2(pe, pe, xb, activation="relu"), np.maximum(x, 0.0))
    # W1 = -identity, relu, x >= 0  ->  zero
    neg = orc.pack(synth.f32_to_bf16_bits(-np.eye(n, dtype=np.float32)), b, diag)
    xpos = synth.f32_to_bf16_bits(np.abs(x.T).astype(np.float32))
    assert not orc.mlp2(neg, pe, xpos, activation="relu").any()
    # gelu is odd up to x:  gelu(x) - gelu(-x) = x;  with identity weights the two outputs differ by x within bf16 rounding
    yp = orc.mlp2(pe, pe, xb, activation="gelu")
    yn = orc.mlp2(neg, pe, xb, activation="gelu")
    assert np.max(np.abs((yp - yn) - x)) <= 2.0 ** -8 * np.max(np.abs(x)) * 2
    # the second matrix is linear: scaling W2 by 2 doubles Y exactly, a permutation W2 permutes rows of H
    two = orc.pack(synth.f32_to_bf16_bits(2 * np.eye(n, dtype=np.float32)), b, diag)
    assert np.array_equal(orc.mlp2(pe, two, xb, activation="silu"), 2 * orc.mlp2(pe, pe, xb, activation="silu"))
    perm = rng.permutation(n)
    P = np.zeros((n, n), dtype=np.float32)
    P[np.arange(n), perm] = 1
    pp = orc.pack(synth.f32_to_bf16_bits(P), b, np.ones((n // b, n // b), dtype=np.uint8))
    Yh, H = orc.mlp2(pe, pp, xb, activation="silu", return_h=True)
    assert np.array_equal(Yh, f64(H)[perm])
    # zero input -> zero output (act(0) = 0)
    assert not orc.mlp2(pe, pe, np.zeros_like(xb)).any()


def test_mlp2_is_the_gated_mlp_with_a_constant_up_projection():
    # The three-matrix form with U == 1 everywhere reduces to the two-matrix form.  Make W_up X = 1 by
    # appending a constant-one feature to X and giving W_up a single 1 in that column of every row.
    rng = np.random.default_rng(23)
    E, I, b, T = 32, 64, 8, 6
    w1 = synth.gauss_bf16(rng, (I, E), 0.3)
    w1f = f64(w1)
    w1f[:, E - b:] = 0  # last block column unused by W1, so the constant feature does not leak into G
    w1 = synth.f32_to_bf16_bits(w1f.astype(np.float32))
    w2 = synth.gauss_bf16(rng, (E, I), 0.3)
    up = np.zeros((I, E), dtype=np.float32)
    up[:, E - 1] = 1.0
    xf = f64(synth.gauss_bf16(rng, (T, E), 1.0))
    xf[:, E - 1] = 1.0
    xb = synth.f32_to_bf16_bits(xf.astype(np.float32))
    full = lambda r, c: np.ones((r // b, c // b), dtype=np.uint8)
    p1, pu, p2 = orc.pack(w1, b, full(I, E)), orc.pack(synth.f32_to_bf16_bits(up), b, full(I, E)), orc.pack(w2, b, full(E, I))
    for act in ("silu", "gelu", "relu"):
        assert np.array_equal(orc.mlp2(p1, p2, xb, activation=act), orc.mlp(p1, pu, p2, xb, activation=act))


# ---- backward pass on the pruned weight (Sec. 3.2, Sec. 3.4): dX = W~^T dY, dW~ = (dY X^T) on kept blocks ----

def _int_bf16(rng, shape, lo=-4, hi=5):
    """Small integers as bf16 bits: every product and sum below stays exact in fp64 (and in fp32)."""
    return synth.f32_to_bf16_bits(rng.integers(lo, hi, size=shape).astype(np.float32))


def test_spmm_t_equals_numpy_and_the_forward_product_of_the_transpose():
    rng = np.random.default_rng(31)
    M, K, b, T = 96, 64, 16, 9
    W = synth.gauss_bf16(rng, (M, K), 0.3)
    mask = synth.uniform_mask(rng, M // b, K // b, 0.5)
    mask[2, :] = 0  # empty block row
    mask[:, 1] = 0  # empty block column -> zero rows of dX
    p = orc.pack(W, b, mask)
    dY = synth.gauss_bf16(rng, (T, M), 1.0)
    dX = orc.spmm_t(p, dY)
    ref = (f64(W) * expand(mask, b)).T @ f64(dY).T
    np.testing.assert_allclose(dX, ref, rtol=1e-12, atol=1e-14)
    assert not dX[b:2 * b].any()
    # feature-major dY, same numbers
    assert np.array_equal(dX, orc.spmm_t(p, np.ascontiguousarray(dY.T), layout="feature_major"))
    # the forward product of the packed transpose (summation order is the same: ascending row of W)
    pt = orc.pack(np.ascontiguousarray(W.T), b, np.ascontiguousarray(mask.T))
    assert np.array_equal(dX, orc.spmm(pt, dY))


def test_spmm_t_is_the_adjoint_of_spmm_exactly():
    # <dY, W X> == <W^T dY, X> for any dY, X; with small-integer data both sides are exact integers
    rng = np.random.default_rng(32)
    M, K, b, T = 64, 96, 32, 5
    W = _int_bf16(rng, (M, K))
    mask = synth.uniform_mask(rng, M // b, K // b, 0.4)
    p = orc.pack(W, b, mask)
    X, dY = _int_bf16(rng, (T, K)), _int_bf16(rng, (T, M))
    lhs = float((f64(dY).T * orc.spmm(p, X)).sum())
    rhs = float((orc.spmm_t(p, dY) * f64(X).T).sum())
    assert lhs == rhs and lhs == round(lhs)


def test_sddmm_equals_numpy_on_kept_blocks():
    rng = np.random.default_rng(33)
    M, K, b, T = 64, 96, 16, 11
    W = synth.gauss_bf16(rng, (M, K), 0.3)
    mask = synth.uniform_mask(rng, M // b, K // b, 0.6)
    mask[1, :] = 0
    p = orc.pack(W, b, mask)
    X, dY = synth.gauss_bf16(rng, (T, K), 1.0), synth.gauss_bf16(rng, (T, M), 1.0)
    dv = orc.sddmm(p, dY, X)
    full = f64(dY).T @ f64(X)  # [M, K] = dY X^T in the (feature, token) convention
    assert dv.shape == (p.nnz, b, b)
    q = 0
    for r in range(M // b):
        for c in range(K // b):
            if mask[r, c]:
                assert p.col_idx[q] == c and p.row_ptr[r] <= q < p.row_ptr[r + 1]
                np.testing.assert_allclose(dv[q], full[r * b:(r + 1) * b, c * b:(c + 1) * b], rtol=1e-12, atol=1e-14)
                q += 1
    assert q == p.nnz
    dv2 = orc.sddmm(p, np.ascontiguousarray(dY.T), np.ascontiguousarray(X.T), layout="feature_major")
    assert np.array_equal(dv, dv2)


def test_sddmm_is_the_exact_derivative_of_the_linear_loss():
    # L(W~) = <dY, W~ X> is linear in every stored weight: bumping one stored entry by 1 changes L by exactly
    # its gradient entry.  Integer data keeps everything exact.  Also: a rank-one case with a closed form.
    rng = np.random.default_rng(34)
    M, K, b, T = 32, 48, 16, 4
    W = _int_bf16(rng, (M, K))
    mask = synth.uniform_mask(rng, M // b, K // b, 0.5)
    p = orc.pack(W, b, mask)
    X, dY = _int_bf16(rng, (T, K)), _int_bf16(rng, (T, M))
    dv = orc.sddmm(p, dY, X)
    L0 = float((f64(dY).T * orc.spmm(p, X)).sum())
    rr, cc = np.nonzero(mask)
    for q, i, j in [(0, 0, 0), (p.nnz - 1, b - 1, b - 1), (p.nnz // 2, 3, 7), (1, 15, 2)]:
        Wf = f64(W).copy()
        Wf[rr[q] * b + i, cc[q] * b + j] += 1.0
        p1 = orc.pack(synth.f32_to_bf16_bits(Wf.astype(np.float32)), b, mask)
        L1 = float((f64(dY).T * orc.spmm(p1, X)).sum())
        assert L1 - L0 == dv[q, i, j], (q, i, j)
    # one token: dW = dy x^T (outer product) on kept blocks
    x1, dy1 = _int_bf16(rng, (1, K)), _int_bf16(rng, (1, M))
    dv1 = orc.sddmm(p, dy1, x1)
    outer = np.outer(f64(dy1)[0], f64(x1)[0])
    for q in range(p.nnz):
        assert np.array_equal(dv1[q], outer[rr[q] * b:(rr[q] + 1) * b, cc[q] * b:(cc[q] + 1) * b])


@pytest.mark.parametrize("M,K,b,T,seed", [(8, 8, 4, 3, 1), (8, 12, 4, 2, 2)])
def test_backward_brute_force_exact(M, K, b, T, seed):
    # exact rational arithmetic, plain Python loops, tiny sizes
    rng = np.random.default_rng(40 + seed)
    W = synth.gauss_bf16(rng, (M, K), 1.0)
    mask = synth.uniform_mask(rng, M // b, K // b, 0.5)
    p = orc.pack(W, b, mask)
    X, dY = synth.gauss_bf16(rng, (T, K), 1.0), synth.gauss_bf16(rng, (T, M), 1.0)
    Wi = [[Fraction(float(v)) for v in row] for row in f64(W)]
    Xi = [[Fraction(float(v)) for v in row] for row in f64(X)]
    Yi = [[Fraction(float(v)) for v in row] for row in f64(dY)]
    dX = orc.spmm_t(p, dY)
    for k in range(K):
        for t in range(T):
            s = sum((Wi[i][k] * Yi[t][i] for i in range(M) if mask[i // b, k // b]), Fraction(0))
            assert abs(Fraction(float(dX[k, t])) - s) <= abs(s) * Fraction(1, 2 ** 45) + Fraction(1, 2 ** 60)
    dv = orc.sddmm(p, dY, X)
    rr, cc = np.nonzero(mask)
    for q in range(p.nnz):
        for i in range(b):
            for j in range(b):
                s = sum((Yi[t][rr[q] * b + i] * Xi[t][cc[q] * b + j] for t in range(T)), Fraction(0))
                assert abs(Fraction(float(dv[q, i, j])) - s) <= abs(s) * Fraction(1, 2 ** 45) + Fraction(1, 2 ** 60)


# ---- blocked prune-and-grow mask update and the sparsity schedule (Sec. 3.2, Eq. (2)) ----

def test_generate_masks_is_union_of_the_two_selections():
    rng = np.random.default_rng(51)
    M, K, b, s = 128, 96, 16, 0.75
    W, G = synth.gauss_bf16(rng, (M, K), 1.0), synth.gauss_bf16(rng, (M, K), 1.0)
    m = orc.generate_masks(W, G, b, s)
    mw, _ = orc.topk_mask(orc.block_scores(W, b), s)
    mg, _ = orc.topk_mask(orc.block_scores(G, b), s)
    n_keep = orc.n_keep(mw.size, s)
    assert np.array_equal(m == 1, mw.reshape(m.shape).astype(bool))
    assert np.array_equal(m == 2, (mg.reshape(m.shape) == 1) & (mw.reshape(m.shape) == 0))  # the set difference
    assert np.array_equal(m != 0, (mw | mg).reshape(m.shape).astype(bool))
    assert int((m == 1).sum()) == n_keep and n_keep <= int((m != 0).sum()) <= 2 * n_keep
    # independent numpy ranking: stable argsort of (-score, index)
    def np_topk(A):
        sc = (f64(A).reshape(M // b, b, K // b, b) ** 2).sum(axis=(1, 3)).ravel()
        keep = np.argsort(-sc, kind="stable")[:n_keep]
        out = np.zeros(sc.size, dtype=bool)
        out[keep] = True
        return out.reshape(M // b, K // b)
    assert np.array_equal(m == 1, np_topk(W)) and np.array_equal(m != 0, np_topk(W) | np_topk(G))


def test_generate_masks_special_cases():
    rng = np.random.default_rng(52)
    M, K, b, s = 64, 64, 16, 0.5
    W = synth.gauss_bf16(rng, (M, K), 1.0)
    # gradient ranks like the weight: nothing to regrow
    assert not (orc.generate_masks(W, W, b, s) == 2).any()
    # gradient mass only on the blocks the weight drops: exactly those come back (n_keep of them at s = 0.5)
    mw, _ = orc.topk_mask(orc.block_scores(W, b), s)
    mw = mw.reshape(M // b, K // b)
    Gf = np.kron(1 - mw, np.ones((b, b))) * (1.0 + np.arange(M * K).reshape(M, K) % 7)
    m = orc.generate_masks(W, synth.f32_to_bf16_bits(Gf.astype(np.float32)), b, s)
    assert np.array_equal(m == 2, mw == 0) and (m != 0).all()
    # s = 0: everything kept by the weight itself; s = 1: nothing survives and nothing regrows
    assert (orc.generate_masks(W, W, b, 0.0) == 1).all()
    assert not orc.generate_masks(W, synth.gauss_bf16(rng, (M, K), 1.0), b, 1.0).any()
    # packing a regrown block stores zeros (they must not change the current transform)
    m2 = np.zeros((M // b, K // b), dtype=np.uint8)
    m2[0, 1], m2[2, 3] = 1, 2
    p = orc.pack(W, b, m2)
    assert p.nnz == 2 and np.array_equal(p.vals[0], W[:b, b:2 * b]) and not p.vals[1].any()
    x = synth.gauss_bf16(rng, (3, K), 1.0)
    m1 = m2.copy()
    m1[2, 3] = 0
    assert np.array_equal(orc.spmm(p, x), orc.spmm(orc.pack(W, b, m1), x))


def test_sparsity_schedule_closed_forms():
    # Eq. (2): s(0) = s_init, s(m - d) = s_max, halfway the cube leaves an eighth of the distance
    m, d, s0, s1 = 9000, 1000, 0.1, 0.8
    assert orc.sparsity_schedule(0, m, d, s0, s1) == pytest.approx(s0, abs=1e-15)
    assert orc.sparsity_schedule(m - d, m, d, s0, s1) == s1
    assert orc.sparsity_schedule((m - d) // 2, m, d, s0, s1) == pytest.approx(s1 + (s0 - s1) / 8, abs=1e-15)
    assert orc.sparsity_schedule(2000, m, d, s0, s1) == pytest.approx(s1 + (s0 - s1) * Fraction(3, 4) ** 3, abs=1e-15)
    vals = [orc.sparsity_schedule(i, m, d, s0, s1) for i in range(0, m + 1, 250)]
    assert all(a <= b_ + 1e-15 for a, b_ in zip(vals, vals[1:]))  # sparsity never decreases
    assert all(s0 - 1e-15 <= v <= s1 + 1e-15 for v in vals)
    # held at the ends: the cube is not followed past i = m - d
    assert orc.sparsity_schedule(m, m, d, s0, s1) == s1 and orc.sparsity_schedule(-5, m, d, s0, s1) == pytest.approx(s0)


# ---- block scores by 2D average pooling of a sensitivity matrix (Sec. 3.3) ----

def test_pooled_scores_equal_numpy_mean_and_frobenius_ranking():
    rng = np.random.default_rng(61)
    M, K, b = 96, 64, 16
    S = rng.standard_normal((M, K)).astype(np.float32)  # sensitivities of either sign
    sc = orc.pooled_scores(S, b)
    ref = S.astype(np.float64).reshape(M // b, b, K // b, b).mean(axis=(1, 3))
    np.testing.assert_allclose(sc, ref, rtol=1e-13, atol=1e-16)
    # a constant block pools to the constant; a one-hot block to 1 / b^2
    S2 = np.zeros((2 * b, 2 * b), dtype=np.float32)
    S2[:b, :b] = -3.5
    S2[b + 3, b + 5] = 1.0
    sc2 = orc.pooled_scores(S2, b)
    assert sc2[0, 0] == -3.5 and sc2[1, 1] == 1.0 / (b * b) and sc2[0, 1] == 0.0 and sc2[1, 0] == 0.0
    # pooling the squared weights ranks exactly like the Frobenius norm: same mask
    W = synth.gauss_bf16(rng, (M, K), 1.0)
    Wsq = (f64(W) ** 2).astype(np.float32)  # bf16 squared is exact in fp32
    for s in (0.25, 0.5, 0.9):
        m_pool, _ = orc.pooled_topk_mask(Wsq, b, s)
        m_fro, _ = orc.topk_mask(orc.block_scores(W, b), s)
        assert np.array_equal(m_pool, m_fro.reshape(m_pool.shape))


def test_pooled_topk_mask_ranking_and_ties():
    rng = np.random.default_rng(62)
    M, K, b, s = 64, 64, 8, 0.6
    S = rng.standard_normal((M, K)).astype(np.float32)
    m, gap = orc.pooled_topk_mask(S, b, s)
    n = (M // b) * (K // b)
    n_keep = orc.n_keep(n, s)
    ref = S.astype(np.float64).reshape(M // b, b, K // b, b).mean(axis=(1, 3)).ravel()
    keep = np.argsort(-ref, kind="stable")[:n_keep]
    want = np.zeros(n, dtype=np.uint8)
    want[keep] = 1
    assert np.array_equal(m.ravel(), want) and int(m.sum()) == n_keep and gap > 0
    # all blocks equal: the lowest indices survive
    m_eq, gap_eq = orc.pooled_topk_mask(np.full((M, K), -1.25, dtype=np.float32), b, s)
    assert np.array_equal(np.nonzero(m_eq.ravel())[0], np.arange(n_keep)) and gap_eq == 0.0


# ---- E5M2 (the 8-bit floating-point type of Sec. 5.2) ----

def test_e5m2_known_codes_and_roundtrip():
    dec = orc.e5m2_decode(np.arange(256, dtype=np.uint8))
    # format facts: bias 15, 2 mantissa bits, IEEE-style subnormals / inf / nan
    table = {0x00: 0.0, 0x01: 2.0 ** -16, 0x03: 3 * 2.0 ** -16, 0x04: 2.0 ** -14, 0x38: 0.5, 0x3C: 1.0, 0x3D: 1.25,
             0x3E: 1.5, 0x3F: 1.75, 0x40: 2.0, 0xC0: -2.0, 0x7B: 57344.0, 0xFB: -57344.0}
    for code, val in table.items():
        assert dec[code] == val, hex(code)
    assert np.isinf(dec[0x7C]) and dec[0x7C] > 0 and np.isinf(dec[0xFC]) and dec[0xFC] < 0 and np.isnan(dec[0x7D])
    # E5M2 is the upper byte of IEEE half precision
    half = (np.arange(256, dtype=np.uint16) << 8).view(np.float16).astype(np.float64)
    fin = np.isfinite(half)
    assert np.array_equal(dec[fin], half[fin])
    # every finite code encodes to itself; positive codes are strictly increasing
    fin_codes = np.nonzero(np.isfinite(dec))[0].astype(np.uint8)
    assert np.array_equal(orc.e5m2_quantize(dec[fin_codes].astype(np.float32)), fin_codes)
    assert np.all(np.diff(dec[:0x7C]) > 0)


def test_e5m2_rounding_is_nearest_even_against_enumeration():
    dec = orc.e5m2_decode(np.arange(256, dtype=np.uint8))
    pos = [(Fraction(float(dec[c])), c) for c in range(0x7C)]  # finite non-negative codes, ascending
    rng = np.random.default_rng(71)
    xs = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(0.02),       # weights: deep in the subnormal range too
        rng.standard_normal(2000).astype(np.float32),
        (rng.standard_normal(500) * 2e4).astype(np.float32),
        np.array([1.125, 1.375, 1.625, 1.875, 2.0 ** -17, 3 * 2.0 ** -17, 5 * 2.0 ** -17, 7 * 2.0 ** -17,  # exact ties
                  2.0 ** -18, 61439.0, 57344.0, 59392.0, 0.0, -0.0], dtype=np.float32)])
    got = orc.e5m2_quantize(xs)
    for x, g in zip(xs.tolist(), got.tolist()):
        a = abs(Fraction(x))
        sign = 0x80 if math.copysign(1.0, x) < 0 else 0
        # nearest representable magnitude by exhaustive search; ties -> even mantissa (even code)
        best = min(pos, key=lambda vc: (abs(vc[0] - a), vc[1] & 1))
        if a >= Fraction(61440):   # halfway between the largest finite value and 2^16: rounds to infinity
            want = sign | 0x7C
        else:
            want = sign | best[1]
        assert g == want, (x, hex(g), hex(want))
    # the listed ties, spelled out
    assert orc.e5m2_quantize(np.array([1.125, 1.375, 2.0 ** -17, 3 * 2.0 ** -17], dtype=np.float32)).tolist() == [0x3C, 0x3E, 0x00, 0x02]
    assert orc.e5m2_quantize(np.array([61439.0, 61440.0, 1e9], dtype=np.float32)).tolist() == [0x7B, 0x7C, 0x7C]


def test_spmm_e5m2_equals_numpy_on_decoded_values():
    rng = np.random.default_rng(72)
    M, K, b, T = 64, 96, 16, 7
    W = synth.gauss_bf16(rng, (M, K), 0.3)
    mask = synth.uniform_mask(rng, M // b, K // b, 0.5)
    mask[1, :] = 0
    p = orc.pack(W, b, mask)
    vals8 = orc.e5m2_quantize(f64(p.vals).astype(np.float32))
    X8 = orc.e5m2_quantize(rng.standard_normal((T, K)).astype(np.float32))
    Y = orc.spmm_e5m2(p, vals8, X8)
    # dense reference from decoded values scattered by the index arrays
    Wd = np.zeros((M, K))
    rr = np.repeat(np.arange(M // b), np.diff(p.row_ptr))
    for q in range(p.nnz):
        Wd[rr[q] * b:(rr[q] + 1) * b, p.col_idx[q] * b:(p.col_idx[q] + 1) * b] = orc.e5m2_decode(vals8[q])
    np.testing.assert_allclose(Y, Wd @ orc.e5m2_decode(X8).T, rtol=1e-12, atol=1e-15)
    assert not Y[b:2 * b].any()
    assert np.array_equal(Y, orc.spmm_e5m2(p, vals8, np.ascontiguousarray(X8.T), layout="feature_major"))
    # values that are exact in E5M2 (small powers of two and their multiples): same numbers as the bf16 product
    Wp = synth.f32_to_bf16_bits(rng.choice([-2.0, -1.0, -0.5, 0.0, 0.5, 1.0, 1.5], size=(M, K)).astype(np.float32))
    Xp = rng.choice([-1.0, 0.25, 0.5, 1.0, 3.0], size=(T, K)).astype(np.float32)
    pp = orc.pack(Wp, b, mask)
    assert np.array_equal(orc.spmm_e5m2(pp, orc.e5m2_quantize(f64(pp.vals).astype(np.float32)), orc.e5m2_quantize(Xp)),
                          orc.spmm(pp, synth.f32_to_bf16_bits(Xp)))


def _dense_from_codes(p, vals8):
    """Dense masked matrix from E5M2 codes, decoded through numpy's float16 (a code is the upper byte of a half)."""
    b = p.b
    Wd = np.zeros((p.rows, p.cols))
    rr = np.repeat(np.arange(p.rows // b), np.diff(p.row_ptr))
    for q in range(p.nnz):
        blk = (vals8[q].astype(np.uint16) << 8).view(np.float16).astype(np.float64)
        Wd[rr[q] * b:(rr[q] + 1) * b, p.col_idx[q] * b:(p.col_idx[q] + 1) * b] = blk
    return Wd


def test_e5m2_weight_product_and_mlp_equal_numpy_on_decoded_weights():
    """Weights in E5M2, activations and the intermediate in bf16 (the decode form of the 8-bit run of Sec. 5.2):
    the product against numpy on weights decoded independently (float16 view), the MLP against the dense
    formula with a bit-equal intermediate, and against the bf16 MLP when the weights are exact in E5M2."""
    rng = np.random.default_rng(73)
    E, I, b, T = 64, 96, 16, 5
    Ws = [synth.gauss_bf16(rng, s, 0.3) for s in ((I, E), (I, E), (E, I))]
    ms = [synth.uniform_mask(rng, r // b, c // b, 0.5) for r, c in ((I, E), (I, E), (E, I))]
    ms[0][1, :] = 0
    ps = [orc.pack(w, b, m) for w, m in zip(Ws, ms)]
    v8 = [orc.e5m2_quantize(f64(p.vals).astype(np.float32)) for p in ps]
    X = synth.gauss_bf16(rng, (T, E), 1.0)
    Xf = f64(X)
    # single product
    Y = orc.spmm_e5m2w(ps[0], v8[0], X)
    np.testing.assert_allclose(Y, _dense_from_codes(ps[0], v8[0]) @ Xf.T, rtol=1e-12, atol=1e-15)
    assert not Y[b:2 * b].any()
    assert np.array_equal(Y, orc.spmm_e5m2w(ps[0], v8[0], np.ascontiguousarray(X.T), layout="feature_major"))
    # quantisation moved the weights: the 8-bit product differs from the 16-bit one, by about a mantissa step
    Y16 = orc.spmm(ps[0], X)
    rel = np.linalg.norm(Y - Y16) / np.linalg.norm(Y16)
    assert 1e-3 < rel < 0.15
    # MLP: dense formula on the decoded weights, intermediate rounded once to bf16
    Wg, Wu, Wd = (_dense_from_codes(p, v) for p, v in zip(ps, v8))
    G, U = Wg @ Xf.T, Wu @ Xf.T
    h = (G / (1.0 + np.exp(-G)) * U).astype(np.float32)
    Hb = synth.f32_to_bf16_bits(h)
    Yw, H = orc.mlp_e5m2w(ps[0], v8[0], ps[1], v8[1], ps[2], v8[2], X, return_h=True)
    assert np.array_equal(H, Hb)
    np.testing.assert_allclose(Yw, Wd @ f64(Hb), rtol=1e-12, atol=1e-15)
    assert not f64(H[b:2 * b]).any()  # an empty gate row: zeros (of either sign)
    # weights that are exact in E5M2: the same numbers as the bf16 MLP, bit for bit
    Wx = [synth.f32_to_bf16_bits(rng.choice([-1.0, -0.5, 0.0, 0.25, 0.5, 1.5], size=w.shape).astype(np.float32)) for w in Ws]
    px = [orc.pack(w, b, m) for w, m in zip(Wx, ms)]
    vx = [orc.e5m2_quantize(f64(p.vals).astype(np.float32)) for p in px]
    assert np.array_equal(orc.mlp_e5m2w(px[0], vx[0], px[1], vx[1], px[2], vx[2], X), orc.mlp(px[0], px[1], px[2], X))
    for act in ("gelu", "relu"):
        assert np.array_equal(orc.mlp_e5m2w(px[0], vx[0], px[1], vx[1], px[2], vx[2], X, activation=act),
                              orc.mlp(px[0], px[1], px[2], X, activation=act))
