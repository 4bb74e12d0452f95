"""Pins for the CPU oracle: every function of oracle/ is checked against something other
than itself -- a library routine on a special case, exact brute force, closed forms,
invariants, and the structure of the paper's worked example."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp
import torch

from paper_1802_10280_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _int_layer(rng, N, C, H, W, M, R, S, density=0.4, lo=-3, hi=4):
    x = rng.integers(0, 5, size=(N, C, H, W)).astype(np.float32)
    w = rng.integers(lo, hi, size=(M, C, R, S)).astype(np.float32)
    w *= rng.random((M, C, R, S)) < density
    return x, w


def _csr(w):
    return wl.dense_to_csr(w)


def _torch_conv(x, w, stride, pad, bias=None):
    y = torch.nn.functional.conv2d(torch.from_numpy(np.asarray(x, dtype=np.float64)),
                                   torch.from_numpy(np.asarray(w, dtype=np.float64)),
                                   bias=None if bias is None else torch.from_numpy(
                                       np.asarray(bias, dtype=np.float64)),
                                   stride=stride, padding=pad)
    return y.numpy()


# ---------------------------------------------------------------- Eq. (1), dense special case
@pytest.mark.parametrize("R,stride,pad,H,W", [(3, 1, 1, 9, 11), (3, 1, 0, 8, 8), (5, 1, 2, 9, 7),
                                              (1, 1, 0, 6, 5), (3, 2, 1, 10, 12), (3, 2, 0, 9, 9),
                                              (5, 2, 2, 11, 8), (3, 3, 1, 10, 7)])
def test_dense_case_matches_library_conv2d(oracle, R, stride, pad, H, W):
    """0 % sparsity is plain dense convolution: compare with torch's conv2d in fp64."""
    rng = np.random.default_rng(11 + R + stride)
    N, C, M = 2, 5, 4
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((M, C, R, R)).astype(np.float32)
    rowptr, colidx, value = _csr(w)
    assert rowptr[-1] == w.size                      # really dense
    Wd = oracle.csr_to_dense(M, C, R, R, rowptr, colidx, value)
    np.testing.assert_array_equal(Wd, w.astype(np.float64))
    out, bound = oracle.conv(x, Wd, stride, pad)
    ref = _torch_conv(x, w, stride, pad)
    assert out.shape == ref.shape
    np.testing.assert_allclose(out, ref, rtol=0, atol=2e-6 * np.abs(ref).max() + 1e-6)
    # B = sum |w*x| is the same convolution on absolute values
    refb = _torch_conv(np.abs(x), np.abs(w), stride, pad)
    np.testing.assert_allclose(bound, refb, rtol=1e-12, atol=1e-12)


def test_sparse_case_matches_library_conv2d(oracle):
    L = wl.custom_layer(2, 7, 10, 9, 6, 3, 3, 1, 1, 0.8, seed=5)
    Wd = oracle.csr_to_dense(6, 7, 3, 3, L.rowptr, L.colidx, L.value)
    out, _ = oracle.conv(L.input, Wd, 1, 1)
    ref = _torch_conv(L.input, L.weight, 1, 1)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-6)


# ---------------------------------------------------------------- exact brute force, tiny
@pytest.mark.parametrize("R,S,stride,pad", [(3, 3, 1, 1), (2, 3, 1, 0), (3, 3, 2, 1), (1, 1, 1, 0),
                                            (3, 2, 2, 2)])
def test_brute_force_exact_on_small_integers(oracle, R, S, stride, pad):
    """Every output by an explicit sum over (c, r, s) in exact rational arithmetic."""
    rng = np.random.default_rng(100 + R * 7 + S + stride)
    N, C, H, W, M = 2, 3, 5, 4, 3
    x, w = _int_layer(rng, N, C, H, W, M, R, S)
    rowptr, colidx, value = _csr(w)
    Wd = oracle.csr_to_dense(M, C, R, S, rowptr, colidx, value)
    out, bound = oracle.conv(x, Wd, stride, pad)
    E = (H + 2 * pad - R) // stride + 1
    F = (W + 2 * pad - S) // stride + 1
    assert out.shape == (N, M, E, F)

    def I(n, c, y, xx):
        return Fraction(int(x[n, c, y, xx])) if 0 <= y < H and 0 <= xx < W else Fraction(0)

    for n, m, h, ww in itertools.product(range(N), range(M), range(E), range(F)):
        terms = [I(n, c, h * stride + r - pad, ww * stride + s - pad) * Fraction(int(w[m, c, r, s]))
                 for c in range(C) for r in range(R) for s in range(S)]
        assert Fraction(float(out[n, m, h, ww])) == sum(terms)
        assert Fraction(float(bound[n, m, h, ww])) == sum(abs(t) for t in terms)


# ---------------------------------------------------------------- identity and shifts
def test_single_centre_weight_reproduces_input(oracle):
    rng = np.random.default_rng(3)
    N, C, H, W, M = 2, 4, 7, 6, 3
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = np.zeros((M, C, 3, 3), dtype=np.float32)
    for m in range(M):
        w[m, (m + 1) % C, 1, 1] = 1.0
    Wd = oracle.csr_to_dense(M, C, 3, 3, *_csr(w))
    out, _ = oracle.conv(x, Wd, 1, 1)
    for m in range(M):
        np.testing.assert_array_equal(out[:, m], x[:, (m + 1) % C])


@pytest.mark.parametrize("r,s", list(itertools.product(range(3), range(3))))
def test_single_weight_is_a_shift_with_zero_fill(oracle, r, s):
    """A single weight 1 at (r, s): out[h][w] = in[h + r - pad][w + s - pad], zero outside.
    Pins cross-correlation (no flip) and which side the padding sits on."""
    rng = np.random.default_rng(17)
    H, W, pad = 6, 5, 1
    x = rng.standard_normal((1, 1, H, W)).astype(np.float32)
    w = np.zeros((1, 1, 3, 3), dtype=np.float32)
    w[0, 0, r, s] = 1.0
    out, _ = oracle.conv(x, oracle.csr_to_dense(1, 1, 3, 3, *_csr(w)), 1, pad)
    exp = np.zeros((H, W), dtype=np.float32)
    for h in range(H):
        for ww in range(W):
            y, xx = h + r - pad, ww + s - pad
            if 0 <= y < H and 0 <= xx < W:
                exp[h, ww] = x[0, 0, y, xx]
    np.testing.assert_array_equal(out[0, 0], exp)


# ---------------------------------------------------------------- 1x1 == CSR SpMM
def test_1x1_equals_csr_spmm(oracle):
    L = wl.custom_layer(3, 24, 6, 7, 10, 1, 1, 1, 0, 0.7, seed=9, dist="normal")
    A = sp.csr_matrix((L.value.astype(np.float64), L.colidx, L.rowptr), shape=(10, 24))
    Wd = oracle.csr_to_dense(10, 24, 1, 1, L.rowptr, L.colidx, L.value)
    out, _ = oracle.conv(L.input, Wd, 1, 0)
    for n in range(3):
        ref = A @ L.input[n].reshape(24, -1).astype(np.float64)
        np.testing.assert_allclose(out[n].reshape(10, -1), ref, rtol=0, atol=1e-6)
    # stretching a 1x1 / pad 0 column index gives c*H*W
    np.testing.assert_array_equal(oracle.stretch(24, 6, 7, 1, 1, 0, L.colidx), L.colidx * 42)


# ---------------------------------------------------------------- Alg. 1 == Alg. 2
@pytest.mark.parametrize("R,stride,pad", [(3, 1, 1), (3, 2, 1), (5, 1, 2), (1, 1, 0), (3, 1, 0),
                                          (5, 2, 1)])
def test_algorithm2_on_stretched_padded_equals_definition(oracle, R, stride, pad):
    L = wl.custom_layer(2, 6, 9, 8, 5, R, R, stride, pad, 0.75, seed=21 + R)
    s = L.spec
    Wd = oracle.csr_to_dense(s.M, s.C, R, R, L.rowptr, L.colidx, L.value)
    out1, bound = oracle.conv(L.input, Wd, stride, pad)
    st = oracle.stretch(s.C, s.H, s.W, R, R, pad, L.colidx)
    P = oracle.pad_input(L.input, pad)
    out2 = oracle.sconv_alg2((s.N, s.C, s.H, s.W, s.M, R, R, stride, pad), L.rowptr, st, L.value, P)
    assert out1.shape == out2.shape == (s.N, s.M, s.E, s.F)
    assert np.all(np.abs(out1.astype(np.float64) - out2) <= 1e-7 * bound + 1e-12)


def test_algorithm2_exact_on_small_integers_and_duplicates(oracle):
    """Duplicated CSR entries add up (Alg. 2's '+='); any order inside a row is accepted."""
    rng = np.random.default_rng(8)
    x, w = _int_layer(rng, 1, 2, 5, 5, 2, 3, 3)
    rowptr, colidx, value = _csr(w)
    # append to row 1 a duplicate of its first entry, then reverse the row's order
    j0, j1 = rowptr[1], rowptr[2]
    colidx2 = np.concatenate([colidx[:j1], colidx[j0:j0 + 1]])
    value2 = np.concatenate([value[:j1], np.float32([2.0])])
    rowptr2 = rowptr.copy()
    rowptr2[2] += 1
    colidx2[j0:] = colidx2[j0:][::-1].copy()
    value2[j0:] = value2[j0:][::-1].copy()
    w2 = w.copy().reshape(2, -1)
    w2[1, colidx[j0]] += 2.0
    w2 = w2.reshape(w.shape)
    Wd = oracle.csr_to_dense(2, 2, 3, 3, rowptr2, colidx2, value2)
    np.testing.assert_array_equal(Wd, w2.astype(np.float64))
    ref = _torch_conv(x, w2, 1, 1)
    out, _ = oracle.conv(x, Wd, 1, 1)
    np.testing.assert_array_equal(out, ref.astype(np.float32))
    st = oracle.stretch(2, 5, 5, 3, 3, 1, colidx2)
    out2 = oracle.sconv_alg2((1, 2, 5, 5, 2, 3, 3, 1, 1), rowptr2, st, value2,
                             oracle.pad_input(x, 1))
    np.testing.assert_array_equal(out2, ref.astype(np.float32))


# ---------------------------------------------------------------- worked example structure
def test_fig5_superposition_structure(oracle):
    """Section 3.2's example: a 3x3 filter with nonzeros 2 and 3 on a 6x6 one-channel input is
    2 x one shifted 4x4 sub-matrix plus 3 x another (exact on small integers)."""
    cfg = {}
    for line in open(os.path.join(GOLDEN, "fig5_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        cfg[k] = [int(t) for t in v]
    H, W, R, S = cfg["H"][0], cfg["W"][0], cfg["R"][0], cfg["S"][0]
    E, F = cfg["E"][0], cfg["F"][0]
    w2, w3 = cfg["weights"]
    rng = np.random.default_rng(55)
    x = rng.integers(0, 10, size=(1, 1, H, W)).astype(np.float32)
    taps = list(itertools.product(range(R), range(S)))
    for (r1, s1), (r2, s2) in itertools.permutations(taps, 2):
        w = np.zeros((1, 1, R, S), dtype=np.float32)
        w[0, 0, r1, s1] = w2
        w[0, 0, r2, s2] = w3
        out, _ = oracle.conv(x, oracle.csr_to_dense(1, 1, R, S, *_csr(w)), 1, 0)
        assert out.shape == (1, 1, E, F)
        exp = w2 * x[0, 0, r1:r1 + E, s1:s1 + F] + w3 * x[0, 0, r2:r2 + E, s2:s2 + F]
        np.testing.assert_array_equal(out[0, 0], exp)


def test_linearity_in_the_weights(oracle):
    rng = np.random.default_rng(4)
    x, wa = _int_layer(rng, 2, 3, 6, 6, 2, 3, 3)
    _, wb = _int_layer(rng, 2, 3, 6, 6, 2, 3, 3)

    def run(w):
        return oracle.conv(x, oracle.csr_to_dense(2, 3, 3, 3, *_csr(w)), 1, 1)[0]

    np.testing.assert_array_equal(run(wa + wb), run(wa) + run(wb))


# ---------------------------------------------------------------- closed forms
def test_all_ones_input_gives_row_sums(oracle):
    L = wl.custom_layer(1, 5, 8, 8, 4, 3, 3, 1, 1, 0.6, seed=2)
    x = np.ones((1, 5, 8, 8), dtype=np.float32)
    Wd = oracle.csr_to_dense(4, 5, 3, 3, L.rowptr, L.colidx, L.value)
    out0, _ = oracle.conv(x, Wd, 1, 0)
    out1, _ = oracle.conv(x, Wd, 1, 1)
    for m in range(4):
        rs = L.weight[m].astype(np.float64).sum()
        np.testing.assert_allclose(out0[0, m], rs, rtol=0, atol=1e-6)          # every pixel
        np.testing.assert_allclose(out1[0, m, 1:-1, 1:-1], rs, rtol=0, atol=1e-6)  # interior
        # top-left corner only sees taps r >= 1, s >= 1; top edge sees r >= 1
        np.testing.assert_allclose(out1[0, m, 0, 0],
                                   L.weight[m, :, 1:, 1:].astype(np.float64).sum(), atol=1e-6)
        np.testing.assert_allclose(out1[0, m, 0, 3],
                                   L.weight[m, :, 1:, :].astype(np.float64).sum(), atol=1e-6)
        np.testing.assert_allclose(out1[0, m, 7, 7],
                                   L.weight[m, :, :2, :2].astype(np.float64).sum(), atol=1e-6)


@pytest.mark.parametrize("stride", [2, 3])
def test_stride_is_subsampling_of_stride_one(oracle, stride):
    L = wl.custom_layer(2, 4, 11, 10, 3, 3, 3, 1, 1, 0.5, seed=31)
    Wd = oracle.csr_to_dense(3, 4, 3, 3, L.rowptr, L.colidx, L.value)
    full, bfull = oracle.conv(L.input, Wd, 1, 1)
    sub, bsub = oracle.conv(L.input, Wd, stride, 1)
    np.testing.assert_array_equal(sub, full[:, :, ::stride, ::stride])
    np.testing.assert_array_equal(bsub, bfull[:, :, ::stride, ::stride])


def test_sampled_points_equal_full_result(oracle):
    L = wl.custom_layer(2, 6, 9, 9, 5, 3, 3, 2, 1, 0.7, seed=77)
    s = L.spec
    Wd = oracle.csr_to_dense(s.M, s.C, 3, 3, L.rowptr, L.colidx, L.value)
    for flags in (0, oracle.F_BIAS | oracle.F_RELU):
        out, bound = oracle.conv(L.input, Wd, 2, 1, bias=L.bias, flags=flags)
        pts = np.array(list(itertools.product(range(s.N), range(s.M), range(s.E), range(s.F))),
                       dtype=np.int32)
        po, pb = oracle.conv_points(L.input, Wd, pts, 2, 1, bias=L.bias, flags=flags)
        np.testing.assert_array_equal(po, out.ravel())
        np.testing.assert_array_equal(pb, bound.ravel())


def test_bias_relu_epilogue_matches_library(oracle):
    L = wl.custom_layer(2, 5, 8, 8, 6, 3, 3, 1, 1, 0.6, seed=13, dist="normal")
    Wd = oracle.csr_to_dense(6, 5, 3, 3, L.rowptr, L.colidx, L.value)
    plain = _torch_conv(L.input, L.weight, 1, 1)
    biased = _torch_conv(L.input, L.weight, 1, 1, bias=L.bias)
    out_b, bb = oracle.conv(L.input, Wd, 1, 1, bias=L.bias, flags=oracle.F_BIAS)
    out_r, _ = oracle.conv(L.input, Wd, 1, 1, bias=L.bias, flags=oracle.F_RELU)
    out_br, _ = oracle.conv(L.input, Wd, 1, 1, bias=L.bias, flags=oracle.F_BIAS | oracle.F_RELU)
    np.testing.assert_allclose(out_b, biased, atol=1e-6)
    np.testing.assert_allclose(out_r, np.maximum(plain, 0), atol=1e-6)   # bias ignored w/o flag
    np.testing.assert_allclose(out_br, np.maximum(biased, 0), atol=1e-6)
    assert (out_br >= 0).all() and (out_b < 0).any()
    _, b0 = oracle.conv(L.input, Wd, 1, 1)
    np.testing.assert_allclose(bb - b0, np.abs(L.bias.astype(np.float64))[None, :, None, None]
                               * np.ones_like(b0), atol=1e-12)


# ---------------------------------------------------------------- weight stretching
@pytest.mark.parametrize("C,H,W,R,S,pad", [(4, 6, 7, 3, 3, 1), (3, 5, 5, 5, 5, 2), (6, 9, 4, 1, 1, 0),
                                           (2, 8, 8, 3, 3, 0), (5, 7, 9, 2, 3, 2)])
def test_stretch_closed_form_roundtrip_additivity(oracle, C, H, W, R, S, pad):
    Hp, Wp = H + 2 * pad, W + 2 * pad
    cols = np.arange(C * R * S, dtype=np.int32)
    st = oracle.stretch(C, H, W, R, S, pad, cols)
    c, r, s = np.unravel_index(cols, (C, R, S))
    # CHW layout function f(c, r, s) = (c*Hin + r)*Win + s on the padded dims (Section 3.1)
    np.testing.assert_array_equal(st, (c * Hp + r) * Wp + s)
    # decode and re-encode
    c2, rem = np.divmod(st, Hp * Wp)
    r2, s2 = np.divmod(rem, Wp)
    np.testing.assert_array_equal((c2 * R + r2) * S + s2, cols)
    # strictly increasing where colidx is
    assert np.all(np.diff(st) > 0)
    # additivity f(c, y+r, x+s) = f(c, y, x) + f(0, r, s) for positions inside the padded plane
    f = lambda cc, y, x: (cc * Hp + y) * Wp + x
    for cc, y, x in [(0, 0, 0), (C - 1, Hp - R, Wp - S), (C // 2, 1, 1)]:
        for rr in range(R):
            for ss in range(S):
                assert f(cc, y + rr, x + ss) == f(cc, y, x) + st[(0 * R + rr) * S + ss]
    assert st.max() == C * Hp * Wp - 1 - (Hp - R) * Wp - (Wp - S)


def test_stretch_rejects_bad_index_and_preserves_order(oracle):
    with pytest.raises(ValueError):
        oracle.stretch(2, 4, 4, 3, 3, 1, np.array([18], dtype=np.int32))
    with pytest.raises(ValueError):
        oracle.stretch(2, 4, 4, 3, 3, 1, np.array([-1], dtype=np.int32))
    cols = np.array([17, 0, 9, 9, 3], dtype=np.int32)           # unsorted, duplicate
    st = oracle.stretch(2, 4, 4, 3, 3, 1, cols)
    np.testing.assert_array_equal(st, [(1 * 6 + 2) * 6 + 2, 0, 36, 36, 6])


def test_csr_footprint_formula():
    """CSR of the filter matrix takes (2*nnz + M + 1)*4 bytes; row lengths are rowptr
    differences (Section 2.3)."""
    L = wl.make_layer("T1")
    nbytes = L.rowptr.nbytes + L.colidx.nbytes + L.value.nbytes
    assert nbytes == (2 * L.nnz + L.spec.M + 1) * 4
    per_row = (L.weight.reshape(L.spec.M, -1) != 0).sum(1)
    np.testing.assert_array_equal(np.diff(L.rowptr), per_row)
    assert abs(L.nnz - 0.2 * L.weight.size) < 5 * np.sqrt(0.16 * L.weight.size)


# ---------------------------------------------------------------- padding
@pytest.mark.parametrize("pad", [0, 1, 2, 3])
def test_pad_interior_and_positive_zero_border(oracle, pad):
    rng = np.random.default_rng(pad)
    x = rng.standard_normal((2, 3, 5, 4)).astype(np.float32)
    x[0, 0, 0, 0] = -0.0
    P = oracle.pad_input(x, pad)
    assert P.shape == (2, 3, 5 + 2 * pad, 4 + 2 * pad)
    inner = P[:, :, pad:pad + 5, pad:pad + 4]
    assert inner.tobytes() == x.tobytes()                 # bit-exact, incl. the -0.0
    mask = np.ones(P.shape, dtype=bool)
    mask[:, :, pad:pad + 5, pad:pad + 4] = False
    assert np.all(P.view(np.uint32)[mask] == 0)           # +0.0f: all bits clear
    if pad == 0:
        assert P.tobytes() == x.tobytes()
    np.testing.assert_array_equal(P, np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad))))


# ---------------------------------------------------------------- workload generators
def test_generators_are_seeded_and_shaped():
    a, b = wl.make_layer("T1"), wl.make_layer("T1")
    assert a.input.tobytes() == b.input.tobytes() and a.value.tobytes() == b.value.tobytes()
    s = a.spec
    assert (s.E, s.F) == (14, 14) and a.input.shape == (1, 16, 14, 14)
    assert 0.4 < (a.input == 0).mean() < 0.6 and a.input.max() <= 1.0 and a.input.min() >= 0.0
    assert np.all(np.abs(a.value) <= 1.0) and np.all(a.value != 0)
    for m in range(s.M):
        row = a.colidx[a.rowptr[m]:a.rowptr[m + 1]]
        assert np.all(np.diff(row) > 0) and (len(row) == 0 or row.max() < s.C * 9)
    r = wl.LAYERS["R56s2"]
    assert (r.E, r.F) == (28, 28)
    g = wl.LAYERS["G5"]
    assert (g.E, g.F) == (28, 28)


def test_skewed_rows_follow_power_law():
    n = wl.skewed_row_nnz(256, 2304, 117965)
    assert n.sum() == 117965 and n.max() == 2304 and n.min() >= 1
    assert (n == 2304).sum() == 21 and abs(int(np.median(n)) - 156) <= 2
    assert np.all(np.diff(n) <= 0)
