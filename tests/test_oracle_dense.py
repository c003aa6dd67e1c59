"""Pins for the oracle's dense definitions (Eq. 1, im2col lowering, selection).

None of these checks re-uses the oracle's own formula: they use a library convolution as a
second witness, closed forms, and hand-derived special cases.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08314_amd import workloads

SHAPES = [
    # C, H, W, K, kh, kw, stride, pad
    (1, 4, 4, 1, 3, 3, 1, 1),
    (3, 7, 9, 4, 3, 3, 1, 1),
    (2, 8, 8, 3, 4, 4, 1, 1),
    (2, 9, 6, 2, 5, 5, 1, 2),
    (3, 10, 11, 2, 3, 3, 2, 1),
    (2, 11, 8, 3, 3, 2, 3, 0),
    (1, 12, 12, 2, 7, 7, 2, 3),
    (4, 6, 5, 5, 1, 3, 1, 0),
    (2, 5, 6, 2, 3, 1, 1, 0),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_direct_conv_matches_library_convolution(shape):
    C, H, W, K, kh, kw, s, p = shape
    act, w = workloads.random_case(11, *shape, zero_frac=0.5)
    got = oracle.conv_direct(act, w, shape)
    ref = torch.nn.functional.conv2d(torch.from_numpy(act).double()[None],
                                     torch.from_numpy(w).double(), stride=s, padding=p)[0].numpy()
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref.astype(np.float32), rtol=0, atol=1e-6 * np.abs(ref).max())


def test_direct_conv_all_ones_closed_form():
    # VALID padding, all-one input and kernel: every output equals C*kh*kw.
    shape = (3, 6, 7, 2, 3, 2, 1, 0)
    act = np.ones((3, 6, 7), np.float32)
    w = np.ones((2, 3, 3, 2), np.float32)
    out = oracle.conv_direct(act, w, shape)
    assert out.shape == (2, 4, 6)
    assert np.all(out == 18.0)


def test_direct_conv_is_cross_correlation_of_a_delta():
    # One unit NZE at (c0, h0, w0): out[k, y, x] = W[k, c0, h0+p-y*s, w0+p-x*s] where that
    # kernel cell exists (no kernel flip), zero elsewhere.  Derived by hand from Eq. 1.
    C, H, W, K, kh, kw, s, p = shape = (2, 7, 8, 3, 3, 4, 2, 1)
    rng = np.random.default_rng(5)
    w = rng.integers(1, 50, size=(K, C, kh, kw)).astype(np.float32)
    c0, h0, w0 = 1, 4, 5
    act = np.zeros((C, H, W), np.float32)
    act[c0, h0, w0] = 1.0
    out = oracle.conv_direct(act, w, shape)
    Oh, Ow = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
    expect = np.zeros((K, Oh, Ow), np.float32)
    for y in range(Oh):
        for x in range(Ow):
            l, ww = h0 + p - y * s, w0 + p - x * s
            if 0 <= l < kh and 0 <= ww < kw:
                expect[:, y, x] = w[:, c0, l, ww]
    assert np.array_equal(out, expect)
    assert np.count_nonzero(expect) > 0


@pytest.mark.parametrize("shape", SHAPES)
def test_im2col_lowered_matrix_definition(shape):
    C, H, W, K, kh, kw, s, p = shape
    act, w = workloads.random_case(3, *shape, zero_frac=0.4)
    low = oracle.im2col_lower(act, shape)
    Oh, Ow = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
    assert low.shape == (C * kh * kw, Oh * Ow)          # S_im2col = C*kh*kw*Oh*Ow
    padded = np.pad(act, ((0, 0), (p, p), (p, p)))
    for c in range(C):
        for l in range(kh):
            for ww in range(kw):
                patch = padded[c, l:l + s * (Oh - 1) + 1:s, ww:ww + s * (Ow - 1) + 1:s]
                assert np.array_equal(low[(c * kh + l) * kw + ww].reshape(Oh, Ow), patch)
    # lowering followed by the matrix product is the convolution
    out = oracle.im2col_conv(act, w, shape)
    ref = oracle.conv_direct(act, w, shape)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-6 * max(1.0, np.abs(ref).max()))


def test_gemm_against_numpy():
    rng = np.random.default_rng(0)
    a = rng.standard_normal((5, 7)).astype(np.float32)
    b = rng.standard_normal((7, 3)).astype(np.float32)
    np.testing.assert_allclose(oracle.gemm(a, b), (a.astype(np.float64) @ b.astype(np.float64)),
                               rtol=1e-6, atol=1e-6)


def test_select_layer_algo_rules():
    # Section 3.5: totals over the M offline inputs decide; favour time compares im2col with
    # CPO, favour space compares im2col with CPS; the default (im2col) keeps a tie.
    t_im = [10.0, 10.0, 10.0, 10.0, 10.0]
    t_cpo = [1.0, 30.0, 1.0, 1.0, 1.0]     # total 34 < 50 although one input is slower
    t_cps = [12.0, 12.0, 12.0, 12.0, 12.0]
    assert oracle.select_layer_algo(t_im, t_cpo, t_cps, 0) == 1
    assert oracle.select_layer_algo(t_im, t_cpo, t_cps, 1) == 0
    assert oracle.select_layer_algo(t_im, t_cps, t_cpo, 0) == 0
    assert oracle.select_layer_algo(t_im, t_cps, t_cpo, 1) == 2
    assert oracle.select_layer_algo([5.0, 5.0], [4.0, 6.0], [6.0, 4.0], 0) == 0
    assert oracle.select_layer_algo([5.0, 5.0], [4.0, 6.0], [6.0, 4.0], 1) == 0
