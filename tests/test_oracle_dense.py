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
    # rows and columns padded differently: (.., stride, pad_h, pad_w)
    (2, 9, 8, 3, 1, 7, 1, 0, 3),
    (2, 9, 8, 3, 7, 1, 1, 3, 0),
    (3, 6, 7, 2, 3, 3, 1, 0, 1),
    (3, 6, 7, 2, 3, 3, 2, 2, 0),
    (2, 8, 9, 2, 5, 3, 1, 2, 1),
]


def _unpack(shape):
    v = tuple(shape)
    return v if len(v) == 9 else v + (v[7],)


@pytest.mark.parametrize("shape", SHAPES)
def test_direct_conv_matches_library_convolution(shape):
    C, H, W, K, kh, kw, s, ph, pw = _unpack(shape)
    p = (ph, pw)
    act, w = workloads.random_case(11, *shape[:8], zero_frac=0.5)
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
    _delta_case((2, 7, 8, 3, 3, 4, 2, 1))
    _delta_case((2, 7, 8, 3, 3, 4, 2, 2, 0))   # rows and columns padded differently
    _delta_case((2, 7, 8, 3, 1, 5, 1, 0, 2))


def _delta_case(shape):
    C, H, W, K, kh, kw, s, p, pw = _unpack(shape)
    rng = np.random.default_rng(5)
    w = rng.integers(1, 50, size=(K, C, kh, kw)).astype(np.float32)
    c0, h0, w0 = 1, 4, 5
    act = np.zeros((C, H, W), np.float32)
    act[c0, h0, w0] = 1.0
    out = oracle.conv_direct(act, w, shape)
    Oh, Ow = (H + 2 * p - kh) // s + 1, (W + 2 * pw - kw) // s + 1
    expect = np.zeros((K, Oh, Ow), np.float32)
    for y in range(Oh):
        for x in range(Ow):
            l, ww = h0 + p - y * s, w0 + pw - x * s
            if 0 <= l < kh and 0 <= ww < kw:
                expect[:, y, x] = w[:, c0, l, ww]
    assert np.array_equal(out, expect)
    assert np.count_nonzero(expect) > 0


@pytest.mark.parametrize("shape", SHAPES)
def test_im2col_lowered_matrix_definition(shape):
    C, H, W, K, kh, kw, s, ph, pw = _unpack(shape)
    act, w = workloads.random_case(3, *shape[:8], zero_frac=0.4)
    low = oracle.im2col_lower(act, shape)
    Oh, Ow = (H + 2 * ph - kh) // s + 1, (W + 2 * pw - kw) // s + 1
    assert low.shape == (C * kh * kw, Oh * Ow)          # S_im2col = C*kh*kw*Oh*Ow
    padded = np.pad(act, ((0, 0), (ph, ph), (pw, pw)))
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


# --- the producer epilogue (bias, ReLU) and chained layers --------------------------------------
def test_bias_relu_special_values():
    """Value table: only z > 0 survives; -0, negatives and NaN become +0; denormals and inf stay."""
    tiny = np.float32(1e-45)                      # smallest denormal
    pre = np.array([[[-1.5, -0.0, 0.0, 2.5, np.nan, np.inf, -np.inf, tiny, -tiny]]], np.float32)
    got = oracle.bias_relu(pre)
    want = np.array([[[0.0, 0.0, 0.0, 2.5, 0.0, np.inf, 0.0, tiny, 0.0]]], np.float32)
    assert got.dtype == np.float32
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))   # bit for bit: zeros are +0


def test_bias_relu_adds_the_channel_bias_in_fp32_before_the_threshold():
    pre = np.array([[[1.0, -1.0]], [[1.0, -1.0]], [[16777216.0, 0.25]]], np.float32)
    bias = np.array([-1.0, 2.0, 1.0], np.float32)
    got = oracle.bias_relu(pre, bias)
    # channel 0: 1-1 = 0 -> 0, -2 -> 0;  channel 1: 3, 1;  channel 2: 2^24 + 1 rounds to 2^24 (one fp32 addition)
    want = np.array([[[0.0, 0.0]], [[3.0, 1.0]], [[16777216.0, 1.25]]], np.float32)
    assert np.array_equal(got, want)


def test_bias_relu_matches_library_relu():
    rng = np.random.default_rng(11)
    pre = rng.standard_normal((5, 9, 7)).astype(np.float32)
    bias = rng.standard_normal(5).astype(np.float32)
    lib = torch.relu(torch.from_numpy(pre) + torch.from_numpy(bias)[:, None, None]).numpy()
    assert np.array_equal(oracle.bias_relu(pre, bias), lib)
    assert np.array_equal(oracle.bias_relu(np.abs(pre)), np.abs(pre))      # identity on positive maps


def test_encoding_of_a_relu_output_holds_exactly_the_positive_elements():
    rng = np.random.default_rng(12)
    shape = (4, 9, 10, 3, 3, 3, 1, 1)
    pre = rng.standard_normal(shape[:3]).astype(np.float32)
    m = oracle.cpo_encode(oracle.bias_relu(pre), shape)
    assert m.da.size == int((pre > 0).sum())
    assert np.array_equal(oracle.decode(m), np.maximum(pre, 0))


def _chain_case(seed):
    rng = np.random.default_rng(seed)
    shapes = [(3, 11, 12, 5, 3, 3, 1, 1), (5, 11, 12, 4, 3, 3, 2, 1), (4, 6, 6, 6, 5, 5, 1, 2)]
    chain = []
    for i, s in enumerate(shapes):
        w = (rng.standard_normal((s[3], s[0], s[4], s[5])) * 0.3).astype(np.float32)
        b = None if i == 0 else rng.standard_normal(s[0]).astype(np.float32) * 0.2
        chain.append((s, w, b, i > 0))
    act = np.maximum(rng.standard_normal(shapes[0][:3]), 0).astype(np.float32)
    return act, chain


def test_chain_forward_matches_library_network():
    act, chain = _chain_case(21)
    outs = oracle.chain_forward(act, chain)
    x = torch.from_numpy(act).double()[None]
    for (s, w, b, relu_in), got in zip(chain, outs):
        if relu_in:
            x = torch.relu(x + torch.from_numpy(b).double()[None, :, None, None])
        x = torch.nn.functional.conv2d(x, torch.from_numpy(w).double(), stride=s[6], padding=s[7])
        assert got.shape == tuple(x.shape[1:])
        assert np.abs(got - x[0].numpy()).max() <= 1e-5 * float(x.abs().max())


def test_chain_of_identity_kernels_is_repeated_relu():
    """1x1 identity kernels: every layer's output is its (activated) input, so the chain's outputs
    are pre, relu(pre + b1), relu(relu(pre + b1) + b2)."""
    rng = np.random.default_rng(22)
    C = 4
    pre = rng.standard_normal((C, 6, 5)).astype(np.float32)
    eye = np.eye(C, dtype=np.float32).reshape(C, C, 1, 1)
    b1, b2 = rng.standard_normal(C).astype(np.float32), rng.standard_normal(C).astype(np.float32)
    s = (C, 6, 5, C, 1, 1, 1, 0)
    outs = oracle.chain_forward(pre, [(s, eye, None, False), (s, eye, b1, True), (s, eye, b2, True)])
    r1 = np.maximum(pre + b1[:, None, None], 0)
    assert np.array_equal(outs[0], pre)
    assert np.array_equal(outs[1], r1)
    assert np.array_equal(outs[2], np.maximum(r1 + b2[:, None, None], 0))
