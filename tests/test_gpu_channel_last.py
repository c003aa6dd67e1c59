"""Channel-last (H x W x C) input maps, the other input layout of Table 1's batched input I_n.

Only the readers of the dense map look at the layout (the three encoders, both lowering kernels):
the same values given as H x W x C must produce, bit for bit, the streams and outputs of the
channel-first call, which in turn are checked against the oracle (run on the C x H x W array).
"""
import sys

import numpy as np
import pytest

import oracle
from paper_2104_08314_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4
BF16_TOL = 1e-2


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def api():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2104_08314_amd import api as _api
    _api.lib()
    return _api


def _hwc(shape, api):
    s = list(api.make_shape(shape).as_tuple())
    s[9] = api.LAYOUT_HWC
    return tuple(s)


# one shape per reader: workgroup-per-channel encoder (also the column-run convolution's table), the
# wavefront-per-channel encoder, the band encoder (few channels, large map), strides, one-sided padding
SHAPES = [
    (24, 30, 30, 70, 3, 3, 1, 1),
    (40, 14, 14, 64, 3, 3, 1, 1),
    (3, 130, 140, 20, 7, 7, 2, 3),
    (10, 33, 29, 9, 5, 5, 1, 2),
    (12, 28, 28, 16, 3, 3, 2, 1),
    (16, 17, 17, 24, 1, 7, 1, 0, 3),
    (5, 70, 9, 6, 3, 3, 1, 1),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_channel_last_single_image(api, shape):
    act_np, w_np = workloads.random_case(4242, *shape[:8], zero_frac=0.6, zero_channels=1 if shape[0] > 2 else 0)
    hwc = _hwc(shape, api)
    _say(f"[case] channel-last {shape}")
    ref_cpo, ref_cps = oracle.cpo_encode(act_np, shape), oracle.cps_encode(act_np, shape)
    ref_out = oracle.conv_direct(act_np, w_np, shape)
    scale = float(np.abs(ref_out).max())
    first = api.LayerBuffers(shape)
    last = api.LayerBuffers(hwc)
    act_first = torch.from_numpy(act_np).cuda()
    act_last = torch.from_numpy(np.ascontiguousarray(act_np.transpose(1, 2, 0))).cuda()
    w = torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, first.wt)
    for label, enc, fused, m_first, m_last, ref in (("cpo", api.cpo_encode, api.cpo_encode_conv, first.cpo, last.cpo, ref_cpo),
                                                    ("cps", api.cps_encode, api.cps_encode_conv, first.cps, last.cps, ref_cps)):
        _say(f"[step] {label}_encode")
        enc(act_last, hwc, m_last, last.scratch)
        torch.cuda.synchronize()
        got = m_last.to_host()
        assert got[4][7] == 0
        assert np.array_equal(got[0], ref.ptr) and np.array_equal(got[2], ref.ind)
        assert np.array_equal(got[1].view(np.int32), ref.da.view(np.int32))
        assert np.array_equal(got[3], ref.chan_off)
        _say(f"[step] {label}_encode_conv")
        fused(act_first, shape, m_first, first.wt, first.out, first.scratch)
        last.out.fill_(float("nan"))
        fused(act_last, hwc, m_last, first.wt, last.out, last.scratch)
        torch.cuda.synchronize()
        assert torch.equal(first.out, last.out), label
        assert float(np.abs(last.out.cpu().numpy() - ref_out).max()) <= FP32_TOL * scale
    for prec, tol in ((0, FP32_TOL), (1, BF16_TOL)):
        _say(f"[step] im2col_conv precision={prec}")
        api.im2col_conv(act_first, shape, w, first.lowered, first.out, prec)
        last.out.fill_(float("nan"))
        api.im2col_conv(act_last, hwc, w, last.lowered, last.out, prec)
        torch.cuda.synchronize()
        assert torch.equal(first.out, last.out), prec
        assert float(np.abs(last.out.cpu().numpy() - ref_out).max()) <= tol * scale


@pytest.mark.parametrize("shape,n_images", [((24, 30, 30, 70, 3, 3, 1, 1), 3), ((32, 14, 14, 128, 3, 3, 1, 1), 40),
                                            ((6, 20, 36, 10, 3, 3, 1, 1), 9)])
def test_channel_last_batches(api, shape, n_images):
    """N x H x W x C batches: every image's streams equal the oracle's, the outputs those of the N x C x H x W call
    (also through the LDS-band lowering of eight or more images and the fused bias + ReLU readers)."""
    hwc = _hwc(shape, api)
    _say(f"[case] channel-last batch {shape} n={n_images}")
    rng = np.random.default_rng(99)
    acts = np.stack([workloads.random_case(600 + n, *shape, zero_frac=(0.3, 0.8, 0.6)[n % 3], zero_channels=1)[0]
                     for n in range(n_images)])
    acts -= 0.25      # so that the ReLU of the fused readers has something to cut
    bias_np = rng.normal(0.0, 0.2, shape[0]).astype(np.float32)
    w_np = workloads.random_case(600, *shape, zero_frac=0.5)[1]
    first = api.LayerBuffers(shape, n_images=n_images)
    last = api.LayerBuffers(hwc, n_images=n_images)
    act_first = torch.from_numpy(acts).cuda()
    act_last = torch.from_numpy(np.ascontiguousarray(acts.transpose(0, 2, 3, 1))).cuda()
    w, bias = torch.from_numpy(w_np).cuda(), torch.from_numpy(bias_np).cuda()
    api.cpoconv_prepare_weights(w, shape, first.wt)
    _say("[step] cps_encode_relu")
    api.cps_encode_relu(act_last, bias, hwc, last.cps, last.scratch)
    torch.cuda.synchronize()
    for n in (0, n_images // 2, n_images - 1):
        ref = oracle.cps_encode(oracle.bias_relu(acts[n], bias_np), shape)
        got = last.cps.to_host(image=n)
        assert got[4][7] == 0
        assert np.array_equal(got[0], ref.ptr) and np.array_equal(got[2], ref.ind)
        assert np.array_equal(got[1].view(np.int32), ref.da.view(np.int32))
    _say("[step] cpo_encode_conv_batch")
    api.cpo_encode_conv(act_first, shape, first.cpo, first.wt, first.out, first.scratch)
    last.out.fill_(float("nan"))
    api.cpo_encode_conv(act_last, hwc, last.cpo, first.wt, last.out, last.scratch)
    torch.cuda.synchronize()
    assert torch.equal(first.out, last.out)
    for prec in (0, 1):
        _say(f"[step] im2col_conv_relu precision={prec}")
        api.im2col_conv_relu(act_first, bias, shape, n_images, w, first.lowered, first.out, prec)
        last.out.fill_(float("nan"))
        api.im2col_conv_relu(act_last, bias, hwc, n_images, w, last.lowered, last.out, prec)
        torch.cuda.synchronize()
        assert torch.equal(first.out, last.out), prec
    ref_out = oracle.conv_direct(oracle.bias_relu(acts[1], bias_np), w_np, shape)
    assert float(np.abs(last.out[1].cpu().numpy() - ref_out).max()) <= BF16_TOL * float(np.abs(ref_out).max())
