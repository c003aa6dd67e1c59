"""Seeded random layers through the batched entry points: kernel shapes, strides, one- and two-sided
paddings, channel and kernel counts drawn so that every launch shape of the SpMV kernels and both
encoders are reached by shapes nobody picked by hand.  Streams bit for bit, sums within the fp32
tolerance, against the oracle image by image."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2104_08314_amd import workloads

pytestmark = pytest.mark.gpu
FP32_TOL = 1e-4


@pytest.fixture(scope="module")
def api():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2104_08314_amd import api as _api
    _api.lib()
    return _api


def _draw(rng):
    while True:
        k = int(rng.choice([3, 3, 3, 5]))
        kh, kw = k, k
        if rng.random() < 0.4:
            kh, kw = [(1, 7), (7, 1), (1, 3), (3, 1)][int(rng.integers(4))]
        s = int(rng.choice([1, 1, 2]))
        ph = int(rng.choice([0, 1, kh // 2]))
        pw = int(rng.choice([0, 1, kw // 2]))
        H, W = int(rng.integers(max(kh - 2 * ph, 1), 40)), int(rng.integers(max(kw - 2 * pw, 1), 40))
        if kh != kw and rng.random() < 0.7:     # the widths the wide strips of these kernels take
            W = int(rng.integers(12, 20)) if max(kh, kw) == 7 else int(rng.integers(4, 10))
            H = int(rng.integers(max(kh - 2 * ph, 1), 24))
        if H + 2 * ph < kh or W + 2 * pw < kw:
            continue
        C = int(rng.choice([3, 32, 33, 40, 64]))
        K = int(rng.choice([64, 70, 128, 160, 192, 256, 384]))
        N = int(rng.choice([1, 4, 8, 9]))
        if C * H * W * N > 400000 or K * C * kh * kw * H * W * N > 3e9:
            continue
        shape = (C, H, W, K, kh, kw, s, ph) if pw == ph else (C, H, W, K, kh, kw, s, ph, pw)
        return N, shape, int(rng.choice([32, 16]))


def test_random_layers(api):
    rng = np.random.default_rng(20210408)
    for case in range(40):
        n_images, shape, bits = _draw(rng)
        print(f"[case] {case}: n={n_images} shape={shape} in_bits={bits}", file=sys.stderr, flush=True)
        acts = np.stack([workloads.random_case(int(rng.integers(1 << 30)), *shape[:8],
                                               zero_frac=float(rng.choice([0.2, 0.5, 0.8, 0.95])),
                                               zero_channels=int(rng.integers(0, 2)))[0] for _ in range(n_images)])
        w_np = (rng.standard_normal((shape[3], shape[0], shape[4], shape[5])) * 0.2).astype(np.float32)
        buf = api.LayerBuffers(shape, n_images=n_images, in_bits=bits)
        act, w = torch.from_numpy(acts).cuda(), torch.from_numpy(w_np).cuda()
        api.cpoconv_prepare_weights(w, shape, buf.wt)
        api.cpo_encode_batch(act, shape, buf.cpo, buf.scratch)
        api.cps_encode_batch(act, shape, buf.cps, buf.scratch)
        torch.cuda.synchronize()
        for n in range(n_images):
            for m, ref in ((buf.cpo, oracle.cpo_encode(acts[n], shape)), (buf.cps, oracle.cps_encode(acts[n], shape))):
                ptr, da, ind, chan_off, hdr = m.to_host(image=n)
                assert hdr[7] == 0 and np.array_equal(ptr, ref.ptr), (case, n)
                assert np.array_equal(da.view(np.int32), ref.da.view(np.int32)), (case, n)
                assert np.array_equal(ind.astype(np.int32), ref.ind) and np.array_equal(chan_off, ref.chan_off), (case, n)
        ref = np.stack([oracle.conv_direct(acts[n], w_np, shape) for n in range(n_images)])
        scale = max(float(np.abs(ref).max()), 1e-30)
        for fn, m in ((api.cpo_conv_batch, buf.cpo), (api.cps_conv_batch, buf.cps)):
            buf.out.fill_(float("nan"))
            fn(m, shape, buf.wt, buf.out, buf.scratch)
            torch.cuda.synchronize()
            got = buf.out.cpu().numpy().reshape(ref.shape)
            assert np.isfinite(got).all(), case
            assert float(np.abs(got - ref).max()) <= FP32_TOL * scale, case
        buf.out.fill_(float("nan"))
        api.im2col_conv_batch(act, shape, n_images, w, buf.lowered, buf.out, 0)
        torch.cuda.synchronize()
        assert float(np.abs(buf.out.cpu().numpy().reshape(ref.shape) - ref).max()) <= FP32_TOL * scale, case
        del buf
