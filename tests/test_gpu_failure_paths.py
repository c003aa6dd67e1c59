"""Failure handling of the HIP path, forced from the host: every kernel still exits normally.

* A map whose encoder gave up (hdr[7] != 0): cpoconv_map_header_to_host reports CPOCONV_ERR_MAP
  and every convolution given the map leaves its output untouched.
* A scratch buffer overwritten by something else: either the encoder gives up and says so, or the
  map is right; after cpoconv_scratch_init the same buffers work again.
* A map that holds the other algorithm's streams (hdr[3]): the convolution leaves its output
  untouched.
* One scratch buffer shared by calls of different batch sizes and channel counts in turn: the
  look-back words lie at a fixed place, so no call reads another call's data as lengths; every
  encoding stays bit for bit the oracle's.
"""
import sys

import numpy as np
import pytest

import oracle
from paper_2104_08314_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


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


def _same_map(got, ref):
    ptr, da, ind, chan_off, hdr = got
    assert hdr[7] == 0
    assert np.array_equal(ptr, ref.ptr) and np.array_equal(ind, ref.ind)
    assert np.array_equal(da.view(np.int32), ref.da.view(np.int32))
    assert np.array_equal(chan_off, ref.chan_off)


def test_failed_map_is_reported_and_skipped(api):
    """A failed map (made here by the host from a good one: on the device the flag word is raised by
    storing the stamp the header word carries above the index width): the header call says so, every
    convolution leaves its output untouched."""
    shape = (24, 20, 22, 70, 3, 3, 1, 1)
    act_np, w_np = workloads.random_case(77, *shape, zero_frac=0.5)
    buf = api.LayerBuffers(shape)
    act, w = torch.from_numpy(act_np).cuda(), torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    ref = oracle.conv_direct(act_np, w_np, shape)
    for encode, conv, m in ((api.cpo_encode, api.cpo_conv, buf.cpo), (api.cps_encode, api.cps_conv, buf.cps)):
        encode(act, shape, m, buf.scratch)
        assert m.header()[7] == 0
        m.hdr[7] = int(m.hdr[6].item()) >> 8
        with pytest.raises(api.CpoconvError) as err:
            m.header()
        assert err.value.code == api.ERR_MAP and err.value.hdr[7] == 1
        buf.out.fill_(float("nan"))
        conv(m, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        assert bool(torch.isnan(buf.out).all())          # the convolution did not touch its output
        m.hdr[7] = 0
        conv(m, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        assert float(np.abs(buf.out.cpu().numpy() - ref).max()) <= 1e-4 * float(np.abs(ref).max())


@pytest.mark.parametrize("shape", [(24, 20, 22, 70, 3, 3, 1, 1), (40, 9, 9, 64, 3, 3, 1, 1), (3, 70, 66, 8, 3, 3, 1, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_overwritten_scratch_is_never_silently_wrong(api, shape):
    """A scratch buffer overwritten by something else.  Worst case: the foreign data looks like
    look-back words of the running call (matching tags) with lengths that are not lengths.  A reader
    that picks such a word up must give up (hdr[7]); a reader that sees its predecessor's real word
    is right.  So either the map is flagged and the convolution skips it, or every stream is bit for
    bit the oracle's - never a wrong map without a flag.  Random bytes (no matching tags) only cost
    waiting: the encoding is right."""
    _say(f"[case] overwritten scratch shape={shape}")
    act_np, w_np = workloads.random_case(79, *shape, zero_frac=0.5)
    buf = api.LayerBuffers(shape)
    act, w = torch.from_numpy(act_np).cuda(), torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    ref_map = oracle.cpo_encode(act_np, shape)
    words = buf.scratch[: buf.scratch.numel() // 8 * 8].view(torch.int64)
    # epoch word and look-back words alike: tag 0x10 in the upper half, and a lower half chosen so that
    # the tag the encoder derives from this "epoch" is 0x10 as well
    pattern = (0x10 << 32) | (0xFFFFFFFE - 17)
    for fill in (pattern, None):
        if fill is None:
            buf.scratch.copy_(torch.randint(0, 256, (buf.scratch.numel(),), dtype=torch.uint8, device="cuda"))
        else:
            words.fill_(fill)
        buf.out.fill_(float("nan"))
        api.cpo_encode_conv(act, shape, buf.cpo, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        try:
            hdr = buf.cpo.header()
        except api.CpoconvError as err:
            assert err.code == api.ERR_MAP
            assert bool(torch.isnan(buf.out).all())
            assert fill is not None                      # random bytes carry no matching tag
            continue
        assert hdr[7] == 0
        _same_map(buf.cpo.to_host(), ref_map)
    # prepared again, everything works
    api.cpoconv_scratch_init(buf.scratch)
    ref = oracle.conv_direct(act_np, w_np, shape)
    api.cpo_encode_conv(act, shape, buf.cpo, buf.wt, buf.out, buf.scratch)
    torch.cuda.synchronize()
    _same_map(buf.cpo.to_host(), ref_map)
    assert float(np.abs(buf.out.cpu().numpy() - ref).max()) <= 1e-4 * float(np.abs(ref).max())


def test_map_of_the_other_algorithm_is_skipped(api):
    shape = (16, 20, 20, 64, 3, 3, 1, 1)
    act_np, w_np = workloads.random_case(78, *shape, zero_frac=0.3)
    buf = api.LayerBuffers(shape)
    act, w = torch.from_numpy(act_np).cuda(), torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    api.cpo_encode(act, shape, buf.cpo, buf.scratch)
    api.cps_encode(act, shape, buf.cps, buf.scratch)
    for conv, m in ((api.cps_conv, buf.cpo), (api.cpo_conv, buf.cps)):
        buf.out.fill_(float("nan"))
        conv(m, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        assert bool(torch.isnan(buf.out).all())
    ref = oracle.conv_direct(act_np, w_np, shape)
    for conv, m in ((api.cpo_conv, buf.cpo), (api.cps_conv, buf.cps)):
        buf.out.fill_(float("nan"))
        conv(m, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        assert float(np.abs(buf.out.cpu().numpy() - ref).max()) <= 1e-4 * float(np.abs(ref).max())


def test_one_scratch_buffer_serves_calls_of_different_batch_sizes(api):
    """Batch 1 and batch 8, 20 and 600 channels (one launch and two), large and small maps, all on
    one scratch buffer, twice round."""
    cases = [((20, 30, 31, 8, 3, 3, 1, 1), 1, "cps_layer"), ((20, 30, 31, 8, 3, 3, 1, 1), 8, "cpo"),
             ((600, 6, 7, 4, 3, 3, 1, 1), 2, "cps"), ((3, 70, 66, 8, 3, 3, 1, 1), 1, "cpo"),
             ((64, 12, 12, 8, 3, 3, 1, 1), 5, "cps"), ((20, 30, 31, 8, 3, 3, 1, 1), 1, "cpo_layer")]
    sizes = [api.cpoconv_batch_sizes(shape, n) for shape, n, _ in cases]
    scratch = torch.empty(max(s.scratch_bytes for s in sizes), dtype=torch.uint8, device="cuda")
    api.cpoconv_scratch_init(scratch)
    for rnd in range(2):
        for i, (shape, n, what) in enumerate(cases):
            _say(f"[case] shared scratch round {rnd} shape={shape} n={n} {what}")
            acts = np.stack([workloads.random_case(300 + 10 * i + j + rnd, *shape, zero_frac=0.6, zero_channels=1)[0]
                             for j in range(n)])
            w_np = workloads.random_case(300 + i, *shape, zero_frac=0.6)[1]
            act = torch.from_numpy(acts if n > 1 else acts[0]).cuda()
            m = api.EncodedMap(shape, n_images=n)
            cps = what.startswith("cps")
            if what.endswith("_layer"):
                sz = api.cpoconv_batch_sizes(shape, n)
                wt = torch.empty(sz.wt_len, dtype=torch.float32, device="cuda")
                api.cpoconv_prepare_weights(torch.from_numpy(w_np).cuda(), shape, wt)
                out = torch.empty((shape[3], sz.Oh, sz.Ow), dtype=torch.float32, device="cuda")
                (api.cps_encode_conv if cps else api.cpo_encode_conv)(act, shape, m, wt, out, scratch)
                torch.cuda.synchronize()
                ref = oracle.conv_direct(acts[0], w_np, shape)
                assert float(np.abs(out.cpu().numpy() - ref).max()) <= 1e-4 * float(np.abs(ref).max())
            elif n > 1:
                (api.cps_encode_batch if cps else api.cpo_encode_batch)(act, shape, m, scratch)
            else:
                (api.cps_encode if cps else api.cpo_encode)(act, shape, m, scratch)
            torch.cuda.synchronize()
            for j in range(n):
                _same_map(m.to_host(image=j), (oracle.cps_encode if cps else oracle.cpo_encode)(acts[j], shape))
