"""The entry point that allocates nothing: cpo_encode_static_scratch against cpo_encode.

Same streams, side band and header, bit for bit, on two calls in a row - the second with a
smaller input, so that it meets the first call's words in the shared device array - and again
after a call of another shape; layers whose look-back words exceed the array are refused.
"""
import sys

import numpy as np
import pytest

from paper_2104_08314_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2104_08314_amd import api as _api
    _api.lib()
    return _api


def _encode_both(api, shape, seed):
    act_np, _ = workloads.random_case(seed, *shape, zero_frac=0.6, zero_channels=1)
    print(f"[case] static scratch shape={shape} seed={seed}", flush=True)
    sys.stdout.flush()
    act = torch.from_numpy(act_np).cuda()
    buf = api.LayerBuffers(shape)
    api.cpo_encode(act, shape, buf.cpo, buf.scratch)
    other = api.EncodedMap(shape)
    other.ptr.fill_(-77); other.da.fill_(float("nan")); other.ind.fill_(-77)
    api.cpo_encode_static_scratch(act, shape, other)
    torch.cuda.synchronize()
    a, b = buf.cpo.to_host(), other.to_host()
    assert a[4] == b[4] and b[4][7] == 0                                   # header
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[2], b[2])       # ptr, IN
    assert np.array_equal(a[1].view(np.int32), b[1].view(np.int32))        # DA, bit for bit
    assert np.array_equal(a[3], b[3])                                      # side band


def test_static_scratch_encoder_equals_cpo_encode(api):
    # two calls in a row, the second smaller; then other kernels of the encoder (small maps,
    # bands) and the first shape again on new data
    _encode_both(api, (96, 40, 44, 8, 3, 3, 1, 1), 501)
    _encode_both(api, (24, 13, 11, 8, 3, 3, 1, 1), 502)
    _encode_both(api, (3, 100, 90, 8, 5, 5, 1, 2), 503)
    _encode_both(api, (300, 7, 7, 8, 3, 3, 1, 1), 504)
    _encode_both(api, (96, 40, 44, 8, 3, 3, 1, 1), 505)


def test_static_scratch_encoder_refuses_what_does_not_fit(api):
    shape = (70000, 2, 2, 4, 1, 1, 1, 0)      # the two-launch encoder's words alone exceed the array
    m = api.EncodedMap(shape)
    act = torch.zeros((shape[0], 2, 2), dtype=torch.float32, device="cuda")
    with pytest.raises(api.CpoconvError) as err:
        api.cpo_encode_static_scratch(act, shape, m)
    assert err.value.code == api.ERR_SMALL
