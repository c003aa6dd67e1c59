"""GPU parity of compact maps (int16 IN entries) through the C ABI.

The narrow stream holds the same values as the int32 one, so the oracle's IN stream is the
expected value entry by entry; ptr, DA and the side band do not change; a convolution from a
compact map gives, bit for bit, the output it gives from the int32 map of the same input.
"""
import sys

import numpy as np
import pytest

import oracle
from paper_2104_08314_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4


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


def _assert_compact_map(got, ref, algo_code):
    ptr, da, ind, chan_off, hdr = got
    assert ind.dtype == np.int16
    assert hdr[0] == ref.ptr.size and hdr[1] == ref.da.size and hdr[2] == ref.ind.size
    assert hdr[3] == algo_code and hdr[6] == 16 and hdr[7] == 0
    assert np.array_equal(ptr, ref.ptr)
    assert np.array_equal(da.view(np.int32), ref.da.view(np.int32))
    assert np.array_equal(ind.astype(np.int32), ref.ind)
    assert np.array_equal(chan_off, ref.chan_off)


SHAPES = [
    (5, 12, 13, 70, 3, 3, 1, 1),
    (20, 9, 11, 66, 3, 3, 1, 1),          # one-wavefront-per-channel encoder
    (3, 70, 33, 4, 3, 3, 1, 0),           # three-entry NOP segments
    (6, 30, 29, 3, 5, 5, 2, 2),
    (2, 30, 30, 3, 11, 11, 4, 2),         # generic convolution kernel
    (4, 250, 9, 3, 3, 3, 1, 3),           # the tallest map: the largest indices (255 * 3 + 2)
    (520, 5, 6, 3, 3, 3, 1, 1),           # two-launch encoder
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_compact_streams_and_convolutions(api, shape):
    act_np, w_np = workloads.random_case(909, *shape, zero_frac=0.55, zero_channels=1 if shape[0] > 2 else 0)
    _say(f"[case] compact map shape={shape}")
    wide, narrow = api.LayerBuffers(shape), api.LayerBuffers(shape, in_bits=16)
    act, w = torch.from_numpy(act_np).cuda(), torch.from_numpy(w_np).cuda()
    for buf in (wide, narrow):
        api.cpoconv_prepare_weights(w, shape, buf.wt)
        api.cpo_encode(act, shape, buf.cpo, buf.scratch)
        api.cps_encode(act, shape, buf.cps, buf.scratch)
    torch.cuda.synchronize()
    ref_cpo, ref_cps = oracle.cpo_encode(act_np, shape), oracle.cps_encode(act_np, shape)
    _assert_compact_map(narrow.cpo.to_host(), ref_cpo, api.ALGO_CPO)
    _assert_compact_map(narrow.cps.to_host(), ref_cps, api.ALGO_CPS)
    assert wide.cpo.header()[6] == 32
    ref = oracle.conv_direct(act_np, w_np, shape)
    scale = max(float(np.abs(ref).max()), 1e-30)
    for label, conv, fused, which in (("cpo", api.cpo_conv, api.cpo_encode_conv, "cpo"), ("cps", api.cps_conv, api.cps_encode_conv, "cps")):
        outs = []
        for buf in (wide, narrow):
            buf.out.fill_(float("nan"))
            conv(getattr(buf, which), shape, buf.wt, buf.out, buf.scratch)
            torch.cuda.synchronize()
            outs.append(buf.out.clone())
        assert torch.equal(outs[0], outs[1]), label
        assert float(np.abs(outs[1].cpu().numpy() - ref).max()) <= FP32_TOL * scale, label
        narrow.out.fill_(float("nan"))
        fused(act, shape, getattr(narrow, which), narrow.wt, narrow.out, narrow.scratch)
        torch.cuda.synchronize()
        assert torch.equal(narrow.out, outs[1]), label
        _assert_compact_map(getattr(narrow, which).to_host(), ref_cpo if which == "cpo" else ref_cps,
                            api.ALGO_CPO if which == "cpo" else api.ALGO_CPS)


@pytest.mark.parametrize("name", ["cfg1.16@28", "cfg2.128@56", "cfg3.256@14", "cfg4a.5x5.64@27", "cfg4b.3x3s2.128@56",
                                  "cfg5.stem7x7s2", "cfg5.l16.512@7s1"])
def test_compact_workload_layers(api, name):
    spec = {s.name: s for s in workloads.all_layers()}[name]
    shape = spec.shape_tuple
    act_np, w_np = workloads.make_layer(spec)
    _say(f"[case] compact map {name}")
    buf = api.LayerBuffers(shape, in_bits=16)
    act, w = torch.from_numpy(act_np).cuda(), torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    api.cpo_encode_conv(act, shape, buf.cpo, buf.wt, buf.out, buf.scratch)
    torch.cuda.synchronize()
    _assert_compact_map(buf.cpo.to_host(), oracle.cpo_encode(act_np, shape), api.ALGO_CPO)
    ref = oracle.conv_direct(act_np, w_np, shape)
    assert float(np.abs(buf.out.cpu().numpy() - ref).max()) <= FP32_TOL * float(np.abs(ref).max())
    api.cps_encode_conv(act, shape, buf.cps, buf.wt, buf.out, buf.scratch)
    torch.cuda.synchronize()
    _assert_compact_map(buf.cps.to_host(), oracle.cps_encode(act_np, shape), api.ALGO_CPS)
    assert float(np.abs(buf.out.cpu().numpy() - ref).max()) <= FP32_TOL * float(np.abs(ref).max())


@pytest.mark.parametrize("case", [(3, (5, 12, 13, 70, 3, 3, 1, 1)), (8, (36, 13, 9, 70, 3, 3, 2, 1)),
                                  (4, (40, 14, 14, 128, 3, 3, 1, 1)), (9, (33, 7, 7, 64, 3, 3, 1, 1)),
                                  (40, (52, 36, 35, 6, 3, 3, 1, 1))],   # four-wavefront encoder workgroups
                         ids=lambda c: f"n{c[0]}-" + "x".join(map(str, c[1])))
def test_compact_batched(api, case):
    n_images, shape = case
    rng = np.random.default_rng(77)
    acts = np.stack([workloads.random_case(500 + n, *shape, zero_frac=(0.3, 0.8, 0.6)[n % 3], zero_channels=1)[0]
                     for n in range(n_images)])
    acts[1] = 0.0
    w_np = (rng.standard_normal((shape[3], shape[0], shape[4], shape[5])) * 0.2).astype(np.float32)
    _say(f"[case] compact batch n={n_images} shape={shape}")
    buf = api.LayerBuffers(shape, n_images=n_images, in_bits=16)
    act, w = torch.from_numpy(acts).cuda(), torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    api.cpo_encode_batch(act, shape, buf.cpo, buf.scratch)
    api.cps_encode_batch(act, shape, buf.cps, buf.scratch)
    torch.cuda.synchronize()
    ref = np.stack([oracle.conv_direct(acts[n], w_np, shape) for n in range(n_images)])
    scale = max(float(np.abs(ref).max()), 1e-30)
    for n in range(n_images):
        _assert_compact_map(buf.cpo.to_host(image=n), oracle.cpo_encode(acts[n], shape), api.ALGO_CPO)
        _assert_compact_map(buf.cps.to_host(image=n), oracle.cps_encode(acts[n], shape), api.ALGO_CPS)
    for fn, m in ((api.cpo_conv_batch, buf.cpo), (api.cps_conv_batch, buf.cps)):
        buf.out.fill_(float("nan"))
        fn(m, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        assert float(np.abs(buf.out.cpu().numpy().reshape(ref.shape) - ref).max()) <= FP32_TOL * scale


def test_compact_chain(api):
    """The chained workload's first seven layers with a compact shared map: same outputs as with the int32 map."""
    specs = workloads.chain_specs()[:7]
    shapes = [s.shape_tuple for s in specs]
    act_np, w_np, b_np = workloads.make_chain()
    ws = [torch.from_numpy(w).cuda() for w in w_np[:7]]
    bs = [None if b is None else torch.from_numpy(b).cuda() for b in b_np[:7]]
    act = torch.from_numpy(act_np[None]).cuda()
    outs = []
    for bits in (32, 16):
        chain = api.Chain(shapes, ws, bs, [b is not None for b in b_np[:7]], [api.ALGO_CPO, api.ALGO_CPS] * 3 + [api.ALGO_CPO],
                          in_bits=bits)
        chain.forward(act)
        torch.cuda.synchronize()
        outs.append([o.clone() for o in chain.outs])
        assert chain.map.view(shapes[-1]).header()[6] == bits
    for a, b in zip(*outs):
        assert torch.equal(a, b)
