"""GPU parity of the fused producers (bias + ReLU applied while a map is read) and of chained
layers, through the C ABI, against the CPU oracle on the same seeded inputs.

A single fused call is exact where the separate calls are: the encoders' streams match
oracle.encode(oracle.bias_relu(pre, bias)) bit for bit (one fp32 addition and a sign test on each
side), the comparator matches Eq. 1 on that map within the per-layer tolerance.

In a chain, layer i reads what layer i-1 computed in fp32 with the GPU's own summation order, so
an element whose exact value is within rounding of zero may be an NZE on one side and a zero on
the other: the streams of inner layers are not unique.  What is unique is checked - every layer's
output against the oracle's chain within (i + 1) * 1e-4 * max|out_i| (each layer adds at most the
single-layer bound to what it inherits; the layers' gain is about one with these weights), and the
decoded last encoding against the oracle's activated map within the same tolerance - and the rest
is checked for validity: the streams the GPU wrote are bit for bit the oracle's encoding of the
map they decode to.
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


def _assert_same_map(got, ref, algo_code):
    ptr, da, ind, chan_off, hdr = got
    assert hdr[0] == ref.ptr.size and hdr[1] == ref.da.size and hdr[2] == ref.ind.size
    assert hdr[3] == algo_code and hdr[7] == 0
    assert np.array_equal(ptr, ref.ptr)
    assert np.array_equal(da.view(np.int32), ref.da.view(np.int32))      # bit for bit
    assert np.array_equal(ind, ref.ind)
    assert np.array_equal(chan_off, ref.chan_off)


def _pre_activation(seed, n_images, shape, special=True):
    """Pre-activation maps: signed values, with the values a sign test must get right sprinkled in."""
    rng = np.random.default_rng(seed)
    C, H, W = shape[:3]
    pre = rng.standard_normal((n_images, C, H, W)).astype(np.float32)
    if special:
        flat = pre.reshape(-1)
        tiny = np.float32(1e-45)
        for k, v in enumerate((-0.0, 0.0, np.nan, np.inf, -np.inf, tiny, -tiny, np.float32(1.1754944e-38))):
            flat[rng.choice(flat.size, size=max(1, flat.size // 97), replace=False)] = v
    if C > 2:
        pre[:, rng.choice(C, size=1)] = -1.0          # a channel the ReLU switches off entirely
    bias = (0.5 * rng.standard_normal(C)).astype(np.float32)
    return pre, bias


RELU_CASES = [
    # (n_images, shape): wide-kernel path, one-wavefront-per-channel path, two-launch path, strides, CPS packing
    (1, (5, 12, 13, 4, 3, 3, 1, 1)),
    (3, (20, 9, 11, 6, 3, 3, 1, 1)),
    (1, (7, 40, 70, 3, 3, 3, 1, 1)),
    (2, (6, 30, 29, 3, 5, 5, 2, 2)),
    (1, (520, 5, 6, 3, 3, 3, 1, 1)),
    (2, (3, 70, 33, 4, 3, 3, 1, 0)),
    (3, (400, 20, 22, 3, 3, 3, 1, 1)),
]


@pytest.mark.parametrize("with_bias", [False, True], ids=["nobias", "bias"])
@pytest.mark.parametrize("case", RELU_CASES, ids=lambda c: f"n{c[0]}-" + "x".join(map(str, c[1])))
def test_encode_relu_streams(api, case, with_bias):
    n_images, shape = case
    pre_np, bias_np = _pre_activation(707, n_images, shape)
    _say(f"[case] encode_relu n={n_images} shape={shape} bias={with_bias}")
    buf = api.LayerBuffers(shape, n_images=n_images)
    pre = torch.from_numpy(pre_np).cuda()
    bias = torch.from_numpy(bias_np).cuda() if with_bias else None
    api.cpo_encode_relu(pre, bias, shape, buf.cpo, buf.scratch)
    api.cps_encode_relu(pre, bias, shape, buf.cps, buf.scratch)
    torch.cuda.synchronize()
    for n in range(n_images):
        act = oracle.bias_relu(pre_np[n], bias_np if with_bias else None)
        _assert_same_map(buf.cpo.to_host(image=n), oracle.cpo_encode(act, shape), api.ALGO_CPO)
        _assert_same_map(buf.cps.to_host(image=n), oracle.cps_encode(act, shape), api.ALGO_CPS)


@pytest.mark.parametrize("case", RELU_CASES[:4], ids=lambda c: f"n{c[0]}-" + "x".join(map(str, c[1])))
def test_im2col_conv_relu(api, case):
    n_images, shape = case
    pre_np, bias_np = _pre_activation(808, n_images, shape, special=False)
    rng = np.random.default_rng(809)
    w_np = (rng.standard_normal((shape[3], shape[0], shape[4], shape[5])) * 0.2).astype(np.float32)
    _say(f"[case] im2col_conv_relu n={n_images} shape={shape}")
    buf = api.LayerBuffers(shape, n_images=n_images)
    pre, bias, w = (torch.from_numpy(a).cuda() for a in (pre_np, bias_np, w_np))
    ref = np.stack([oracle.conv_direct(oracle.bias_relu(pre_np[n], bias_np), w_np, shape) for n in range(n_images)])
    scale = float(np.abs(ref).max())
    for prec, tol in ((0, FP32_TOL), (1, BF16_TOL)):
        buf.out.fill_(float("nan"))
        api.im2col_conv_relu(pre, bias, shape, n_images, w, buf.lowered, buf.out, prec)
        torch.cuda.synchronize()
        got = buf.out.cpu().numpy().reshape(ref.shape)
        assert np.isfinite(got).all(), prec
        assert float(np.abs(got - ref).max()) <= tol * scale, prec


# --- chained layers ------------------------------------------------------------------------------
def _run_chain(api, act_np, shapes, w_np, b_np, methods, n_images, precision=0):
    """Runs the chain on the GPU; returns (chain object, list of per-layer outputs as numpy)."""
    ws = [torch.from_numpy(w).cuda() for w in w_np]
    bs = [None if b is None else torch.from_numpy(b).cuda() for b in b_np]
    chain = api.Chain(shapes, ws, bs, [b is not None for b in b_np], methods, n_images=n_images, precision=precision)
    for o in chain.outs:
        o.fill_(float("nan"))
    act = torch.from_numpy(act_np).cuda()
    chain.forward(act)
    torch.cuda.synchronize()
    return chain, [o.cpu().numpy() for o in chain.outs]


def _check_chain(api, act_np, shapes, w_np, b_np, methods, tol=FP32_TOL, precision=0):
    n_images = act_np.shape[0]
    chain, outs = _run_chain(api, act_np, shapes, w_np, b_np, methods, n_images, precision)
    table = [(s, w, b, b is not None) for s, w, b in zip(shapes, w_np, b_np)]
    for n in range(n_images):
        refs = oracle.chain_forward(act_np[n], table)
        for i, ref in enumerate(refs):
            got = outs[i][n]
            scale = max(float(np.abs(ref).max()), 1e-30)
            err = float(np.abs(got - ref).max())
            assert np.isfinite(got).all(), (n, i)
            assert err <= (i + 1) * tol * scale, (n, i, methods[i], err, scale)
        # the last encoding left in the shared map
        last = max((i for i, m in enumerate(methods) if m != api.ALGO_IM2COL), default=None)
        if last is None:
            continue
        code = methods[last]
        ptr, da, ind, chan_off, hdr = chain.map.view(shapes[last]).to_host(image=n)
        assert hdr[3] == code and hdr[7] == 0
        algo = oracle.ALGO_CPO if code == api.ALGO_CPO else oracle.ALGO_CPS
        held = oracle.EncodedMap(algo, tuple(shapes[last]), ptr, da, ind, chan_off)
        dense = oracle.decode(held)
        want = act_np[n] if last == 0 else refs[last - 1]
        if b_np[last] is not None:
            want = oracle.bias_relu(want, b_np[last])
        scale = max(float(np.abs(want).max()), 1e-30)
        assert float(np.abs(dense - want).max()) <= max(last, 1) * tol * scale
        again = oracle.encode(dense, tuple(shapes[last]), algo)      # valid: the encoding of what it decodes to
        assert np.array_equal(again.ptr, ptr) and np.array_equal(again.ind, ind)
        assert np.array_equal(again.da.view(np.int32), da.view(np.int32))
    return chain


def _small_chain(seed, n_images):
    rng = np.random.default_rng(seed)
    shapes = [(6, 20, 22, 70, 3, 3, 1, 1), (70, 20, 22, 9, 3, 3, 2, 1), (9, 10, 11, 12, 5, 5, 1, 2), (12, 10, 11, 5, 3, 3, 1, 1)]
    w_np, b_np = [], []
    for i, s in enumerate(shapes):
        w_np.append((rng.standard_normal((s[3], s[0], s[4], s[5])) * np.sqrt(2.0 / (s[0] * s[4] * s[5]))).astype(np.float32))
        b_np.append(None if i == 0 else (0.3 * rng.standard_normal(s[0])).astype(np.float32))
    act = np.maximum(rng.standard_normal((n_images,) + shapes[0][:3]), 0).astype(np.float32)
    act[-1] = 0.0                                   # an all-zero image: every later layer sees relu(bias)
    return act, shapes, w_np, b_np


@pytest.mark.parametrize("n_images", [1, 3])
@pytest.mark.parametrize("methods", ["cpo", "cps", "im2col", "mixed"])
def test_small_chain(api, methods, n_images):
    act, shapes, w_np, b_np = _small_chain(31, n_images)
    table = {"cpo": [api.ALGO_CPO] * 4, "cps": [api.ALGO_CPS] * 4, "im2col": [api.ALGO_IM2COL] * 4,
             "mixed": [api.ALGO_CPS, api.ALGO_IM2COL, api.ALGO_CPO, api.ALGO_IM2COL]}[methods]
    _say(f"[case] chain {methods} n={n_images}")
    _check_chain(api, act, shapes, w_np, b_np, table)


@pytest.mark.parametrize("n_images", [1, 8])
def test_chain_of_line_layers(api, n_images):
    """1 x 7 then 7 x 1 then 3 x 3 (the factorised 7 x 7 of the SI's layer tables): every layer
    keeps the 17 x 17 map, the first two with padding in one direction only."""
    rng = np.random.default_rng(41)
    shapes = [(36, 17, 17, 40, 1, 7, 1, 0, 3), (40, 17, 17, 70, 7, 1, 1, 3, 0), (70, 17, 17, 33, 3, 3, 1, 1)]
    w_np, b_np = [], []
    for i, s in enumerate(shapes):
        w_np.append((rng.standard_normal((s[3], s[0], s[4], s[5])) * np.sqrt(2.0 / (s[0] * s[4] * s[5]))).astype(np.float32))
        b_np.append(None if i == 0 else (0.3 * rng.standard_normal(s[0])).astype(np.float32))
    act = np.maximum(rng.standard_normal((n_images,) + shapes[0][:3]), 0).astype(np.float32)
    for table in ([api.ALGO_CPO] * 3, [api.ALGO_CPS, api.ALGO_IM2COL, api.ALGO_CPO]):
        _say(f"[case] chain of line layers n={n_images} {table}")
        _check_chain(api, act, shapes, w_np, b_np, table)


def test_chain_relu_in_front_of_the_first_layer_and_method_changes(api):
    """Layer 0 may itself read a pre-activation map; changing the methods reuses the buffers."""
    act, shapes, w_np, b_np = _small_chain(32, 2)
    rng = np.random.default_rng(33)
    act = rng.standard_normal(act.shape).astype(np.float32)
    b_np[0] = (0.2 * rng.standard_normal(shapes[0][0])).astype(np.float32)
    chain = _check_chain(api, act, shapes, w_np, b_np, [api.ALGO_CPO] * 4)
    first = [o.clone() for o in chain.outs]
    chain.set_methods([api.ALGO_CPS, api.ALGO_CPS, api.ALGO_IM2COL, api.ALGO_CPO])
    chain.forward(torch.from_numpy(act).cuda())
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(zip(first, chain.outs)):
        scale = float(a.abs().max())
        assert float((a - b).abs().max()) <= (i + 1) * FP32_TOL * scale
    assert torch.equal(first[0], chain.outs[0])     # CPS and CPO feed the same NZEs to the same kernel


def test_chain_workload_full_size(api):
    """The sixteen chained 3x3 layers of workload 5 at full size: all CPO, then a hybrid."""
    specs = workloads.chain_specs()
    shapes = [s.shape_tuple for s in specs]
    act, w_np, b_np = workloads.make_chain()
    _say("[case] chain workload, all CPO")
    _check_chain(api, act[None], shapes, w_np, b_np, [api.ALGO_CPO] * len(specs))
    _say("[case] chain workload, hybrid im2col / CPS / CPO")
    hybrid = [(api.ALGO_IM2COL, api.ALGO_CPS, api.ALGO_CPO)[i % 3] for i in range(len(specs))]
    _check_chain(api, act[None], shapes, w_np, b_np, hybrid)


def test_chain_workload_batched_bf16_comparator(api):
    """Two images through the chain with the bf16 comparator on every layer: the looser bound."""
    specs = workloads.chain_specs()[:7]
    shapes = [s.shape_tuple for s in specs]
    act0, w_np, b_np = workloads.make_chain()
    act1, _, _ = workloads.make_chain(1)
    _say("[case] chain workload, 7 layers, bf16 im2col, 2 images")
    _check_chain(api, np.stack([act0, act1]), shapes, w_np[:7], b_np[:7], [api.ALGO_IM2COL] * 7, tol=BF16_TOL, precision=1)
    _say("[case] the same with the bf16 kernel matrices prepared once")
    _check_chain(api, np.stack([act0, act1]), shapes, w_np[:7], b_np[:7], [api.ALGO_IM2COL] * 7, tol=BF16_TOL, precision=2)


def test_chain_workload_eight_images(api):
    """Eight images through the whole chained workload: the batched launch shapes of the sparse
    kernels (wide strips, workgroups shared by images, several kernels per lane) on chained data."""
    specs = workloads.chain_specs()
    shapes = [s.shape_tuple for s in specs]
    act0, w_np, b_np = workloads.make_chain()
    acts = np.stack([act0] + [workloads.make_activation(specs[0], m) for m in range(1, 8)])
    _say("[case] chain workload, 8 images, all CPO")
    _check_chain(api, acts, shapes, w_np, b_np, [api.ALGO_CPO] * len(specs))


def test_chain_replays_in_a_hip_graph(api):
    """A captured cpoconv_chain_forward (kernel launches only) replays on new inputs and gives,
    bit for bit, what the eager call gives; eager calls between the replays share its scratch."""
    acts, shapes, w_np, b_np = _small_chain(41, 2)
    ws = [torch.from_numpy(w).cuda() for w in w_np]
    bs = [None if b is None else torch.from_numpy(b).cuda() for b in b_np]
    methods = [api.ALGO_CPO, api.ALGO_IM2COL, api.ALGO_CPS, api.ALGO_CPO]
    chain = api.Chain(shapes, ws, bs, [b is not None for b in b_np], methods, n_images=2)
    act = torch.from_numpy(acts).cuda()
    chain.forward(act)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    _say("[case] chain graph capture")
    with torch.cuda.graph(graph):
        chain.forward(act)
    rng = np.random.default_rng(42)
    for rnd in range(3):
        new = np.maximum(rng.standard_normal(acts.shape), 0).astype(np.float32)
        act.copy_(torch.from_numpy(new))            # eager work between the replays
        chain.forward(act)
        torch.cuda.synchronize()
        eager = [o.clone() for o in chain.outs]
        for o in chain.outs:
            o.fill_(float("nan"))
        _say(f"[step] chain replay {rnd}")
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, chain.outs):
            assert torch.equal(a, b)
        table = [(s, w, b, b is not None) for s, w, b in zip(shapes, w_np, b_np)]
        ref = oracle.chain_forward(new[0], table)[-1]
        assert float(np.abs(chain.outs[-1][0].cpu().numpy() - ref).max()) <= 4 * FP32_TOL * float(np.abs(ref).max())
