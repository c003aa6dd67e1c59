"""GPU parity: the HIP path through the C ABI against the CPU oracle, on the same seeded inputs.

Encodings (ptr, DA, IN, side band, header) must match bit for bit; convolution outputs must
match the dense definition within max|err| <= 1e-4 * max|out| in fp32 (1e-2 for the bf16
im2col variant).  Tolerance: the GPU accumulates in fp32 over at most C*kh*kw <= 4608 terms in
a fixed order while the oracle accumulates in double; the error of such a sum is bounded by
about n * 2^-24 * sum|terms| and is in practice near sqrt(n) * 6e-8 * max|out| ~ 4e-6 * max|out|.
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


def _run_encoders(api, act_np, shape):
    buf = api.LayerBuffers(shape)
    act = torch.from_numpy(act_np).cuda()
    api.cpo_encode(act, shape, buf.cpo, buf.scratch)
    api.cps_encode(act, shape, buf.cps, buf.scratch)
    torch.cuda.synchronize()
    return buf, act


def _assert_same_map(got, ref, algo_code):
    ptr, da, ind, chan_off, hdr = got
    assert hdr[7] == 0                                                     # no encoder workgroup gave up
    assert hdr[0] == ref.ptr.size and hdr[1] == ref.da.size and hdr[2] == ref.ind.size
    assert hdr[3] == algo_code
    assert np.array_equal(ptr, ref.ptr)
    assert np.array_equal(da.view(np.int32), ref.da.view(np.int32))      # bit for bit
    assert np.array_equal(ind, ref.ind)
    assert np.array_equal(chan_off, ref.chan_off)


def _check_layer(api, act_np, w_np, shape, convs=True, name=""):
    _say(f"[case] {name} shape={tuple(shape)}")
    buf, act = _run_encoders(api, act_np, shape)
    ref_cpo, ref_cps = oracle.cpo_encode(act_np, shape), oracle.cps_encode(act_np, shape)
    _assert_same_map(buf.cpo.to_host(), ref_cpo, api.ALGO_CPO)
    _assert_same_map(buf.cps.to_host(), ref_cps, api.ALGO_CPS)
    if not convs:
        return
    ref = oracle.conv_direct(act_np, w_np, shape)
    scale = max(float(np.abs(ref).max()), 1e-30)
    w = torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    for label, fn, m in (("cpo", api.cpo_conv, buf.cpo), ("cps", api.cps_conv, buf.cps)):
        _say(f"[step] {label}_conv")
        buf.out.fill_(float("nan"))                   # the call must overwrite, not accumulate
        fn(m, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        got = buf.out.cpu().numpy()
        err = float(np.abs(got - ref).max())
        assert np.isfinite(got).all(), label
        assert err <= FP32_TOL * scale, (label, err, scale)
    # encoding + convolution in one call: the same streams and the same output, bit for bit
    for label, fused, conv, m, ref_map, code in (("cpo", api.cpo_encode_conv, api.cpo_conv, buf.cpo, ref_cpo, api.ALGO_CPO),
                                                 ("cps", api.cps_encode_conv, api.cps_conv, buf.cps, ref_cps, api.ALGO_CPS)):
        _say(f"[step] {label}_encode_conv")
        conv(m, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        separate = buf.out.clone()
        m.da.fill_(-3.0)
        buf.out.fill_(float("nan"))
        fused(act, shape, m, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        _assert_same_map(m.to_host(), ref_map, code)
        assert torch.equal(buf.out, separate), label
    for prec, tol in ((0, FP32_TOL), (1, BF16_TOL)):
        _say(f"[step] im2col_conv precision={prec}")
        buf.out.fill_(float("nan"))
        api.im2col_conv(act, shape, w, buf.lowered, buf.out, prec)
        torch.cuda.synchronize()
        got = buf.out.cpu().numpy()
        err = float(np.abs(got - ref).max())
        assert np.isfinite(got).all(), prec
        assert err <= tol * scale, (prec, err, scale)
    # the bf16 kernel matrix prepared once: the same product, bit for bit
    _say("[step] im2col_conv precision=2")
    rounded = buf.out.clone()
    api.im2col_prepare_weights_bf16(w, shape, buf.wb)
    buf.out.fill_(float("nan"))
    api.im2col_conv(act, shape, buf.wb, buf.lowered, buf.out, 2)
    torch.cuda.synchronize()
    assert torch.equal(buf.out, rounded)


# --- the five workloads at full size ------------------------------------------------------
WORKLOAD_LAYERS = workloads.layers(1) + workloads.layers(2) + workloads.layers(3) + workloads.layers(4)
CFG5 = workloads.layers(5)


@pytest.mark.parametrize("spec", WORKLOAD_LAYERS, ids=lambda s: s.name)
def test_workloads_1_to_4(api, spec):
    act, w = workloads.make_layer(spec)
    _check_layer(api, act, w, spec.shape_tuple, name=spec.name)


@pytest.mark.parametrize("spec", CFG5, ids=lambda s: s.name)
def test_workload_5_layers(api, spec):
    act, w = workloads.make_layer(spec)
    _check_layer(api, act, w, spec.shape_tuple, name=spec.name)


@pytest.mark.parametrize("spec", workloads.line_layers(), ids=lambda s: s.name)
def test_line_layers(api, spec):
    """The 1 x n / n x 1 layers at full size, one image (register-tile kernel)."""
    act, w = workloads.make_layer(spec)
    _check_layer(api, act, w, spec.shape_tuple, name=spec.name)


# --- edge cases: ragged tiles, strides, paddings, degenerate geometries ----------------------
EDGE_SHAPES = [
    (1, 4, 4, 1, 3, 3, 1, 1),
    (3, 7, 9, 2, 3, 3, 1, 1),
    (2, 8, 8, 3, 4, 4, 1, 1),
    (2, 9, 10, 65, 5, 5, 1, 2),      # K just above one wavefront of kernels
    (3, 10, 11, 2, 3, 3, 2, 1),
    (2, 11, 8, 2, 3, 2, 3, 0),
    (2, 12, 13, 2, 7, 7, 2, 3),
    (4, 6, 5, 2, 1, 3, 1, 0),
    (2, 5, 6, 2, 3, 1, 1, 0),        # kw = 1: no overlap at all
    (2, 6, 3, 2, 3, 3, 1, 0),        # Ow = 1
    (2, 6, 4, 2, 3, 3, 1, 0),        # Ow = 2 < kw: no overlap-kw type
    (3, 13, 9, 2, 3, 5, 2, 2),
    (2, 9, 9, 2, 3, 3, 1, 2),        # more padding than overlap
    (5, 17, 19, 70, 3, 3, 1, 0),     # VALID padding: three-entry NOP segment
    (3, 70, 33, 4, 3, 3, 1, 1),      # more than 64 padded rows: two row chunks
    (2, 33, 130, 4, 5, 3, 1, 1),     # wide map
    (1, 254, 254, 2, 3, 3, 1, 1),    # largest supported map
    (2, 30, 30, 3, 11, 11, 4, 2),    # largest kernel, stride 4
    (2, 16, 16, 130, 2, 2, 2, 0),
    # more than 16 channels: the register-tile kernel rather than the strip kernel
    (20, 9, 11, 66, 3, 3, 1, 1),
    (18, 13, 9, 3, 3, 3, 2, 1),
    (17, 15, 14, 5, 7, 7, 2, 3),
    (40, 30, 29, 70, 3, 3, 1, 1),     # several channel slices, ragged tiles
    (33, 21, 37, 4, 3, 3, 1, 0),      # VALID padding in the register-tile kernel
    (520, 5, 6, 3, 3, 3, 1, 1),       # more channels than the encoder's single-launch look-back takes
    (520, 40, 38, 3, 3, 3, 1, 1),     # the same on a map the workgroup-per-channel encoder takes: its two-launch form
    (24, 62, 60, 130, 3, 3, 1, 1),    # 64 padded rows: the column-run kernel's bitmaps full to the last bit
    (130, 28, 28, 128, 3, 3, 1, 1),   # column-run kernel with channel slices and the slice sum
    # shapes without an instantiation of the fast kernels: the general kernel, with channel slices
    (40, 20, 20, 70, 4, 4, 1, 1),
    (33, 19, 19, 5, 5, 5, 2, 2),
    (24, 15, 15, 66, 7, 7, 1, 3),
    (5, 15, 17, 70, 3, 3, 2, 1),      # strip kernel, stride 2, two kernels per lane, ragged
    (3, 17, 17, 70, 7, 1, 1, 0),      # 7 x 1 kernel: the K_w = 1 special case of the SI
    (6, 8, 8, 5, 3, 1, 1, 0),         # 3 x 1
    (3, 17, 17, 4, 1, 7, 1, 0),       # 1 x 7 (K_h = 1): the general algorithm
    # rows and columns padded differently (.., stride, pad_h, pad_w): the 1 x n and n x 1 layers
    # that keep their map size, and 3 x 3 layers padded in one direction only
    (3, 17, 17, 70, 7, 1, 1, 3, 0),
    (3, 17, 17, 4, 1, 7, 1, 0, 3),
    (6, 8, 9, 5, 3, 1, 1, 1, 0),
    (6, 8, 9, 5, 1, 3, 1, 0, 1),
    (33, 17, 17, 70, 7, 1, 1, 3, 0),
    (33, 17, 17, 70, 1, 7, 1, 0, 3),
    (20, 9, 11, 66, 3, 3, 1, 0, 1),   # register-tile kernel, columns padded only
    (20, 9, 11, 66, 3, 3, 1, 2, 0),   # rows padded, columns not: three-entry NOP segment
    (5, 15, 17, 70, 3, 3, 2, 0, 1),   # strip kernel, stride 2
    (3, 70, 33, 4, 3, 3, 1, 0, 2),    # two row chunks in the encoder, no row padding
    (2, 30, 30, 3, 11, 5, 2, 5, 1),
    (40, 8, 8, 70, 1, 3, 1, 0, 1),
    (40, 8, 8, 70, 3, 1, 1, 1, 0),
    (33, 17, 19, 70, 1, 7, 1, 0, 0),  # 1 x 7 without padding: three-entry NOP segment, six overlap types
    (33, 19, 17, 70, 7, 1, 1, 0, 0),
    (33, 17, 19, 5, 1, 7, 1, 1, 2),   # padding narrower than the kernel's reach, rows padded too
    (20, 15, 17, 70, 3, 3, 2, 1),     # column-run kernel at stride 2: odd map, ragged 3 x 3 tiles
    (130, 30, 30, 128, 3, 3, 2, 1),   # the same, channel slices, two kernels per lane, last padded column unused
    (8, 61, 61, 130, 3, 3, 2, 1),     # 63 padded rows
    (24, 16, 16, 64, 3, 3, 2, 0),     # stride 2 without padding: a column of the map under no kernel position
    (24, 17, 15, 64, 3, 3, 2, 0),
    (20, 13, 17, 70, 5, 5, 1, 2),     # column-run kernel, 5 x 5: an 8 x 8 window fills the wavefront
    (70, 27, 27, 192, 5, 5, 1, 2),
    (24, 30, 29, 64, 5, 5, 1, 0),     # without padding
    (9, 60, 60, 130, 5, 5, 1, 2),     # 64 padded rows and columns
    (3, 64, 64, 64, 3, 3, 1, 0),      # band encoder in front of the column-run kernel: the column table rebuilt from its offsets
    (2, 64, 64, 130, 3, 3, 2, 0),
]


@pytest.mark.parametrize("shape", EDGE_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("zero_frac", [0.0, 0.55, 0.93])
def test_edge_shapes(api, shape, zero_frac):
    act, w = workloads.random_case(91, *shape[:8], zero_frac=zero_frac, zero_channels=1 if shape[0] > 2 else 0)
    _check_layer(api, act, w, shape, name=f"edge z={zero_frac}")


def test_all_zero_map(api):
    shape = (5, 12, 12, 8, 3, 3, 1, 1)
    act = np.zeros((5, 12, 12), np.float32)
    act[2, 3, 4] = -0.0                               # a negative zero is a zero
    _, w = workloads.random_case(1, *shape, zero_frac=0.5)
    _say("[case] all-zero map")
    buf, _ = _run_encoders(api, act, shape)
    ptr, da, ind, chan_off, hdr = buf.cpo.to_host()
    assert ptr.tolist() == [api.NPC] * 5 and da.size == 0 and ind.size == 0
    _check_layer(api, act, w, shape, name="all-zero")
    api.cpoconv_prepare_weights(torch.from_numpy(w).cuda(), shape, buf.wt)
    buf.out.fill_(7.0)
    api.cpo_conv(buf.cpo, shape, buf.wt, buf.out, buf.scratch)
    torch.cuda.synchronize()
    assert float(buf.out.abs().max()) == 0.0


def test_special_values_are_non_zero_elements(api):
    shape = (2, 9, 9, 2, 3, 3, 1, 1)
    act, _ = workloads.random_case(4, *shape, zero_frac=0.7)
    act[0, 1, 1] = np.float32(1e-45)                  # denormal
    act[0, 2, 5] = np.float32(-1e-40)
    act[1, 4, 4] = np.float32("nan")
    act[1, 0, 8] = np.float32("inf")
    _check_layer(api, act, None, shape, convs=False, name="special values")


def test_integer_valued_layer_is_exact(api):
    # small integers: every fp32 sum is exact, so the sparse and dense paths must agree exactly
    for shape in [(6, 20, 21, 70, 3, 3, 1, 1), (4, 15, 14, 5, 5, 5, 1, 2), (4, 19, 18, 5, 3, 3, 2, 1)]:
        act, w = workloads.random_case(8, *shape, zero_frac=0.6, zero_channels=1, integer=True)
        _say(f"[case] integer-valued {shape}")
        buf, a = _run_encoders(api, act, shape)
        ref = oracle.conv_direct(act, w, shape)
        wd = torch.from_numpy(w).cuda()
        api.cpoconv_prepare_weights(wd, shape, buf.wt)
        api.cpo_conv(buf.cpo, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        assert np.array_equal(buf.out.cpu().numpy(), ref)
        api.cps_conv(buf.cps, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        assert np.array_equal(buf.out.cpu().numpy(), ref)
        api.im2col_conv(a, shape, wd, buf.lowered, buf.out, 0)
        torch.cuda.synchronize()
        assert np.array_equal(buf.out.cpu().numpy(), ref)


def test_results_are_bitwise_repeatable(api):
    spec = workloads.layers(3)[0]
    act, w = workloads.make_layer(spec)
    shape = spec.shape_tuple
    _say("[case] repeatability")
    outs = []
    for _ in range(2):
        buf, _a = _run_encoders(api, act, shape)
        api.cpoconv_prepare_weights(torch.from_numpy(w).cuda(), shape, buf.wt)
        api.cps_conv(buf.cps, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        outs.append((buf.out.cpu().numpy().copy(), [t.copy() for t in buf.cps.to_host()[:3]]))
    assert np.array_equal(outs[0][0].view(np.int32), outs[1][0].view(np.int32))
    for a, b in zip(outs[0][1], outs[1][1]):
        assert np.array_equal(a.view(np.int32), b.view(np.int32))


def test_runs_on_a_side_stream(api):
    shape = (8, 14, 14, 16, 3, 3, 1, 1)
    act, w = workloads.random_case(2, *shape, zero_frac=0.6)
    _say("[case] side stream")
    st = torch.cuda.Stream()
    buf = api.LayerBuffers(shape)
    a, wd = torch.from_numpy(act).cuda(), torch.from_numpy(w).cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        api.cpo_encode(a, shape, buf.cpo, buf.scratch, stream=st)
        api.cpoconv_prepare_weights(wd, shape, buf.wt, stream=st)
        api.cpo_conv(buf.cpo, shape, buf.wt, buf.out, buf.scratch, stream=st)
    st.synchronize()
    ref = oracle.conv_direct(act, w, shape)
    assert float(np.abs(buf.out.cpu().numpy() - ref).max()) <= FP32_TOL * float(np.abs(ref).max())


def test_selection_end_to_end_on_measured_times(api):
    # Section 3.5 on one small layer: time the three methods on M = 5 inputs, select
    spec = workloads.layers(1)[0]
    shape = spec.shape_tuple
    buf = api.LayerBuffers(shape)
    w = torch.from_numpy(workloads.make_weights(spec)).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    _say("[case] selection")
    times = {"im2col": [], "cpo": [], "cps": []}
    for m in range(5):
        act = torch.from_numpy(workloads.make_activation(spec, m)).cuda()
        for key in times:
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            ev0.record()
            if key == "im2col":
                api.im2col_conv(act, shape, w, buf.lowered, buf.out, 0)
            elif key == "cpo":
                api.cpo_encode(act, shape, buf.cpo, buf.scratch)
                api.cpo_conv(buf.cpo, shape, buf.wt, buf.out, buf.scratch)
            else:
                api.cps_encode(act, shape, buf.cps, buf.scratch)
                api.cps_conv(buf.cps, shape, buf.wt, buf.out, buf.scratch)
            ev1.record()
            torch.cuda.synchronize()
            times[key].append(ev0.elapsed_time(ev1))
    for mode, sparse in ((0, "cpo"), (1, "cps")):
        algo = api.select_layer_algo(times["im2col"], times["cpo"], times["cps"], mode)
        assert algo == oracle.select_layer_algo(times["im2col"], times["cpo"], times["cps"], mode)
        expect = {0: api.ALGO_CPO, 1: api.ALGO_CPS}[mode] if sum(times[sparse]) < sum(times["im2col"]) else api.ALGO_IM2COL
        assert algo == expect


# --- batched calls: n_images maps per launch, every image equal to its single-image result ----
BATCH_CASES = [
    # (n_images, shape) - strip kernel / register-tile kernel / generic kernel, ragged tiles, strides
    (3, (5, 12, 13, 70, 3, 3, 1, 1)),
    (4, (20, 9, 11, 66, 3, 3, 1, 1)),
    (2, (18, 13, 9, 3, 3, 3, 2, 1)),
    (3, (3, 10, 12, 4, 5, 5, 1, 2)),
    (2, (2, 30, 30, 3, 11, 11, 4, 2)),
    (5, (33, 21, 37, 4, 3, 3, 1, 0)),
    (40, (4, 8, 8, 5, 3, 3, 1, 1)),               # enough images that no layer is sliced over channels
    (2, (3, 70, 33, 4, 3, 3, 1, 1)),
    (1024, (2, 5, 6, 3, 3, 3, 1, 1)),             # the largest batch the calls take
    # mid-sized maps with >= 1024 channel-images: the one-wavefront-per-channel encoder, in one
    # launch and (more than 512 channels) in two
    (3, (400, 20, 22, 3, 3, 3, 1, 1)),
    (2, (600, 19, 37, 2, 3, 3, 1, 0)),
    (130, (3, 40, 38, 4, 3, 3, 1, 1)),            # more images than one launch's look-back slots: two launches
    (3, (24, 30, 30, 70, 3, 3, 1, 1)),            # three images through the column-run kernel
    (3, (20, 12, 13, 70, 4, 4, 1, 1)),            # the general kernel with channel slices, three images
    # several images of small 3 x 3 maps: strips of two or four tiles per workgroup, stride 1 and 2,
    # one and two kernels per lane
    (4, (40, 14, 14, 128, 3, 3, 1, 1)),
    (4, (33, 28, 28, 70, 3, 3, 1, 1)),            # two seven-column tiles per strip
    (4, (32, 55, 56, 128, 3, 3, 2, 1)),           # the same at stride 2, two kernels per lane
    (8, (36, 13, 9, 70, 3, 3, 2, 1)),             # four images per workgroup
    (8, (32, 27, 30, 128, 3, 3, 2, 1)),           # stride 2, four tiles per strip
    (9, (33, 7, 7, 64, 3, 3, 1, 1)),              # four images per workgroup, the last workgroup with one
    (4, (32, 29, 31, 64, 3, 3, 2, 0)),            # wide strips without padding (three-entry NOP segments)
    (4, (32, 12, 12, 64, 3, 3, 1, 2)),            # padding wider than the overlap: a single overlap type
    # 256 kernels or a multiple, eight workgroups or more: four kernels per lane (strips of 4, 2, 1 tiles)
    (8, (33, 14, 14, 256, 3, 3, 1, 1)),
    (16, (32, 7, 7, 512, 3, 3, 1, 1)),
    (4, (32, 28, 28, 256, 3, 3, 1, 1)),
    (4, (32, 40, 22, 250, 3, 3, 1, 1)),
    (4, (32, 80, 22, 256, 3, 3, 2, 1)),
    # several images of wide maps: tiles of eight columns, or seven where seven divides the width
    (4, (6, 50, 52, 70, 3, 3, 1, 1)),
    (4, (5, 46, 47, 128, 3, 3, 1, 1)),
    (4, (6, 47, 49, 70, 3, 3, 1, 1)),
    (4, (5, 56, 56, 128, 3, 3, 1, 1)),
    # rows and columns padded differently
    (4, (40, 14, 14, 128, 3, 3, 1, 0, 1)),
    (4, (33, 28, 28, 70, 3, 3, 1, 2, 1)),
    (8, (33, 17, 17, 70, 1, 7, 1, 0, 3)),
    (8, (33, 17, 17, 70, 7, 1, 1, 3, 0)),
    (4, (5, 56, 56, 128, 3, 3, 1, 1, 0)),
    # 1 x 7 / 7 x 1: one strip of three six-column tiles; 1 x 3 / 3 x 1: two four-column tiles,
    # four images per workgroup; one and two kernels per lane
    (4, (40, 17, 17, 128, 7, 1, 1, 3, 0)),
    (4, (40, 17, 15, 128, 1, 7, 1, 0, 3)),
    (4, (40, 18, 18, 70, 1, 7, 1, 0, 3)),
    (4, (40, 13, 13, 70, 7, 1, 1, 3, 0)),
    (4, (36, 17, 19, 70, 1, 7, 1, 0, 0)),         # without padding: output 13 wide, three-entry NOP segment
    (8, (40, 8, 8, 128, 1, 3, 1, 0, 1)),
    (9, (33, 8, 7, 70, 3, 1, 1, 1, 0)),
    (8, (40, 8, 8, 70, 3, 1, 1, 0, 0)),
    (4, (36, 17, 17, 160, 1, 7, 1, 0, 3)),        # 160 kernels pad to 192: three kernels per lane
    (4, (36, 17, 17, 192, 7, 1, 1, 3, 0)),
    (8, (36, 8, 8, 384, 1, 3, 1, 0, 1)),
    (8, (36, 8, 8, 180, 3, 1, 1, 1, 0)),
    # 3 x 3 with three kernels per lane (kernel counts that pad to a multiple of 192)
    (4, (33, 17, 17, 192, 3, 3, 1, 1)),
    (8, (36, 8, 8, 384, 3, 3, 1, 1)),
    (4, (33, 17, 17, 160, 3, 3, 2, 1)),
    (3, (33, 17, 17, 160, 3, 3, 2, 1)),           # column-run kernel at stride 2, three images
    (2, (130, 29, 30, 128, 3, 3, 2, 1)),
    (3, (20, 13, 17, 70, 5, 5, 1, 2)),            # column-run kernel, 5 x 5
    (40, (52, 36, 35, 6, 3, 3, 1, 1)),            # 2080 channel-images on a map beyond 4 KiB: four-wavefront encoder workgroups
    (36, (60, 40, 38, 4, 5, 5, 1, 2)),            # the same: five overlap types, 44 padded rows
    (34, (64, 33, 34, 4, 3, 3, 2, 0)),            # stride 2 without padding
    (4, (520, 40, 38, 3, 3, 3, 1, 1)),            # and in two launches (more than 512 channels)
    (33, (64, 62, 60, 2, 3, 3, 1, 1)),            # 64 padded rows: sixteen rows per wavefront, all of them used
    (4, (33, 30, 31, 190, 3, 3, 1, 1)),
    # 5 x 5 with two and three kernels per lane
    (4, (20, 27, 27, 192, 5, 5, 1, 2)),
    (4, (20, 13, 14, 128, 5, 5, 1, 2)),
]


def _batch_inputs(n_images, shape, seed):
    acts = []
    for n in range(n_images):
        # densities differ per image; image 1 is all zero, so its streams are empty
        act, w = workloads.random_case(seed + n, *shape[:8], zero_frac=(0.3, 0.9, 0.6)[n % 3],
                                       zero_channels=1 if shape[0] > 2 else 0)
        if n == 1:
            act[...] = 0.0
        acts.append(act)
    return np.stack(acts), w


@pytest.mark.parametrize("case", BATCH_CASES, ids=lambda c: f"n{c[0]}-" + "x".join(map(str, c[1])))
def test_batched_calls(api, case):
    n_images, shape = case
    acts, w_np = _batch_inputs(n_images, shape, 505)
    _say(f"[case] batch n={n_images} shape={shape}")
    buf = api.LayerBuffers(shape, n_images=n_images)
    act = torch.from_numpy(acts).cuda()
    w = torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    api.cpo_encode_batch(act, shape, buf.cpo, buf.scratch)
    api.cps_encode_batch(act, shape, buf.cps, buf.scratch)
    torch.cuda.synchronize()
    refs = []
    for n in range(n_images):
        _assert_same_map(buf.cpo.to_host(image=n), oracle.cpo_encode(acts[n], shape), api.ALGO_CPO)
        _assert_same_map(buf.cps.to_host(image=n), oracle.cps_encode(acts[n], shape), api.ALGO_CPS)
        refs.append(oracle.conv_direct(acts[n], w_np, shape))
    ref = np.stack(refs)
    scale = max(float(np.abs(ref).max()), 1e-30)
    for label, fn, m in (("cpo", api.cpo_conv_batch, buf.cpo), ("cps", api.cps_conv_batch, buf.cps)):
        _say(f"[step] {label}_conv_batch")
        buf.out.fill_(float("nan"))
        fn(m, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        got = buf.out.cpu().numpy().reshape(ref.shape)
        assert np.isfinite(got).all(), label
        assert float(np.abs(got - ref).max()) <= FP32_TOL * scale, label
    for label, fused, m in (("cpo", api.cpo_encode_conv, buf.cpo), ("cps", api.cps_encode_conv, buf.cps)):
        _say(f"[step] {label}_encode_conv (batched)")
        buf.out.fill_(float("nan"))
        fused(act, shape, m, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        got = buf.out.cpu().numpy().reshape(ref.shape)
        assert np.isfinite(got).all(), label
        assert float(np.abs(got - ref).max()) <= FP32_TOL * scale, label
    for prec, tol in ((0, FP32_TOL), (1, BF16_TOL)):
        _say(f"[step] im2col_conv_batch precision={prec}")
        buf.out.fill_(float("nan"))
        api.im2col_conv_batch(act, shape, n_images, w, buf.lowered, buf.out, prec)
        torch.cuda.synchronize()
        got = buf.out.cpu().numpy().reshape(ref.shape)
        assert np.isfinite(got).all(), prec
        assert float(np.abs(got - ref).max()) <= tol * scale, prec
    _say("[step] im2col_conv_batch precision=2")
    rounded = buf.out.clone()
    api.im2col_prepare_weights_bf16(w, shape, buf.wb)
    buf.out.fill_(float("nan"))
    api.im2col_conv_batch(act, shape, n_images, buf.wb, buf.lowered, buf.out, 2)
    torch.cuda.synchronize()
    assert torch.equal(buf.out, rounded)


def test_batched_workload_layers(api):
    """Two workload layers at full size with eight images each, sampled against the oracle."""
    for name, n_images in (("cfg3.256@14", 8), ("cfg5.l05.128@28s1", 8), ("line.1x7.160to160@17", 8),
                           ("line.7x1.128to192@17", 8), ("line.3x1.384to384@8", 8)):
        spec = {s.name: s for s in workloads.all_layers() + workloads.line_layers()}[name]
        shape = spec.shape_tuple
        _say(f"[case] batched {name} n={n_images}")
        acts = np.stack([workloads.make_activation(spec, m) for m in range(n_images)])
        w_np = workloads.make_weights(spec)
        buf = api.LayerBuffers(shape, n_images=n_images)
        act, w = torch.from_numpy(acts).cuda(), torch.from_numpy(w_np).cuda()
        api.cpoconv_prepare_weights(w, shape, buf.wt)
        api.cpo_encode_batch(act, shape, buf.cpo, buf.scratch)
        api.cpo_conv_batch(buf.cpo, shape, buf.wt, buf.out, buf.scratch)
        torch.cuda.synchronize()
        got = buf.out.cpu().numpy()
        for n in (0, n_images - 1):
            _assert_same_map(buf.cpo.to_host(image=n), oracle.cpo_encode(acts[n], shape), api.ALGO_CPO)
            ref = oracle.conv_direct(acts[n], w_np, shape)
            assert float(np.abs(got[n] - ref).max()) <= FP32_TOL * float(np.abs(ref).max())


# --- the scratch buffer: prepared once, shared between shapes -------------------------------------
def test_scratch_shared_between_shapes(api):
    """One scratch buffer serves layers of different channel counts in turn (the encoders' epoch
    and stream-length words live in it)."""
    shapes = [(40, 30, 29, 7, 3, 3, 1, 1), (3, 7, 9, 2, 3, 3, 1, 1), (20, 9, 11, 66, 3, 3, 1, 1)]
    sizes = [api.cpoconv_sizes(s).scratch_bytes for s in shapes]
    scratch = torch.empty(max(sizes), dtype=torch.uint8, device="cuda")
    api.cpoconv_scratch_init(scratch)
    for rnd in range(3):
        for i, shape in enumerate(shapes):
            act_np, _ = workloads.random_case(700 + 10 * rnd + i, *shape, zero_frac=0.6, zero_channels=1)
            _say(f"[case] shared scratch round {rnd} shape={shape}")
            m = api.EncodedMap(shape)
            api.cps_encode(torch.from_numpy(act_np).cuda(), shape, m, scratch)
            _assert_same_map(m.to_host(), oracle.cps_encode(act_np, shape), api.ALGO_CPS)


def test_layer_call_replays_in_a_hip_graph(api):
    """A captured cpo_encode_conv + im2col_conv replays correctly on new inputs: the library queues
    kernels only (no memset nodes), and the encoder's epoch lives on the device, so a replay is a new call."""
    shape = (24, 20, 19, 70, 3, 3, 1, 1)
    inputs = [workloads.random_case(800 + i, *shape, zero_frac=z, zero_channels=2)[0] for i, z in enumerate((0.5, 0.8, 0.3, 0.6))]
    _, w_np = workloads.random_case(800, *shape, zero_frac=0.5)
    buf = api.LayerBuffers(shape)
    w = torch.from_numpy(w_np).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    act = torch.from_numpy(inputs[0]).cuda()
    out_dense = torch.empty_like(buf.out)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    _say("[case] graph capture")
    with torch.cuda.graph(graph):
        api.cpo_encode_conv(act, shape, buf.cpo, buf.wt, buf.out, buf.scratch)
        api.im2col_conv(act, shape, w, buf.lowered, out_dense, 0)
    for rnd, act_np in enumerate(inputs):
        _say(f"[step] replay {rnd}")
        act.copy_(torch.from_numpy(act_np))          # eager work between the replays
        buf.out.fill_(float("nan"))
        out_dense.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.conv_direct(act_np, w_np, shape)
        scale = float(np.abs(ref).max())
        _assert_same_map(buf.cpo.to_host(), oracle.cpo_encode(act_np, shape), api.ALGO_CPO)
        assert float(np.abs(buf.out.cpu().numpy() - ref).max()) <= FP32_TOL * scale
        assert float(np.abs(out_dense.cpu().numpy() - ref).max()) <= FP32_TOL * scale
        # an eager call between replays shares the scratch buffer and the epoch
        api.cps_encode(act, shape, buf.cps, buf.scratch)
        _assert_same_map(buf.cps.to_host(), oracle.cps_encode(act_np, shape), api.ALGO_CPS)
