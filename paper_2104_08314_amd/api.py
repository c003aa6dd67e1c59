"""Thin ctypes binding of libcpoconv (include/cpoconv.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch supplies device memory and
the stream.  There is no fallback: without the built library every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcpoconv.so")

ALGO_IM2COL, ALGO_CPO, ALGO_CPS = 0, 1, 2
NPF, NPC = -2, -3
ERR_NULL, ERR_SHAPE, ERR_SMALL, ERR_HIP, ERR_ALGO, ERR_MAP = -1, -2, -3, -4, -5, -6
LAYOUT_CHW, LAYOUT_HWC = 0, 1
MAX_I = 256


class CpoconvError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"cpoconv error {code}: {message}")
        self.code = code


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("C", "H", "W", "K", "kh", "kw", "stride", "pad_h", "pad_w", "layout")]

    def as_tuple(self) -> Tuple[int, ...]:
        return tuple(int(getattr(self, n)) for n, _ in self._fields_)


class _Map(ctypes.Structure):
    _fields_ = [
        ("ptr", ctypes.c_void_p), ("ptr_cap", ctypes.c_int64),
        ("da", ctypes.c_void_p), ("da_cap", ctypes.c_int64),
        ("ind", ctypes.c_void_p), ("in_cap", ctypes.c_int64),
        ("chan_off", ctypes.c_void_p), ("hdr", ctypes.c_void_p), ("in_bits", ctypes.c_int32),
    ]


class Sizes(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("ptr_cap", "da_cap", "in_cap", "chan_off_len", "wt_len",
                                               "out_len", "lowered_bytes", "scratch_bytes", "wb_len")] + \
               [("Oh", ctypes.c_int32), ("Ow", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (no CPU or PyTorch fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2104_08314_amd.build`; "
                "this package has no fallback path")
        # PyTorch ships its own HIP runtime (same soname as the system one).  Import it first so
        # that this library binds to the runtime that owns PyTorch's device memory and streams;
        # two HIP runtimes in one process do not see each other's devices.
        import torch  # noqa: F401

        _lib = ctypes.CDLL(LIB_PATH)
        _lib.cpoconv_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            getattr(_lib, name)  # fail loudly on a missing symbol
    return _lib


EXPORTS = (
    "cpoconv_sizes", "cpo_encode", "cps_encode", "cpoconv_prepare_weights", "cpo_conv", "cps_conv",
    "im2col_conv", "select_layer_algo", "cpoconv_map_header_to_host", "cpoconv_geometry",
    "cpoconv_strerror", "cpoconv_last_hip_error", "cpoconv_kernel_timing", "cpoconv_kernel_timing_read",
    "cpoconv_scratch_init", "cpoconv_batch_sizes", "cpo_encode_batch", "cps_encode_batch", "cpo_conv_batch", "cps_conv_batch",
    "im2col_conv_batch", "im2col_prepare_weights_bf16", "cpo_encode_conv", "cps_encode_conv", "cpo_encode_conv_batch", "cps_encode_conv_batch",
    "cpo_encode_relu", "cps_encode_relu", "im2col_conv_relu", "cpoconv_chain_sizes", "cpoconv_chain_forward",
    "cpo_encode_static_scratch",
)


def cpoconv_strerror(code: int) -> str:
    return lib().cpoconv_strerror(int(code)).decode()


def cpoconv_kernel_timing(enable: bool) -> None:
    """Measurement aid: bracket every kernel launch of the library with HIP events."""
    _check(lib().cpoconv_kernel_timing(1 if enable else 0))


def cpoconv_kernel_timing_read():
    """{kernel name: (average microseconds, launches)} recorded since timing was enabled."""
    out = {}
    name = ctypes.create_string_buffer(64)
    avg, calls = ctypes.c_double(0.0), ctypes.c_int(0)
    i = 0
    while True:
        rc = lib().cpoconv_kernel_timing_read(i, name, 64, ctypes.byref(avg), ctypes.byref(calls))
        if rc == ERR_SHAPE:
            break
        _check(rc)
        out[name.value.decode()] = (float(avg.value), int(calls.value))
        i += 1
    return out


def _check(rc: int) -> None:
    if rc != 0:
        msg = cpoconv_strerror(rc)
        if rc == ERR_HIP:
            msg += f" (hipError {lib().cpoconv_last_hip_error()})"
        raise CpoconvError(rc, msg)


def make_shape(shape) -> Shape:
    if isinstance(shape, Shape):
        return shape
    # (C, H, W, K, kh, kw, stride, pad) pads rows and columns alike; a ninth entry gives the
    # columns their own padding: (.., stride, pad_h, pad_w); a tenth the layout of the dense input
    # map: LAYOUT_CHW (default) or LAYOUT_HWC
    v = [int(x) for x in shape]
    if len(v) == 8:
        v.append(v[7])
    if len(v) == 9:
        v.append(LAYOUT_CHW)
    if len(v) != 10:
        raise ValueError("a shape has eight to ten entries: (C, H, W, K, kh, kw, stride, pad_h[, pad_w[, layout]])")
    return Shape(*v)


def cpoconv_sizes(shape) -> Sizes:
    sz = Sizes()
    sh = make_shape(shape)
    _check(lib().cpoconv_sizes(ctypes.byref(sh), ctypes.byref(sz)))
    return sz


def cpoconv_geometry(shape):
    """Host-side partition / overlap-type table: (info dict, per-column int arrays)."""
    sh = make_shape(shape)
    info = (ctypes.c_int32 * 8)()
    cols = [np.zeros(MAX_I, np.int32) for _ in range(4)]
    _check(lib().cpoconv_geometry(ctypes.byref(sh), info, *[c.ctypes.data_as(ctypes.c_void_p) for c in cols]))
    keys = ("Ih", "Iw", "Oh", "Ow", "n_cols", "n_types", "nop3", "top")
    d = {k: int(v) for k, v in zip(keys, info)}
    n = d["n_cols"]
    return d, {"j": cols[0][:n], "type": cols[1][:n], "p0": cols[2][:n], "what": cols[3][:n]}


def select_layer_algo(t_im2col: Sequence[float], t_cpo: Optional[Sequence[float]],
                      t_cps: Optional[Sequence[float]], mode: int) -> int:
    def arr(t):
        if t is None:
            return None, None
        a = (ctypes.c_double * len(t))(*[float(v) for v in t])
        return a, len(t)
    a, n = arr(t_im2col)
    b, _ = arr(t_cpo)
    c, _ = arr(t_cps)
    out = ctypes.c_int(-1)
    _check(lib().select_layer_algo(a, b, c, int(n or 0), int(mode), ctypes.byref(out)))
    return int(out.value)


# ----------------------------------------------------------------------------------------
# device-side calls (torch tensors supply the memory)
# ----------------------------------------------------------------------------------------

def _stream_handle(stream) -> ctypes.c_void_p:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _weights_ptr(weights, precision: int) -> ctypes.c_void_p:
    """im2col weights: fp32 K x C x kh x kw for precision 0 and 1, the int16-typed bf16 kernel matrix
    of im2col_prepare_weights_bf16 for precision 2."""
    import torch

    return _dev_ptr(weights, torch.int16 if int(precision) == 2 else torch.float32)


def _dev_ptr(t, dtype=None) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


class EncodedMap:
    """Device buffers of one encoded activation map (cpoconv_map of the C ABI), or of a batch of
    n_images maps: then every buffer holds n_images regions of the per-image capacity."""

    def __init__(self, shape, device="cuda:0", n_images=1, sizes=None, in_bits=32):
        import torch

        self.shape = make_shape(shape)
        self.n_images = int(n_images)
        self.in_bits = int(in_bits)     # 32, or 16 for a compact map with int16 IN entries
        sz = cpoconv_sizes(self.shape) if sizes is None else sizes   # sizes: capacities larger than the shape's own
        self.sizes = sz
        n = self.n_images
        self.ptr = torch.empty(n * sz.ptr_cap, dtype=torch.int32, device=device)
        self.da = torch.empty(n * sz.da_cap, dtype=torch.float32, device=device)
        self.ind = torch.empty(n * sz.in_cap, dtype=torch.int16 if self.in_bits == 16 else torch.int32, device=device)
        self.chan_off = torch.empty(n * sz.chan_off_len, dtype=torch.int32, device=device)
        self.hdr = torch.zeros(n * 8, dtype=torch.int32, device=device)

    def c_struct(self, image=0) -> _Map:
        """The struct of image `image` (image 0 describes the whole batch to the batched calls)."""
        sz = self.sizes
        return _Map(ctypes.c_void_p(self.ptr.data_ptr() + 4 * image * sz.ptr_cap), sz.ptr_cap,
                    ctypes.c_void_p(self.da.data_ptr() + 4 * image * sz.da_cap), sz.da_cap,
                    ctypes.c_void_p(self.ind.data_ptr() + self.ind.element_size() * image * sz.in_cap), sz.in_cap,
                    ctypes.c_void_p(self.chan_off.data_ptr() + 4 * image * 3 * (self.shape.C + 1)),
                    ctypes.c_void_p(self.hdr.data_ptr() + 4 * image * 8), self.in_bits)

    def view(self, shape) -> "EncodedMap":
        """The same buffers seen as the map of another layer shape (a chain's layers share one map;
        the side band's stride between images follows the layer's channel count)."""
        import copy

        other = copy.copy(self)
        other.shape = make_shape(shape)
        return other

    def header(self, stream=None, image=0):
        return cpoconv_map_header_to_host(self, stream, image)

    def to_host(self, stream=None, image=0):
        """(ptr, da, ind, chan_off[3, C+1], hdr) of one image as numpy arrays trimmed to their lengths."""
        hdr = self.header(stream, image)
        C, sz = self.shape.C, self.sizes
        p0, d0, i0, c0 = image * sz.ptr_cap, image * sz.da_cap, image * sz.in_cap, image * 3 * (C + 1)
        return (self.ptr[p0:p0 + hdr[0]].cpu().numpy(), self.da[d0:d0 + hdr[1]].cpu().numpy(),
                self.ind[i0:i0 + hdr[2]].cpu().numpy(),
                self.chan_off[c0:c0 + 3 * (C + 1)].cpu().numpy().reshape(3, C + 1), hdr)


def _encode(fn_name: str, act, shape, m: EncodedMap, scratch, stream) -> None:
    import torch

    sh = make_shape(shape)
    cm = m.c_struct()
    _check(getattr(lib(), fn_name)(_dev_ptr(act, torch.float32), ctypes.byref(sh), ctypes.byref(cm),
                                   _dev_ptr(scratch), ctypes.c_int64(scratch.numel() * scratch.element_size()),
                                   _stream_handle(stream)))


def cpo_encode(act, shape, m: EncodedMap, scratch, stream=None) -> None:
    _encode("cpo_encode", act, shape, m, scratch, stream)


def cps_encode(act, shape, m: EncodedMap, scratch, stream=None) -> None:
    _encode("cps_encode", act, shape, m, scratch, stream)


def cpo_encode_static_scratch(act, shape, m: EncodedMap, stream=None) -> None:
    """cpo_encode without a scratch buffer from the caller (the library's own device array)."""
    import torch

    sh = make_shape(shape)
    cm = m.c_struct()
    _check(lib().cpo_encode_static_scratch(_dev_ptr(act, torch.float32), ctypes.byref(sh), ctypes.byref(cm),
                                           _stream_handle(stream)))


def cpoconv_prepare_weights(weights, shape, wt, stream=None) -> None:
    import torch

    sh = make_shape(shape)
    _check(lib().cpoconv_prepare_weights(_dev_ptr(weights, torch.float32), ctypes.byref(sh),
                                         _dev_ptr(wt, torch.float32), _stream_handle(stream)))


def _conv(fn_name: str, m: EncodedMap, shape, wt, out, scratch, stream) -> None:
    import torch

    sh = make_shape(shape)
    cm = m.c_struct()
    _check(getattr(lib(), fn_name)(ctypes.byref(cm), ctypes.byref(sh), _dev_ptr(wt, torch.float32),
                                   _dev_ptr(out, torch.float32), _dev_ptr(scratch),
                                   ctypes.c_int64(scratch.numel() * scratch.element_size()),
                                   _stream_handle(stream)))


def cpo_conv(m: EncodedMap, shape, wt, out, scratch, stream=None) -> None:
    _conv("cpo_conv", m, shape, wt, out, scratch, stream)


def cps_conv(m: EncodedMap, shape, wt, out, scratch, stream=None) -> None:
    _conv("cps_conv", m, shape, wt, out, scratch, stream)


def im2col_conv(act, shape, weights, lowered, out, precision: int = 0, stream=None) -> None:
    import torch

    sh = make_shape(shape)
    _check(lib().im2col_conv(_dev_ptr(act, torch.float32), ctypes.byref(sh), _weights_ptr(weights, precision),
                             _dev_ptr(lowered), _dev_ptr(out, torch.float32), int(precision),
                             _stream_handle(stream)))


def im2col_prepare_weights_bf16(weights, shape, wb, stream=None) -> None:
    """wb: int16 device tensor of cpoconv_sizes(shape).wb_len elements (bf16 bit patterns)."""
    import torch

    sh = make_shape(shape)
    _check(lib().im2col_prepare_weights_bf16(_dev_ptr(weights, torch.float32), ctypes.byref(sh),
                                             _dev_ptr(wb, torch.int16), _stream_handle(stream)))


def cpoconv_map_header_to_host(m: EncodedMap, stream=None, image=0):
    cm = m.c_struct(image)
    hdr = (ctypes.c_int32 * 8)()
    rc = lib().cpoconv_map_header_to_host(ctypes.byref(cm), hdr, _stream_handle(stream))
    if rc == ERR_MAP:      # the header is filled in all the same: the error carries it
        err = CpoconvError(rc, cpoconv_strerror(rc))
        err.hdr = [int(v) for v in hdr]
        raise err
    _check(rc)
    return [int(v) for v in hdr]


class LayerBuffers:
    """All device buffers one layer (or a batch of n_images inputs of it) needs, allocated once with PyTorch."""

    def __init__(self, shape, device="cuda:0", n_images=1, in_bits=32):
        import torch

        self.shape = make_shape(shape)
        self.n_images = int(n_images)
        sz = cpoconv_batch_sizes(self.shape, self.n_images)
        self.sizes = sz
        self.device = device
        self.cpo = EncodedMap(self.shape, device, self.n_images, in_bits=in_bits)
        self.cps = EncodedMap(self.shape, device, self.n_images, in_bits=in_bits)
        self.scratch = torch.empty(sz.scratch_bytes, dtype=torch.uint8, device=device)
        cpoconv_scratch_init(self.scratch)
        self.wt = torch.empty(sz.wt_len, dtype=torch.float32, device=device)
        self.wb = torch.empty(sz.wb_len, dtype=torch.int16, device=device)
        self.lowered = torch.empty(sz.lowered_bytes, dtype=torch.uint8, device=device)
        dims = (self.shape.K, sz.Oh, sz.Ow) if self.n_images == 1 else (self.n_images, self.shape.K, sz.Oh, sz.Ow)
        self.out = torch.empty(dims, dtype=torch.float32, device=device)


# ---- batched calls: n_images maps of one shape per launch --------------------------------------

def cpoconv_scratch_init(scratch, stream=None) -> None:
    """Zero-fills a scratch buffer: required once before its first use (see include/cpoconv.h)."""
    _check(lib().cpoconv_scratch_init(_dev_ptr(scratch), ctypes.c_int64(scratch.numel() * scratch.element_size()),
                                      _stream_handle(stream)))


def cpoconv_batch_sizes(shape, n_images: int) -> Sizes:
    sh, sz = make_shape(shape), Sizes()
    _check(lib().cpoconv_batch_sizes(ctypes.byref(sh), int(n_images), ctypes.byref(sz)))
    return sz


def _encode_batch(fn_name: str, act, shape, m: EncodedMap, scratch, stream) -> None:
    import torch

    sh = make_shape(shape)
    cm = m.c_struct()
    _check(getattr(lib(), fn_name)(_dev_ptr(act, torch.float32), ctypes.byref(sh), int(m.n_images), ctypes.byref(cm),
                                   _dev_ptr(scratch), ctypes.c_int64(scratch.numel() * scratch.element_size()),
                                   _stream_handle(stream)))


def cpo_encode_batch(act, shape, m: EncodedMap, scratch, stream=None) -> None:
    _encode_batch("cpo_encode_batch", act, shape, m, scratch, stream)


def cps_encode_batch(act, shape, m: EncodedMap, scratch, stream=None) -> None:
    _encode_batch("cps_encode_batch", act, shape, m, scratch, stream)


def _conv_batch(fn_name: str, m: EncodedMap, shape, wt, out, scratch, stream) -> None:
    import torch

    sh = make_shape(shape)
    cm = m.c_struct()
    _check(getattr(lib(), fn_name)(ctypes.byref(cm), ctypes.byref(sh), int(m.n_images), _dev_ptr(wt, torch.float32),
                                   _dev_ptr(out, torch.float32), _dev_ptr(scratch),
                                   ctypes.c_int64(scratch.numel() * scratch.element_size()),
                                   _stream_handle(stream)))


def cpo_conv_batch(m: EncodedMap, shape, wt, out, scratch, stream=None) -> None:
    _conv_batch("cpo_conv_batch", m, shape, wt, out, scratch, stream)


def cps_conv_batch(m: EncodedMap, shape, wt, out, scratch, stream=None) -> None:
    _conv_batch("cps_conv_batch", m, shape, wt, out, scratch, stream)


def im2col_conv_batch(act, shape, n_images: int, weights, lowered, out, precision: int = 0, stream=None) -> None:
    import torch

    sh = make_shape(shape)
    _check(lib().im2col_conv_batch(_dev_ptr(act, torch.float32), ctypes.byref(sh), int(n_images),
                                   _weights_ptr(weights, precision), _dev_ptr(lowered), _dev_ptr(out, torch.float32),
                                   int(precision), _stream_handle(stream)))


# ---- encoding + convolution of a layer in one call ---------------------------------------------

def _encode_conv(fn_name: str, act, shape, m: EncodedMap, wt, out, scratch, stream) -> None:
    import torch

    sh = make_shape(shape)
    cm = m.c_struct()
    args = [_dev_ptr(act, torch.float32), ctypes.byref(sh)]
    if fn_name.endswith("_batch"):
        args.append(int(m.n_images))
    args += [ctypes.byref(cm), _dev_ptr(wt, torch.float32), _dev_ptr(out, torch.float32), _dev_ptr(scratch),
             ctypes.c_int64(scratch.numel() * scratch.element_size()), _stream_handle(stream)]
    _check(getattr(lib(), fn_name)(*args))


def cpo_encode_conv(act, shape, m: EncodedMap, wt, out, scratch, stream=None) -> None:
    _encode_conv("cpo_encode_conv" if m.n_images == 1 else "cpo_encode_conv_batch", act, shape, m, wt, out, scratch, stream)


def cps_encode_conv(act, shape, m: EncodedMap, wt, out, scratch, stream=None) -> None:
    _encode_conv("cps_encode_conv" if m.n_images == 1 else "cps_encode_conv_batch", act, shape, m, wt, out, scratch, stream)


# ---- a layer's input produced on the way in (bias and ReLU of the layer before it) --------------

def _encode_relu(fn_name: str, pre, bias, shape, m: EncodedMap, scratch, stream) -> None:
    import torch

    sh = make_shape(shape)
    cm = m.c_struct()
    _check(getattr(lib(), fn_name)(_dev_ptr(pre, torch.float32), _dev_ptr(bias, torch.float32), ctypes.byref(sh),
                                   int(m.n_images), ctypes.byref(cm), _dev_ptr(scratch),
                                   ctypes.c_int64(scratch.numel() * scratch.element_size()), _stream_handle(stream)))


def cpo_encode_relu(pre, bias, shape, m: EncodedMap, scratch, stream=None) -> None:
    _encode_relu("cpo_encode_relu", pre, bias, shape, m, scratch, stream)


def cps_encode_relu(pre, bias, shape, m: EncodedMap, scratch, stream=None) -> None:
    _encode_relu("cps_encode_relu", pre, bias, shape, m, scratch, stream)


def im2col_conv_relu(pre, bias, shape, n_images: int, weights, lowered, out, precision: int = 0, stream=None) -> None:
    import torch

    sh = make_shape(shape)
    _check(lib().im2col_conv_relu(_dev_ptr(pre, torch.float32), _dev_ptr(bias, torch.float32), ctypes.byref(sh),
                                  int(n_images), _weights_ptr(weights, precision), _dev_ptr(lowered),
                                  _dev_ptr(out, torch.float32), int(precision), _stream_handle(stream)))


# ---- chained layers ------------------------------------------------------------------------------

class ChainLayer(ctypes.Structure):
    _fields_ = [("shape", Shape), ("method", ctypes.c_int32), ("precision", ctypes.c_int32),
                ("relu_in", ctypes.c_int32), ("bias_in", ctypes.c_void_p), ("weights", ctypes.c_void_p),
                ("out", ctypes.c_void_p)]


def cpoconv_chain_sizes(layers, n_images: int) -> Sizes:
    """layers: a ctypes array of ChainLayer (pointer members are not read)."""
    sz = Sizes()
    _check(lib().cpoconv_chain_sizes(layers, len(layers), int(n_images), ctypes.byref(sz)))
    return sz


class Chain:
    """Device buffers and the layer table of cpoconv_chain_forward.  weights: K x C x kh x kw device
    tensors; biases[i] (device tensor or None) and relu_in[i] describe what is applied to layer i's
    input; methods[i] is ALGO_IM2COL / ALGO_CPO / ALGO_CPS (set_methods changes them later)."""

    def __init__(self, shapes, weights, biases, relu_in, methods, n_images=1, precision=0, device="cuda:0", in_bits=32):
        import torch

        self.shapes = [make_shape(s) for s in shapes]
        self.n_images = int(n_images)
        self.weights, self.biases, self.relu_in = list(weights), list(biases), [int(bool(r)) for r in relu_in]
        self.precision = int(precision)
        self.device = device
        n = len(self.shapes)
        self.table = (ChainLayer * n)()
        self.outs, self.prepared, self.prepared_bf16 = [], [None] * n, [None] * n
        for i, sh in enumerate(self.shapes):
            sz = cpoconv_batch_sizes(sh, self.n_images)
            self.outs.append(torch.empty((self.n_images, sh.K, sz.Oh, sz.Ow), dtype=torch.float32, device=device))
            self.table[i].shape = sh
            self.table[i].precision = self.precision
            self.table[i].relu_in = self.relu_in[i]
            self.table[i].bias_in = _dev_ptr(self.biases[i], torch.float32).value
            self.table[i].out = self.outs[i].data_ptr()
        sz = cpoconv_chain_sizes(self.table, self.n_images)
        self.sizes = sz
        self.map = EncodedMap(self.shapes[0], device, self.n_images, sizes=sz, in_bits=in_bits)
        self.scratch = torch.empty(sz.scratch_bytes, dtype=torch.uint8, device=device)
        cpoconv_scratch_init(self.scratch)
        self.lowered = torch.empty(sz.lowered_bytes, dtype=torch.uint8, device=device)
        self.set_methods(methods)

    def set_methods(self, methods) -> None:
        import torch

        assert len(methods) == len(self.shapes)
        self.methods = [int(m) for m in methods]
        for i, (m, sh) in enumerate(zip(self.methods, self.shapes)):
            self.table[i].method = m
            if m == ALGO_IM2COL and self.precision == 2:
                if self.prepared_bf16[i] is None:
                    wb = torch.empty(cpoconv_sizes(sh).wb_len, dtype=torch.int16, device=self.device)
                    im2col_prepare_weights_bf16(self.weights[i], sh, wb)
                    self.prepared_bf16[i] = wb
                self.table[i].weights = self.prepared_bf16[i].data_ptr()
            elif m == ALGO_IM2COL:
                self.table[i].weights = _dev_ptr(self.weights[i], torch.float32).value
            else:
                if self.prepared[i] is None:
                    wt = torch.empty(cpoconv_sizes(sh).wt_len, dtype=torch.float32, device=self.device)
                    cpoconv_prepare_weights(self.weights[i], sh, wt)
                    self.prepared[i] = wt
                self.table[i].weights = self.prepared[i].data_ptr()

    def forward(self, act, stream=None, first=0, count=None) -> None:
        """Runs every layer; layer i's output (before bias / ReLU) lands in outs[i].  With first /
        count only layers first .. first+count-1 run, `act` being the input of layer `first`."""
        import torch

        count = len(self.shapes) - first if count is None else count
        cm = self.map.c_struct()
        sub = ctypes.cast(ctypes.byref(self.table, first * ctypes.sizeof(ChainLayer)), ctypes.POINTER(ChainLayer))
        _check(lib().cpoconv_chain_forward(_dev_ptr(act, torch.float32), sub, int(count), self.n_images,
                                           ctypes.byref(cm), _dev_ptr(self.scratch),
                                           ctypes.c_int64(self.scratch.numel()), _dev_ptr(self.lowered),
                                           ctypes.c_int64(self.lowered.numel()), _stream_handle(stream)))
