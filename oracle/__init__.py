"""ctypes front end of the CPU oracle (``cpoconv_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package.  It shares nothing with the HIP library and never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cpoconv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

NPF = -2
NPC = -3
ALGO_CPO = 0
ALGO_CPS = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no vectoriser flags, no OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC])
    return _LIB


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("C", "H", "W", "K", "kh", "kw", "stride", "pad_h", "pad_w")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_max_ptr.restype = ctypes.c_int64
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _shape(shape) -> _Shape:
    """(C, H, W, K, kh, kw, stride, pad) pads all four sides alike; a ninth entry gives the
    columns their own padding: (.., stride, pad_h, pad_w)."""
    v = [int(x) for x in shape]
    if len(v) == 8:
        v.append(v[7])
    return _Shape(*v)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


@dataclass
class Geometry:
    Ih: int
    Iw: int
    Oh: int
    Ow: int
    nop3: bool
    top: int
    cls: np.ndarray
    p0: np.ndarray
    what: np.ndarray
    real: np.ndarray
    present: np.ndarray


def geometry(shape) -> Geometry:
    sh = _shape(shape)
    Iw = sh.W + 2 * sh.pad_w
    info = np.zeros(6, np.int32)
    cls, p0, what, real = (np.zeros(max(Iw, 1), np.int32) for _ in range(4))
    present = np.zeros(max(sh.kw, 1), np.int32)
    _check(_load().orc_geometry(ctypes.byref(sh), _p(info), _p(cls), _p(p0), _p(what), _p(real),
                                _p(present)), "geometry")
    return Geometry(int(info[0]), int(info[1]), int(info[2]), int(info[3]), bool(info[4]),
                    int(info[5]), cls, p0, what, real, present)


@dataclass
class EncodedMap:
    """The three streams of the paper plus the per-channel side band."""
    algo: int
    shape: Tuple[int, ...]
    ptr: np.ndarray       # int32
    da: np.ndarray        # float32
    ind: np.ndarray       # int32 ("IN")
    chan_off: np.ndarray  # int32, 3 x (C+1): ptr / DA / IN offsets

    @property
    def elements(self) -> int:
        """|ptr| + |DA| + |IN| (SI: total size of the CPO/CPS structure)."""
        return int(self.ptr.size + self.da.size + self.ind.size)


def encode(act: np.ndarray, shape, algo: int) -> EncodedMap:
    sh = _shape(shape)
    act = np.ascontiguousarray(act, dtype=np.float32)
    assert act.shape == (sh.C, sh.H, sh.W), (act.shape, tuple(shape))
    lib = _load()
    ptr_cap = int(lib.orc_max_ptr(ctypes.byref(sh)))
    if ptr_cap < 0:
        raise ValueError("oracle: bad shape")
    da_cap = (sh.C + 1) * (sh.H + 2 * sh.pad_h) * (sh.W + 2 * sh.pad_w)
    ptr = np.zeros(ptr_cap, np.int32)
    da = np.zeros(da_cap, np.float32)
    ind = np.zeros(da_cap, np.int32)
    chan_off = np.zeros(3 * (sh.C + 1), np.int32)
    lens = np.zeros(3, np.int64)
    _check(lib.orc_encode(_p(act), ctypes.byref(sh), int(algo), _p(ptr), ctypes.c_int64(ptr_cap),
                          _p(da), _p(ind), ctypes.c_int64(da_cap), _p(chan_off), _p(lens)), "encode")
    return EncodedMap(int(algo), tuple(int(v) for v in shape), ptr[:lens[0]].copy(),
                      da[:lens[1]].copy(), ind[:lens[2]].copy(), chan_off.reshape(3, sh.C + 1).copy())


def cpo_encode(act, shape) -> EncodedMap:
    return encode(act, shape, ALGO_CPO)


def cps_encode(act, shape) -> EncodedMap:
    return encode(act, shape, ALGO_CPS)


def _out_shape(sh: _Shape) -> Tuple[int, int, int]:
    Oh = (sh.H + 2 * sh.pad_h - sh.kh) // sh.stride + 1
    Ow = (sh.W + 2 * sh.pad_w - sh.kw) // sh.stride + 1
    return sh.K, Oh, Ow


def sparse_conv(m: EncodedMap, weights: np.ndarray) -> np.ndarray:
    """Algorithm 2 / Algorithm 4 on an encoded map; returns K x Oh x Ow."""
    sh = _shape(m.shape)
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    assert weights.shape == (sh.K, sh.C, sh.kh, sh.kw)
    out = np.zeros(_out_shape(sh), np.float32)
    ptr = np.ascontiguousarray(m.ptr); da = np.ascontiguousarray(m.da); ind = np.ascontiguousarray(m.ind)
    _check(_load().orc_sparse_conv(_p(ptr), _p(da), _p(ind), ctypes.byref(sh), int(m.algo),
                                   _p(weights), _p(out)), "sparse_conv")
    return out


def decode(m: EncodedMap) -> np.ndarray:
    sh = _shape(m.shape)
    act = np.zeros((sh.C, sh.H, sh.W), np.float32)
    ptr = np.ascontiguousarray(m.ptr); da = np.ascontiguousarray(m.da); ind = np.ascontiguousarray(m.ind)
    _check(_load().orc_decode(_p(ptr), _p(da), _p(ind), ctypes.byref(sh), int(m.algo), _p(act)),
           "decode")
    return act


def conv_direct(act: np.ndarray, weights: np.ndarray, shape) -> np.ndarray:
    """Eq. 1: the dense definition, K x Oh x Ow."""
    sh = _shape(shape)
    act = np.ascontiguousarray(act, dtype=np.float32)
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    assert act.shape == (sh.C, sh.H, sh.W) and weights.shape == (sh.K, sh.C, sh.kh, sh.kw)
    out = np.zeros(_out_shape(sh), np.float32)
    _check(_load().orc_conv_direct(_p(act), ctypes.byref(sh), _p(weights), _p(out)), "conv_direct")
    return out


def im2col_lower(act: np.ndarray, shape) -> np.ndarray:
    sh = _shape(shape)
    act = np.ascontiguousarray(act, dtype=np.float32)
    _, Oh, Ow = _out_shape(sh)
    low = np.zeros((sh.C * sh.kh * sh.kw, Oh * Ow), np.float32)
    _check(_load().orc_im2col_lower(_p(act), ctypes.byref(sh), _p(low)), "im2col_lower")
    return low


def gemm(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    M, Kd = a.shape
    Kd2, N = b.shape
    assert Kd == Kd2
    out = np.zeros((M, N), np.float32)
    _check(_load().orc_gemm(_p(a), _p(b), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(Kd),
                            _p(out)), "gemm")
    return out


def im2col_conv(act: np.ndarray, weights: np.ndarray, shape) -> np.ndarray:
    sh = _shape(shape)
    low = im2col_lower(act, shape)
    wmat = np.ascontiguousarray(weights, dtype=np.float32).reshape(sh.K, -1)
    return gemm(wmat, low).reshape(_out_shape(sh))


def select_layer_algo(t_im2col, t_cpo, t_cps, mode: int) -> int:
    a = np.ascontiguousarray(t_im2col, dtype=np.float64)
    b = np.ascontiguousarray(t_cpo, dtype=np.float64)
    c = np.ascontiguousarray(t_cps, dtype=np.float64)
    assert a.size == b.size == c.size
    return int(_load().orc_select(_p(a), _p(b), _p(c), int(a.size), int(mode)))


def bias_relu(pre: np.ndarray, bias=None) -> np.ndarray:
    """What a layer's input is when the layer before it ends in a bias and a ReLU: the input I of
    Eq. 1 is the output max(0, z) of the activation function (Section "Sparsity and Patterns
    Motivation").  z = pre + bias[c] is one fp32 addition; every z that is not greater than zero
    (negative values, both zeros, NaN) becomes +0, so the zeros of the result are exactly the
    elements the encoders skip."""
    z = np.asarray(pre, dtype=np.float32)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32)
        assert b.shape == (z.shape[0],)
        z = z + b[:, None, None]
        assert z.dtype == np.float32
    with np.errstate(invalid="ignore"):
        return np.where(z > 0, z, np.float32(0.0)).astype(np.float32)


def chain_forward(act: np.ndarray, chain) -> list:
    """Convolution layers run one after the other (Section "Hybrid Inference Over a Target CNN":
    the conv layers of a CNN, each with the method chosen for it - all methods compute Eq. 1, so
    the oracle is Eq. 1 per layer).  ``chain`` is a sequence of (shape, weights, bias_in, relu_in):
    a layer's input is the previous layer's stored fp32 output, passed through ``bias_relu`` with
    ``bias_in`` when ``relu_in`` is set.  Returns every layer's K x Oh x Ow output."""
    outs = []
    x = np.ascontiguousarray(act, dtype=np.float32)
    for shape, weights, bias_in, relu_in in chain:
        if relu_in:
            x = bias_relu(x, bias_in)
        else:
            assert bias_in is None
        x = conv_direct(x, weights, shape)
        outs.append(x)
    return outs
