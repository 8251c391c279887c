"""ctypes front end of the CPU oracle (``daq_ref.c``).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the product package never does.
All arrays are host numpy arrays; int8 tensors are logically indexed (NCHW,
``[Cout][Cin/groups][kH][kW]``).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "daq_ref.c")
_LIB = os.path.join(_HERE, "libdaq_ref.so")

GAUSS, INVT = 0, 1
ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1
SCHEME_DAQ, SCHEME_GQ, SCHEME_GVQ, SCHEME_MCS = 0, 1, 2, 3   # Algorithm 1 and the ablation study's three variants


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("N", "Cin", "Hin", "Win", "Cout", "kH", "kW", "strideH", "strideW", "padH",
                                       "padW", "dilH", "dilW", "groups")]


@dataclass(frozen=True)
class ConvDesc:
    N: int
    Cin: int
    Hin: int
    Win: int
    Cout: int
    kH: int
    kW: int
    strideH: int = 1
    strideW: int = 1
    padH: int = 0
    padW: int = 0
    dilH: int = 1
    dilW: int = 1
    groups: int = 1

    def c(self) -> _Desc:
        return _Desc(self.N, self.Cin, self.Hin, self.Win, self.Cout, self.kH, self.kW, self.strideH, self.strideW,
                     self.padH, self.padW, self.dilH, self.dilW, self.groups)

    @property
    def Ho(self) -> int:
        return (self.Hin + 2 * self.padH - self.dilH * (self.kH - 1) - 1) // self.strideH + 1

    @property
    def Wo(self) -> int:
        return (self.Win + 2 * self.padW - self.dilW * (self.kW - 1) - 1) // self.strideW + 1

    @property
    def x_shape(self):
        return (self.N, self.Cin, self.Hin, self.Win)

    @property
    def w_shape(self):
        return (self.Cout, self.Cin // self.groups, self.kH, self.kW)

    @property
    def y_shape(self):
        return (self.N, self.Cout, self.Ho, self.Wo)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.daq_ref_uniform16.restype = C.c_float
        _lib.daq_ref_uniform16.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64]
        _lib.daq_ref_fmix32.restype = C.c_uint32
        _lib.daq_ref_fmix32.argtypes = [C.c_uint32]
        _lib.daq_ref_quantize_one.restype = C.c_int8
        _lib.daq_ref_quantize_one.argtypes = [C.c_float, C.c_float, C.c_int, C.c_float]
        _lib.daq_ref_dequantize_one.restype = C.c_float
        _lib.daq_ref_dequantize_one.argtypes = [C.c_int8, C.c_float]
        _lib.daq_ref_clip_value.restype = C.c_float
        _lib.daq_ref_clip_value.argtypes = [C.c_int, C.c_float, C.c_float, C.c_float, C.c_float]
        _lib.daq_ref_classify.restype = C.c_int
        _lib.daq_ref_classify.argtypes = [C.c_uint32, C.c_double, C.c_float]
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


def _chk(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i8(a):
    return np.ascontiguousarray(a, dtype=np.int8)


def num_threads() -> int:
    return int(lib().daq_ref_num_threads())


def fmix32(h: int) -> int:
    return int(lib().daq_ref_fmix32(h & 0xFFFFFFFF))


def uniform16(seed: int, tensor: int, idx: int) -> float:
    return float(lib().daq_ref_uniform16(seed, tensor, idx))


def quantize_one(x: float, s: float, mode: int = ROUND_NEAREST, u: float = 0.0) -> int:
    return int(lib().daq_ref_quantize_one(x, s, mode, u))


def dequantize_one(q: int, s: float) -> float:
    return float(lib().daq_ref_dequantize_one(q, s))


def clip_value(cls: int, gmax: float, s_prev: float, k: float, A: float) -> float:
    return float(lib().daq_ref_clip_value(cls, gmax, s_prev, k, A))


def classify(count: int, M: float, lam: float) -> int:
    return int(lib().daq_ref_classify(count, M, lam))


def channel_stats(g):
    g = _f32(g)
    N, Cc, H, W = g.shape
    gmax = np.zeros(Cc, np.float32)
    mean = np.zeros(Cc, np.float32)
    sigma = np.zeros(Cc, np.float32)
    _chk(lib().daq_ref_channel_stats(_p(g, C.c_float), N, Cc, H, W, _p(gmax, C.c_float), _p(mean, C.c_float),
                                     _p(sigma, C.c_float)), "channel_stats")
    return gmax, mean, sigma


def tail_count(g, sigma):
    g = _f32(g)
    sigma = _f32(sigma)
    N, Cc, H, W = g.shape
    cnt = np.zeros(Cc, np.uint32)
    _chk(lib().daq_ref_tail_count(_p(g, C.c_float), N, Cc, H, W, _p(sigma, C.c_float), _p(cnt, C.c_uint32)),
         "tail_count")
    return cnt


@dataclass
class QuantGrad:
    vq: np.ndarray        # int8 NCHW, per-channel scales
    qg: np.ndarray        # int8 NCHW, global scale
    s_chan: np.ndarray    # fp32 [C]
    s_global: float
    cls: np.ndarray       # u8 [C]
    stats: np.ndarray     # fp32 [C,4]: gmax, mean, sigma, P
    s_state: np.ndarray   # fp32 [C] updated state
    fragile: np.ndarray   # u8 [C]


def quantize_grad(dY, s_state, k=1.0, A=0.8, lam=0.3, mode=ROUND_NEAREST, seed=0, want_fragile=True,
                  scheme=SCHEME_DAQ) -> QuantGrad:
    g = _f32(dY)
    N, Cc, H, W = g.shape
    st = np.array(s_state, dtype=np.float32, copy=True)
    assert st.shape == (Cc,)
    vq = np.zeros(g.shape, np.int8)
    qg = np.zeros(g.shape, np.int8)
    s_chan = np.zeros(Cc, np.float32)
    s_glob = np.zeros(1, np.float32)
    cls = np.zeros(Cc, np.uint8)
    stats = np.zeros((Cc, 4), np.float32)
    frag = np.zeros(Cc, np.uint8) if want_fragile else None
    rc = lib().daq_ref_quantize_grad_scheme(_p(g, C.c_float), N, Cc, H, W, _p(st, C.c_float), C.c_float(k),
                                            C.c_float(A), C.c_float(lam), C.c_int(mode), C.c_uint64(seed),
                                            C.c_int(scheme), _p(vq, C.c_int8), _p(qg, C.c_int8),
                                            _p(s_chan, C.c_float), _p(s_glob, C.c_float), _p(cls, C.c_uint8),
                                            _p(stats, C.c_float), _p(frag, C.c_uint8))
    _chk(rc, "quantize_grad")
    if frag is None:
        frag = np.zeros(Cc, np.uint8)
    return QuantGrad(vq, qg, s_chan, float(s_glob[0]), cls, stats, st, frag)


def widen_bf16(bits) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> the fp32 values they denote: a bfloat16 is the upper half of an fp32 pattern."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def quantize_grad_bf16(dY_bits, s_state, **kw) -> QuantGrad:
    """The quantizer on a gradient stored as bfloat16: by definition the fp32 algorithm on the widened values."""
    return quantize_grad(widen_bf16(dY_bits), s_state, **kw)


def quantize_tensor(x):
    x = _f32(x)
    q = np.zeros(x.shape, np.int8)
    s = np.zeros(1, np.float32)
    _chk(lib().daq_ref_quantize_tensor(_p(x, C.c_float), C.c_size_t(x.size), _p(q, C.c_int8), _p(s, C.c_float)),
         "quantize_tensor")
    return q, float(s[0])


def conv_fwd_acc(d: ConvDesc, qX, qW):
    qX, qW = _i8(qX), _i8(qW)
    assert qX.shape == d.x_shape and qW.shape == d.w_shape
    acc = np.zeros(d.y_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv_fwd_acc(C.byref(dd), _p(qX, C.c_int8), _p(qW, C.c_int8), _p(acc, C.c_int32),
                                    C.byref(ovf)), "conv_fwd_acc")
    return acc, bool(ovf.value)


def conv_bwd_data_acc(d: ConvDesc, qG, qW):
    qG, qW = _i8(qG), _i8(qW)
    assert qG.shape == d.y_shape and qW.shape == d.w_shape
    acc = np.zeros(d.x_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv_bwd_data_acc(C.byref(dd), _p(qG, C.c_int8), _p(qW, C.c_int8), _p(acc, C.c_int32),
                                         C.byref(ovf)), "conv_bwd_data_acc")
    return acc, bool(ovf.value)


def conv_bwd_filter_acc(d: ConvDesc, qX, qG):
    qX, qG = _i8(qX), _i8(qG)
    assert qX.shape == d.x_shape and qG.shape == d.y_shape
    acc = np.zeros(d.w_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv_bwd_filter_acc(C.byref(dd), _p(qX, C.c_int8), _p(qG, C.c_int8), _p(acc, C.c_int32),
                                           C.byref(ovf)), "conv_bwd_filter_acc")
    return acc, bool(ovf.value)


def conv_bwd_data_acc_at(d: ConvDesc, qG, qW, idx):
    """Accumulators of G_X at the linear NCHW indices ``idx`` only (same definition as conv_bwd_data_acc)."""
    qG, qW = _i8(qG), _i8(qW)
    assert qG.shape == d.y_shape and qW.shape == d.w_shape
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.zeros(idx.size, np.int32)
    dd = d.c()
    _chk(lib().daq_ref_conv_bwd_data_acc_at(C.byref(dd), _p(qG, C.c_int8), _p(qW, C.c_int8), _p(idx, C.c_int64),
                                            C.c_int64(idx.size), _p(out, C.c_int32)), "conv_bwd_data_acc_at")
    return out


def conv_bwd_filter_acc_at(d: ConvDesc, qX, qG, idx):
    """Accumulators of G_W at the linear [Cout][Cin/g][kH][kW] indices ``idx`` only."""
    qX, qG = _i8(qX), _i8(qG)
    assert qX.shape == d.x_shape and qG.shape == d.y_shape
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.zeros(idx.size, np.int32)
    dd = d.c()
    _chk(lib().daq_ref_conv_bwd_filter_acc_at(C.byref(dd), _p(qX, C.c_int8), _p(qG, C.c_int8), _p(idx, C.c_int64),
                                              C.c_int64(idx.size), _p(out, C.c_int32)), "conv_bwd_filter_acc_at")
    return out


def conv_fwd_acc_at(d: ConvDesc, qX, qW, idx):
    """Accumulators of the forward convolution at the linear NCHW indices ``idx`` of Y only."""
    qX, qW = _i8(qX), _i8(qW)
    assert qX.shape == d.x_shape and qW.shape == d.w_shape
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.zeros(idx.size, np.int32)
    dd = d.c()
    _chk(lib().daq_ref_conv_fwd_acc_at(C.byref(dd), _p(qX, C.c_int8), _p(qW, C.c_int8), _p(idx, C.c_int64),
                                       C.c_int64(idx.size), _p(out, C.c_int32)), "conv_fwd_acc_at")
    return out


def dequantize_acc(acc, s_a: float, s_b) -> np.ndarray:
    """acc * (s_a/127) * (s_b/127) in the oracle's fp32 operation order; ``s_b`` is a scalar or one scale per element."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    sb = np.ascontiguousarray(np.broadcast_to(np.asarray(s_b, dtype=np.float32), acc.shape), dtype=np.float32)
    out = np.zeros(acc.shape, np.float32)
    _chk(lib().daq_ref_dequantize_acc(_p(acc, C.c_int32), C.c_int64(acc.size), C.c_float(s_a), _p(sb, C.c_float),
                                      _p(out, C.c_float)), "dequantize_acc")
    return out


@dataclass
class Fwd:
    qX: np.ndarray
    qW: np.ndarray
    s_x: float
    s_w: float
    Y: np.ndarray
    acc: np.ndarray
    overflow: bool


def conv_fwd_int8(d: ConvDesc, X, Wt) -> Fwd:
    X, Wt = _f32(X), _f32(Wt)
    assert X.shape == d.x_shape and Wt.shape == d.w_shape
    qX = np.zeros(d.x_shape, np.int8)
    qW = np.zeros(d.w_shape, np.int8)
    sx = np.zeros(1, np.float32)
    sw = np.zeros(1, np.float32)
    Y = np.zeros(d.y_shape, np.float32)
    acc = np.zeros(d.y_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv_fwd_int8(C.byref(dd), _p(X, C.c_float), _p(Wt, C.c_float), _p(qX, C.c_int8),
                                     _p(qW, C.c_int8), _p(sx, C.c_float), _p(sw, C.c_float), _p(Y, C.c_float),
                                     _p(acc, C.c_int32), C.byref(ovf)), "conv_fwd_int8")
    return Fwd(qX, qW, float(sx[0]), float(sw[0]), Y, acc, bool(ovf.value))


def conv_bwd_data_int8(d: ConvDesc, qG, s_global, qW, s_w):
    qG, qW = _i8(qG), _i8(qW)
    assert qG.shape == d.y_shape and qW.shape == d.w_shape
    dX = np.zeros(d.x_shape, np.float32)
    acc = np.zeros(d.x_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv_bwd_data_int8(C.byref(dd), _p(qG, C.c_int8), C.c_float(s_global), _p(qW, C.c_int8),
                                          C.c_float(s_w), _p(dX, C.c_float), _p(acc, C.c_int32), C.byref(ovf)),
         "conv_bwd_data_int8")
    return dX, acc, bool(ovf.value)


def conv_bwd_data_int8_chan(d: ConvDesc, vq, s_chan, qW, s_w):
    """Depthwise layers only: data gradient from the per-channel copy, de-quantized per channel."""
    vq, qW = _i8(vq), _i8(qW)
    sc = _f32(s_chan)
    assert vq.shape == d.y_shape and qW.shape == d.w_shape and sc.shape == (d.Cout,)
    dX = np.zeros(d.x_shape, np.float32)
    acc = np.zeros(d.x_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv_bwd_data_int8_chan(C.byref(dd), _p(vq, C.c_int8), _p(sc, C.c_float), _p(qW, C.c_int8),
                                               C.c_float(s_w), _p(dX, C.c_float), _p(acc, C.c_int32), C.byref(ovf)),
         "conv_bwd_data_int8_chan")
    return dX, acc, bool(ovf.value)


def conv_bwd_filter_int8(d: ConvDesc, qX, s_x, vq, s_chan):
    qX, vq = _i8(qX), _i8(vq)
    s_chan = _f32(s_chan)
    assert qX.shape == d.x_shape and vq.shape == d.y_shape and s_chan.shape == (d.Cout,)
    dW = np.zeros(d.w_shape, np.float32)
    acc = np.zeros(d.w_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv_bwd_filter_int8(C.byref(dd), _p(qX, C.c_int8), C.c_float(s_x), _p(vq, C.c_int8),
                                            _p(s_chan, C.c_float), _p(dW, C.c_float), _p(acc, C.c_int32),
                                            C.byref(ovf)), "conv_bwd_filter_int8")
    return dW, acc, bool(ovf.value)


def bf16_bits(x) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest with ties to even, for finite inputs.

    Not part of the paper's method: the storage rule of the optional narrow data-gradient output.  bfloat16 is the upper
    half of an IEEE binary32; rounding adds half an ulp of the kept part (0x7FFF plus the kept part's last bit, which
    settles ties towards even) and truncates."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def conv_bwd_data_int8_bf16(d: ConvDesc, qG, s_global, qW, s_w) -> np.ndarray:
    """The data gradient of conv_bwd_data_int8, stored as bfloat16 bit patterns."""
    dX, _, ovf = conv_bwd_data_int8(d, qG, s_global, qW, s_w)
    assert not ovf
    return bf16_bits(dX)


def conv_bwd_filter_int8_bf16(d: ConvDesc, qX, s_x, vq, s_chan) -> np.ndarray:
    """The filter gradient of conv_bwd_filter_int8, stored as bfloat16 bit patterns."""
    dW, _, ovf = conv_bwd_filter_int8(d, qX, s_x, vq, s_chan)
    assert not ovf
    return bf16_bits(dW)


def clip_search(dY, alpha: float, J: int):
    """Eq. "e" on a grid of J clip values per channel: (err [C, J] fp64, best_s [C] fp32, best_j [C] int32, 1-based)."""
    g = _f32(dY)
    N, Cc, H, W = g.shape
    err = np.zeros((Cc, J), np.float64)
    best_s = np.zeros(Cc, np.float32)
    best_j = np.zeros(Cc, np.int32)
    _chk(lib().daq_ref_clip_search(_p(g, C.c_float), N, Cc, H, W, C.c_float(alpha), J, _p(err, C.c_double), _p(best_s, C.c_float),
                                   _p(best_j, C.c_int32)), "clip_search")
    return err, best_s, best_j


# --------------------------------------------------------------------------------------------- 3-D convolution

class _Desc3(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("N", "Cin", "Din", "Hin", "Win", "Cout", "kD", "kH", "kW", "strideD", "strideH", "strideW",
                                       "padD", "padH", "padW", "dilD", "dilH", "dilW", "groups")]


@dataclass(frozen=True)
class Conv3dDesc:
    N: int
    Cin: int
    Din: int
    Hin: int
    Win: int
    Cout: int
    kD: int
    kH: int
    kW: int
    strideD: int = 1
    strideH: int = 1
    strideW: int = 1
    padD: int = 0
    padH: int = 0
    padW: int = 0
    dilD: int = 1
    dilH: int = 1
    dilW: int = 1
    groups: int = 1

    def fields(self):
        return (self.N, self.Cin, self.Din, self.Hin, self.Win, self.Cout, self.kD, self.kH, self.kW, self.strideD, self.strideH,
                self.strideW, self.padD, self.padH, self.padW, self.dilD, self.dilH, self.dilW, self.groups)

    def c(self) -> _Desc3:
        return _Desc3(*self.fields())

    @staticmethod
    def _out(i, p, dil, k, s):
        return (i + 2 * p - dil * (k - 1) - 1) // s + 1

    @property
    def Do(self):
        return self._out(self.Din, self.padD, self.dilD, self.kD, self.strideD)

    @property
    def Ho(self):
        return self._out(self.Hin, self.padH, self.dilH, self.kH, self.strideH)

    @property
    def Wo(self):
        return self._out(self.Win, self.padW, self.dilW, self.kW, self.strideW)

    @property
    def x_shape(self):
        return (self.N, self.Cin, self.Din, self.Hin, self.Win)

    @property
    def w_shape(self):
        return (self.Cout, self.Cin // self.groups, self.kD, self.kH, self.kW)

    @property
    def y_shape(self):
        return (self.N, self.Cout, self.Do, self.Ho, self.Wo)


def conv3d_fwd_acc(d: Conv3dDesc, qX, qW):
    qX, qW = _i8(qX), _i8(qW)
    assert qX.shape == d.x_shape and qW.shape == d.w_shape
    acc = np.zeros(d.y_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv3d_fwd_acc(C.byref(dd), _p(qX, C.c_int8), _p(qW, C.c_int8), _p(acc, C.c_int32), C.byref(ovf)), "conv3d_fwd_acc")
    return acc, bool(ovf.value)


def conv3d_bwd_data_acc(d: Conv3dDesc, qG, qW):
    qG, qW = _i8(qG), _i8(qW)
    assert qG.shape == d.y_shape and qW.shape == d.w_shape
    acc = np.zeros(d.x_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv3d_bwd_data_acc(C.byref(dd), _p(qG, C.c_int8), _p(qW, C.c_int8), _p(acc, C.c_int32), C.byref(ovf)),
         "conv3d_bwd_data_acc")
    return acc, bool(ovf.value)


def conv3d_bwd_filter_acc(d: Conv3dDesc, qX, qG):
    qX, qG = _i8(qX), _i8(qG)
    assert qX.shape == d.x_shape and qG.shape == d.y_shape
    acc = np.zeros(d.w_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv3d_bwd_filter_acc(C.byref(dd), _p(qX, C.c_int8), _p(qG, C.c_int8), _p(acc, C.c_int32), C.byref(ovf)),
         "conv3d_bwd_filter_acc")
    return acc, bool(ovf.value)


def conv3d_fwd_int8(d: Conv3dDesc, X, Wt) -> Fwd:
    X, Wt = _f32(X), _f32(Wt)
    assert X.shape == d.x_shape and Wt.shape == d.w_shape
    qX, qW = np.zeros(d.x_shape, np.int8), np.zeros(d.w_shape, np.int8)
    sx, sw = np.zeros(1, np.float32), np.zeros(1, np.float32)
    Y, acc = np.zeros(d.y_shape, np.float32), np.zeros(d.y_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv3d_fwd_int8(C.byref(dd), _p(X, C.c_float), _p(Wt, C.c_float), _p(qX, C.c_int8), _p(qW, C.c_int8),
                                       _p(sx, C.c_float), _p(sw, C.c_float), _p(Y, C.c_float), _p(acc, C.c_int32), C.byref(ovf)),
         "conv3d_fwd_int8")
    return Fwd(qX, qW, float(sx[0]), float(sw[0]), Y, acc, bool(ovf.value))


def conv3d_bwd_data_int8(d: Conv3dDesc, qG, s_global, qW, s_w):
    qG, qW = _i8(qG), _i8(qW)
    assert qG.shape == d.y_shape and qW.shape == d.w_shape
    dX, acc = np.zeros(d.x_shape, np.float32), np.zeros(d.x_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv3d_bwd_data_int8(C.byref(dd), _p(qG, C.c_int8), C.c_float(s_global), _p(qW, C.c_int8), C.c_float(s_w),
                                            _p(dX, C.c_float), _p(acc, C.c_int32), C.byref(ovf)), "conv3d_bwd_data_int8")
    return dX, acc, bool(ovf.value)


def conv3d_bwd_filter_int8(d: Conv3dDesc, qX, s_x, vq, s_chan):
    qX, vq = _i8(qX), _i8(vq)
    s_chan = _f32(s_chan)
    assert qX.shape == d.x_shape and vq.shape == d.y_shape and s_chan.shape == (d.Cout,)
    dW, acc = np.zeros(d.w_shape, np.float32), np.zeros(d.w_shape, np.int32)
    ovf = C.c_int(0)
    dd = d.c()
    _chk(lib().daq_ref_conv3d_bwd_filter_int8(C.byref(dd), _p(qX, C.c_int8), C.c_float(s_x), _p(vq, C.c_int8), _p(s_chan, C.c_float),
                                              _p(dW, C.c_float), _p(acc, C.c_int32), C.byref(ovf)), "conv3d_bwd_filter_int8")
    return dW, acc, bool(ovf.value)


def quantize_grad3d(dY, s_state, **kw) -> QuantGrad:
    """Algorithm 1's quantizer on an (N, C, D, H, W) gradient: its statistics run over (n, d, h, w), i.e. the 2-D routine
    on the tensor viewed as (N, C, D*H, W); the codes are returned in the 5-D shape."""
    g = _f32(dY)
    N, Cc, D, H, W = g.shape
    q = quantize_grad(g.reshape(N, Cc, D * H, W), s_state, **kw)
    q.vq = q.vq.reshape(g.shape)
    q.qg = q.qg.reshape(g.shape)
    return q
