"""Thin ctypes binding of ``libdaq.so`` (argument marshalling only).

Every step of the path runs in the library's HIP kernels; PyTorch is used for
device memory and streams.  The module raises at import time if the library has
not been built -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdaq.so")

OK, ERR_INVALID_ARG, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP, ERR_SCRATCH_LIMIT = range(6)
ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1
SCHEME_DAQ, SCHEME_GQ, SCHEME_GVQ, SCHEME_MCS = range(4)
CLASS_GAUSS, CLASS_INVT = 0, 1
OP_QUANTIZE_GRAD, OP_CONV_FWD, OP_CONV_BWD_DATA, OP_CONV_BWD_FILTER, OP_CONV_BWD, OP_CLIP_SEARCH = range(6)
LAYOUT_NHWC, LAYOUT_CNHW = 0, 1
SCHEDULE_AUTO, SCHEDULE_THREE_SWEEPS, SCHEDULE_EARLY_COPY, SCHEDULE_CHANNEL_RESIDENT = range(4)

EXPORTS = [
    "daq_out_h", "daq_out_w", "daq_layout_vq", "daq_layout_qg", "daq_layout_qx_nhwc", "daq_layout_qx_cnhw",
    "daq_layout_qw", "daq_workspace_bytes", "daq_quantize_grad", "daq_quantize_grad_scheme", "daq_quantize_grad_bf16", "daq_quantize_grad_ex", "daq_quantize_grad_split", "daq_quantize_grad_from_stats", "daq_quantize_grad_noalloc", "daq_conv_fwd_int8", "daq_conv_fwd_int8_ex", "daq_conv_bwd_data_int8",
    "daq_conv_bwd_filter_int8", "daq_conv_bwd_int8", "daq_conv_bwd_data_int8_bf16", "daq_conv_bwd_filter_int8_bf16", "daq_conv_bwd_data_int8_chan", "daq_clip_search", "daq_conv3d_out_d", "daq_conv3d_out_h", "daq_conv3d_out_w", "daq_conv3d_carriers", "daq_conv3d_qw_bytes",
    "daq_conv3d_workspace_bytes", "daq_quantize_grad3d", "daq_conv3d_fwd_int8", "daq_conv3d_bwd_data_int8", "daq_conv3d_bwd_filter_int8",
    "daq_prof_begin", "daq_prof_end", "daq_status_string", "daq_ceiling_mfma_i8", "daq_ceiling_stream",
]


class DaqError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {status_string(code)} (code {code})")


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "Cin", "Hin", "Win", "Cout", "kH", "kW", "strideH", "strideW", "padH",
                                         "padW", "dilH", "dilW", "groups")]

    @classmethod
    def make(cls, N, Cin, Hin, Win, Cout, kH, kW, strideH=1, strideW=1, padH=0, padW=0, dilH=1, dilW=1, groups=1):
        return cls(N, Cin, Hin, Win, Cout, kH, kW, strideH, strideW, padH, padW, dilH, dilW, groups)

    @property
    def Ho(self):
        return int(lib().daq_out_h(C.byref(self)))

    @property
    def Wo(self):
        return int(lib().daq_out_w(C.byref(self)))

    @property
    def x_shape(self):
        return (self.N, self.Cin, self.Hin, self.Win)

    @property
    def w_shape(self):
        return (self.Cout, self.Cin // self.groups, self.kH, self.kW)

    @property
    def y_shape(self):
        return (self.N, self.Cout, self.Ho, self.Wo)


class Conv3dDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "Cin", "Din", "Hin", "Win", "Cout", "kD", "kH", "kW", "strideD", "strideH", "strideW",
                                         "padD", "padH", "padW", "dilD", "dilH", "dilW", "groups")]

    @property
    def Do(self):
        return int(lib().daq_conv3d_out_d(C.byref(self)))

    @property
    def Ho(self):
        return int(lib().daq_conv3d_out_h(C.byref(self)))

    @property
    def Wo(self):
        return int(lib().daq_conv3d_out_w(C.byref(self)))

    @property
    def x_shape(self):
        return (self.N, self.Cin, self.Din, self.Hin, self.Win)

    @property
    def w_shape(self):
        return (self.Cout, self.Cin // self.groups, self.kD, self.kH, self.kW)

    @property
    def y_shape(self):
        return (self.N, self.Cout, self.Do, self.Ho, self.Wo)


class Layout(C.Structure):
    _fields_ = [("kind", C.c_int32), ("C", C.c_int32), ("N", C.c_int32), ("H", C.c_int32), ("W", C.c_int32),
                ("bytes", C.c_int64), ("c_pitch", C.c_int32), ("img_rows", C.c_int32), ("row_pitch", C.c_int32),
                ("phases_h", C.c_int32), ("phases_w", C.c_int32), ("org_h", C.c_int32), ("org_w", C.c_int32),
                ("chan_pitch", C.c_int64), ("plane_pitch", C.c_int64), ("lead", C.c_int64)]

    def offsets(self) -> np.ndarray:
        """Byte offset of every logical element, as an int64 array of shape (N, C, H, W)."""
        n = np.arange(self.N, dtype=np.int64).reshape(-1, 1, 1, 1)
        c = np.arange(self.C, dtype=np.int64).reshape(1, -1, 1, 1)
        h = np.arange(self.H, dtype=np.int64).reshape(1, 1, -1, 1)
        w = np.arange(self.W, dtype=np.int64).reshape(1, 1, 1, -1)
        if self.kind == LAYOUT_NHWC:
            return ((n * self.H + h) * self.W + w) * self.c_pitch + c
        hh, ww = h + self.org_h, w + self.org_w
        plane = (hh % self.phases_h) * self.phases_w + (ww % self.phases_w)
        return (c * self.chan_pitch + plane * self.plane_pitch + self.lead
                + (n * self.img_rows + hh // self.phases_h) * self.row_pitch + ww // self.phases_w)

    def unpack(self, buf) -> np.ndarray:
        """Device/host int8 buffer in this layout -> logical int8 NCHW numpy array."""
        flat = buf.detach().cpu().numpy().view(np.int8).ravel() if isinstance(buf, torch.Tensor) else np.asarray(buf).view(np.int8).ravel()
        return flat[self.offsets()]

    def pack(self, codes: np.ndarray) -> np.ndarray:
        """Logical int8 NCHW array -> flat int8 buffer in this layout (padding bytes zero)."""
        codes = np.ascontiguousarray(codes, dtype=np.int8)
        assert codes.shape == (self.N, self.C, self.H, self.W)
        out = np.zeros(self.bytes, dtype=np.int8)
        out[self.offsets()] = codes
        return out

    def padding_is_zero(self, buf) -> bool:
        flat = buf.detach().cpu().numpy().view(np.int8).ravel().copy()
        flat[self.offsets().ravel()] = 0
        return not flat.any()


class WPackLayout(C.Structure):
    _fields_ = [("bytes", C.c_int64), ("off_plain", C.c_int64), ("off_fwd", C.c_int64), ("off_bwd", C.c_int64),
                ("cig_pitch", C.c_int32), ("cog_pitch", C.c_int32),
                ("off_fwd_frag", C.c_int64), ("off_bwd_frag", C.c_int64)]

    @staticmethod
    def _frag(mat: np.ndarray) -> np.ndarray:
        """[tap][row][k] -> fragment order (see daq.h): [k/64][tap][row/32][(k%64)/32][(k%32)/16][row%32][k%16]."""
        taps, rows, K = mat.shape
        RB, KC = -(-rows // 32), -(-K // 64)
        pad = np.zeros((taps, RB * 32, KC * 64), np.int8)
        pad[:, :rows, :K] = mat
        v = pad.reshape(taps, RB, 32, KC, 2, 2, 16)          # tap, rb, r, kc, sub, kg, b
        return np.ascontiguousarray(v.transpose(3, 0, 1, 4, 5, 2, 6)).ravel()

    def pack(self, d: ConvDesc, qW: np.ndarray) -> np.ndarray:
        qW = np.ascontiguousarray(qW, dtype=np.int8)
        Cout, cig, kH, kW = d.w_shape
        assert qW.shape == (Cout, cig, kH, kW)
        cog, taps = Cout // d.groups, kH * kW
        out = np.zeros(self.bytes, dtype=np.int8)
        out[self.off_plain:self.off_plain + qW.size] = qW.ravel()
        fwd = np.zeros((taps, Cout, self.cig_pitch), np.int8)
        fwd[:, :, :cig] = qW.reshape(Cout, cig, taps).transpose(2, 0, 1)
        out[self.off_fwd:self.off_fwd + fwd.size] = fwd.ravel()
        bwd = np.zeros((taps, d.Cin, self.cog_pitch), np.int8)
        for g in range(d.groups):
            blk = qW[g * cog:(g + 1) * cog].reshape(cog, cig, taps)      # [col][cl][tap]
            bwd[:, g * cig:(g + 1) * cig, :cog] = blk.transpose(2, 1, 0)  # [tap][cl][col]
        out[self.off_bwd:self.off_bwd + bwd.size] = bwd.ravel()
        if d.groups == 1:
            ff = self._frag(fwd[:, :, :cig])
            out[self.off_fwd_frag:self.off_fwd_frag + ff.size] = ff
            bf = self._frag(bwd[:, :, :cog])
            out[self.off_bwd_frag:self.off_bwd_frag + bf.size] = bf
        return out

    def unpack_plain(self, d: ConvDesc, buf) -> np.ndarray:
        flat = buf.detach().cpu().numpy().view(np.int8).ravel()
        n = int(np.prod(d.w_shape))
        return flat[self.off_plain:self.off_plain + n].reshape(d.w_shape)


class QuantizeOpts(C.Structure):
    _fields_ = [("scheme", C.c_int32), ("schedule", C.c_int32), ("dy_bf16", C.c_int32), ("reserved", C.c_int32)]


class ProfRow(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("total_ms", C.c_double), ("launches", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(L, name)  # AttributeError if a declared symbol is not exported
        L.daq_out_h.restype = C.c_int32
        L.daq_out_w.restype = C.c_int32
        L.daq_workspace_bytes.restype = C.c_size_t
        L.daq_workspace_bytes.argtypes = [C.c_int, C.POINTER(ConvDesc)]
        L.daq_status_string.restype = C.c_char_p
        L.daq_status_string.argtypes = [C.c_int]
        vp, f32, u64, sz = C.c_void_p, C.c_float, C.c_uint64, C.c_size_t
        L.daq_quantize_grad.argtypes = [C.POINTER(ConvDesc), vp, vp, f32, f32, f32, C.c_int, u64, vp, vp, vp, vp, vp,
                                        vp, vp, sz, vp]
        L.daq_quantize_grad_scheme.argtypes = [C.POINTER(ConvDesc), vp, vp, f32, f32, f32, C.c_int, u64, C.c_int, vp, vp,
                                               vp, vp, vp, vp, vp, sz, vp]
        L.daq_quantize_grad_bf16.argtypes = L.daq_quantize_grad_scheme.argtypes
        L.daq_quantize_grad_ex.argtypes = [C.POINTER(ConvDesc), vp, vp, f32, f32, f32, C.c_int, u64, C.POINTER(QuantizeOpts),
                                           vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.daq_quantize_grad_split.argtypes = L.daq_quantize_grad_ex.argtypes + [vp]
        L.daq_quantize_grad_from_stats.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp, vp, f32, f32, f32, C.c_int, u64,
                                                   C.POINTER(QuantizeOpts), vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
        L.daq_quantize_grad_noalloc.argtypes = [C.POINTER(ConvDesc), vp, vp, f32, f32, f32, C.c_int, u64, vp, vp, vp, vp, vp,
                                                vp, vp]
        L.daq_conv_fwd_int8.argtypes = [C.POINTER(ConvDesc)] + [vp] * 10 + [sz, vp]
        L.daq_conv_fwd_int8_ex.argtypes = [C.POINTER(ConvDesc)] + [vp] * 9 + [C.c_int, vp, sz, vp]
        L.daq_conv_bwd_data_int8.argtypes = [C.POINTER(ConvDesc)] + [vp] * 7 + [sz, vp]
        L.daq_conv_bwd_filter_int8.argtypes = [C.POINTER(ConvDesc)] + [vp] * 7 + [sz, vp]
        L.daq_conv_bwd_data_int8_chan.argtypes = [C.POINTER(ConvDesc)] + [vp] * 7 + [sz, vp]
        L.daq_conv_bwd_int8.argtypes = [C.POINTER(ConvDesc)] + [vp] * 13 + [sz, vp]
        L.daq_conv_bwd_data_int8_bf16.argtypes = [C.POINTER(ConvDesc)] + [vp] * 6 + [sz, vp]
        L.daq_conv_bwd_filter_int8_bf16.argtypes = [C.POINTER(ConvDesc)] + [vp] * 6 + [sz, vp]
        L.daq_clip_search.argtypes = [C.POINTER(ConvDesc), vp, f32, C.c_int32, vp, vp, vp, vp, sz, vp]
        L.daq_conv3d_carriers.argtypes = [C.POINTER(Conv3dDesc), C.POINTER(ConvDesc), C.POINTER(ConvDesc)]
        L.daq_conv3d_qw_bytes.restype = C.c_int64
        L.daq_conv3d_qw_bytes.argtypes = [C.POINTER(Conv3dDesc)]
        L.daq_conv3d_workspace_bytes.restype = C.c_size_t
        L.daq_conv3d_workspace_bytes.argtypes = [C.c_int, C.POINTER(Conv3dDesc)]
        L.daq_quantize_grad3d.argtypes = [C.POINTER(Conv3dDesc), vp, vp, f32, f32, f32, C.c_int, u64, C.POINTER(QuantizeOpts),
                                          vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.daq_conv3d_fwd_int8.argtypes = [C.POINTER(Conv3dDesc)] + [vp] * 10 + [sz, vp]
        L.daq_conv3d_bwd_data_int8.argtypes = [C.POINTER(Conv3dDesc)] + [vp] * 7 + [sz, vp]
        L.daq_conv3d_bwd_filter_int8.argtypes = [C.POINTER(Conv3dDesc)] + [vp] * 7 + [sz, vp]
        L.daq_prof_end.argtypes = [C.POINTER(ProfRow), C.c_int32, C.POINTER(C.c_int32)]
        L.daq_ceiling_mfma_i8.argtypes = [C.c_int32, C.c_int32, vp, C.POINTER(C.c_double), vp]
        L.daq_ceiling_stream.argtypes = [C.c_int32, vp, vp, sz, C.c_int32, vp, vp]
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().daq_status_string(code).decode()


def _check(code: int, what: str):
    if code != OK:
        raise DaqError(code, what)


def _layout(fn_name: str, d: ConvDesc) -> Layout:
    L = Layout()
    _check(getattr(lib(), fn_name)(C.byref(d), C.byref(L)), fn_name)
    return L


def layout_vq(d): return _layout("daq_layout_vq", d)
def layout_qg(d): return _layout("daq_layout_qg", d)
def layout_qx_nhwc(d): return _layout("daq_layout_qx_nhwc", d)
def layout_qx_cnhw(d): return _layout("daq_layout_qx_cnhw", d)


def layout_qw(d: ConvDesc) -> WPackLayout:
    L = WPackLayout()
    _check(lib().daq_layout_qw(C.byref(d), C.byref(L)), "daq_layout_qw")
    return L


def workspace_bytes(op: int, d: ConvDesc) -> int:
    return int(lib().daq_workspace_bytes(op, C.byref(d)))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ------------------------------------------------------------------------------------------------
# the four entry points (same names as the C ABI, without the prefix)
# ------------------------------------------------------------------------------------------------
@dataclass
class QuantGrad:
    vq: torch.Tensor        # int8, layout_vq
    qg: torch.Tensor        # int8, layout_qg
    s_chan: torch.Tensor    # fp32 [Cout]
    s_global: torch.Tensor  # fp32 [1]
    cls: torch.Tensor       # u8 [Cout]
    stats: Optional[torch.Tensor]  # fp32 [Cout,4]
    workspace: torch.Tensor


def alloc_quantize_grad(d: ConvDesc, device="cuda", want_stats=True) -> QuantGrad:
    i8 = dict(dtype=torch.int8, device=device)
    return QuantGrad(
        vq=torch.empty(layout_vq(d).bytes, **i8), qg=torch.empty(layout_qg(d).bytes, **i8),
        s_chan=torch.empty(d.Cout, dtype=torch.float32, device=device),
        s_global=torch.empty(1, dtype=torch.float32, device=device),
        cls=torch.empty(d.Cout, dtype=torch.uint8, device=device),
        stats=torch.empty((d.Cout, 4), dtype=torch.float32, device=device) if want_stats else None,
        workspace=_ws(workspace_bytes(OP_QUANTIZE_GRAD, d), device))


def quantize_grad(d: ConvDesc, dY: torch.Tensor, s_state: torch.Tensor, k=1.0, A=0.8, lam=0.3, mode=ROUND_NEAREST,
                  seed=0, out: Optional[QuantGrad] = None, stream=None) -> QuantGrad:
    """daq_quantize_grad.  ``s_state`` is updated in place."""
    assert dY.is_cuda and dY.dtype == torch.float32 and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    assert s_state.is_cuda and s_state.dtype == torch.float32 and s_state.numel() == d.Cout
    if out is None:
        out = alloc_quantize_grad(d, dY.device)
    rc = lib().daq_quantize_grad(C.byref(d), _ptr(dY), _ptr(s_state), k, A, lam, mode, seed, _ptr(out.vq), _ptr(out.qg),
                                 _ptr(out.s_chan), _ptr(out.s_global), _ptr(out.cls), _ptr(out.stats),
                                 _ptr(out.workspace), out.workspace.numel(), _stream(stream))
    _check(rc, "daq_quantize_grad")
    return out


def quantize_grad_ex(d: ConvDesc, dY: torch.Tensor, s_state: torch.Tensor, scheme: int = SCHEME_DAQ,
                     schedule: int = SCHEDULE_AUTO, k=1.0, A=0.8, lam=0.3, mode=ROUND_NEAREST, seed=0,
                     out: Optional[QuantGrad] = None, stream=None) -> QuantGrad:
    """daq_quantize_grad_ex: every option explicit; ``dY`` is fp32 or bfloat16.  ``s_state`` is updated in place."""
    assert dY.is_cuda and dY.dtype in (torch.float32, torch.bfloat16) and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    assert s_state.is_cuda and s_state.dtype == torch.float32 and s_state.numel() == d.Cout
    if out is None:
        out = alloc_quantize_grad(d, dY.device)
    opts = QuantizeOpts(scheme, schedule, 1 if dY.dtype == torch.bfloat16 else 0, 0)
    rc = lib().daq_quantize_grad_ex(C.byref(d), _ptr(dY), _ptr(s_state), k, A, lam, mode, seed, C.byref(opts), _ptr(out.vq),
                                    _ptr(out.qg), _ptr(out.s_chan), _ptr(out.s_global), _ptr(out.cls), _ptr(out.stats),
                                    _ptr(out.workspace), out.workspace.numel(), _stream(stream))
    _check(rc, "daq_quantize_grad_ex")
    return out


def quantize_grad_split(d: ConvDesc, dY: torch.Tensor, s_state: torch.Tensor, side_stream, scheme: int = SCHEME_DAQ,
                        schedule: int = SCHEDULE_AUTO, k=1.0, A=0.8, lam=0.3, mode=ROUND_NEAREST, seed=0,
                        out: Optional[QuantGrad] = None, stream=None) -> QuantGrad:
    """daq_quantize_grad_split: ``qg`` and ``s_global`` are ordered on ``stream``, everything else on ``side_stream``."""
    assert dY.is_cuda and dY.dtype in (torch.float32, torch.bfloat16) and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    assert s_state.is_cuda and s_state.dtype == torch.float32 and s_state.numel() == d.Cout
    if out is None:
        out = alloc_quantize_grad(d, dY.device)
    opts = QuantizeOpts(scheme, schedule, 1 if dY.dtype == torch.bfloat16 else 0, 0)
    rc = lib().daq_quantize_grad_split(C.byref(d), _ptr(dY), _ptr(s_state), k, A, lam, mode, seed, C.byref(opts), _ptr(out.vq),
                                       _ptr(out.qg), _ptr(out.s_chan), _ptr(out.s_global), _ptr(out.cls), _ptr(out.stats),
                                       _ptr(out.workspace), out.workspace.numel(), _stream(stream), _stream(side_stream))
    _check(rc, "daq_quantize_grad_split")
    return out


def quantize_grad_from_stats(d: ConvDesc, dY: torch.Tensor, ch_absmax: torch.Tensor, ch_sum: torch.Tensor,
                             ch_sumsq: torch.Tensor, s_state: torch.Tensor, side_stream=None, scheme: int = SCHEME_DAQ,
                             schedule: int = SCHEDULE_AUTO, k=1.0, A=0.8, lam=0.3, mode=ROUND_NEAREST, seed=0,
                             out: Optional[QuantGrad] = None, stream=None) -> QuantGrad:
    """daq_quantize_grad_from_stats: the producer of ``dY`` supplies |g|max (fp32), sum and sum of squares (fp64) per channel."""
    assert dY.is_cuda and dY.dtype in (torch.float32, torch.bfloat16) and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    assert s_state.is_cuda and s_state.dtype == torch.float32 and s_state.numel() == d.Cout
    assert ch_absmax.is_cuda and ch_absmax.dtype == torch.float32 and ch_absmax.numel() == d.Cout and ch_absmax.is_contiguous()
    for a in (ch_sum, ch_sumsq):
        assert a.is_cuda and a.dtype == torch.float64 and a.numel() == d.Cout and a.is_contiguous()
    if out is None:
        out = alloc_quantize_grad(d, dY.device)
    opts = QuantizeOpts(scheme, schedule, 1 if dY.dtype == torch.bfloat16 else 0, 0)
    rc = lib().daq_quantize_grad_from_stats(C.byref(d), _ptr(dY), _ptr(ch_absmax), _ptr(ch_sum), _ptr(ch_sumsq), _ptr(s_state),
                                            k, A, lam, mode, seed, C.byref(opts), _ptr(out.vq), _ptr(out.qg), _ptr(out.s_chan),
                                            _ptr(out.s_global), _ptr(out.cls), _ptr(out.stats), _ptr(out.workspace),
                                            out.workspace.numel(), _stream(stream),
                                            _stream(side_stream) if side_stream is not None else None)
    _check(rc, "daq_quantize_grad_from_stats")
    return out


def quantize_grad_noalloc(d: ConvDesc, dY: torch.Tensor, s_state: torch.Tensor, out: QuantGrad, k=1.0, A=0.8, lam=0.3,
                          mode=ROUND_NEAREST, seed=0, stream=None) -> QuantGrad:
    """daq_quantize_grad_noalloc: the outputs are the caller's (``out``; its workspace is not used), nothing is allocated."""
    assert dY.is_cuda and dY.dtype == torch.float32 and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    assert s_state.is_cuda and s_state.dtype == torch.float32 and s_state.numel() == d.Cout
    rc = lib().daq_quantize_grad_noalloc(C.byref(d), _ptr(dY), _ptr(s_state), k, A, lam, mode, seed, _ptr(out.vq), _ptr(out.qg),
                                         _ptr(out.s_chan), _ptr(out.s_global), _ptr(out.cls), _ptr(out.stats), _stream(stream))
    _check(rc, "daq_quantize_grad_noalloc")
    return out


def quantize_grad_bf16(d: ConvDesc, dY: torch.Tensor, s_state: torch.Tensor, scheme: int = SCHEME_DAQ, k=1.0, A=0.8, lam=0.3,
                       mode=ROUND_NEAREST, seed=0, out: Optional[QuantGrad] = None, stream=None) -> QuantGrad:
    """daq_quantize_grad_bf16: ``dY`` is a bfloat16 tensor.  ``s_state`` is updated in place."""
    assert dY.is_cuda and dY.dtype == torch.bfloat16 and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    assert s_state.is_cuda and s_state.dtype == torch.float32 and s_state.numel() == d.Cout
    if out is None:
        out = alloc_quantize_grad(d, dY.device)
    rc = lib().daq_quantize_grad_bf16(C.byref(d), _ptr(dY), _ptr(s_state), k, A, lam, mode, seed, scheme, _ptr(out.vq),
                                      _ptr(out.qg), _ptr(out.s_chan), _ptr(out.s_global), _ptr(out.cls), _ptr(out.stats),
                                      _ptr(out.workspace), out.workspace.numel(), _stream(stream))
    _check(rc, "daq_quantize_grad_bf16")
    return out


def quantize_grad_scheme(d: ConvDesc, dY: torch.Tensor, s_state: torch.Tensor, scheme: int, k=1.0, A=0.8, lam=0.3,
                         mode=ROUND_NEAREST, seed=0, out: Optional[QuantGrad] = None, stream=None) -> QuantGrad:
    """daq_quantize_grad_scheme.  ``s_state`` is updated in place."""
    assert dY.is_cuda and dY.dtype == torch.float32 and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    assert s_state.is_cuda and s_state.dtype == torch.float32 and s_state.numel() == d.Cout
    if out is None:
        out = alloc_quantize_grad(d, dY.device)
    rc = lib().daq_quantize_grad_scheme(C.byref(d), _ptr(dY), _ptr(s_state), k, A, lam, mode, seed, scheme, _ptr(out.vq),
                                        _ptr(out.qg), _ptr(out.s_chan), _ptr(out.s_global), _ptr(out.cls),
                                        _ptr(out.stats), _ptr(out.workspace), out.workspace.numel(), _stream(stream))
    _check(rc, "daq_quantize_grad_scheme")
    return out


@dataclass
class Fwd:
    qx_nhwc: torch.Tensor
    qx_cnhw: torch.Tensor
    qw: torch.Tensor
    s_x: torch.Tensor
    s_w: torch.Tensor
    Y: torch.Tensor
    acc: Optional[torch.Tensor]
    workspace: torch.Tensor


def alloc_fwd(d: ConvDesc, device="cuda", want_acc=False) -> Fwd:
    i8 = dict(dtype=torch.int8, device=device)
    f32 = dict(dtype=torch.float32, device=device)
    return Fwd(qx_nhwc=torch.empty(layout_qx_nhwc(d).bytes, **i8), qx_cnhw=torch.empty(layout_qx_cnhw(d).bytes, **i8),
               qw=torch.empty(layout_qw(d).bytes, **i8), s_x=torch.empty(1, **f32), s_w=torch.empty(1, **f32),
               Y=torch.empty(d.y_shape, **f32),
               acc=torch.empty(d.y_shape, dtype=torch.int32, device=device) if want_acc else None,
               workspace=_ws(workspace_bytes(OP_CONV_FWD, d), device))


def conv_fwd_int8(d: ConvDesc, X: torch.Tensor, W: torch.Tensor, out: Optional[Fwd] = None, want_acc=False,
                  stream=None, schedule: Optional[int] = None) -> Fwd:
    """daq_conv_fwd_int8, or daq_conv_fwd_int8_ex when a ``schedule`` is given."""
    assert X.is_cuda and X.dtype == torch.float32 and X.is_contiguous() and tuple(X.shape) == d.x_shape
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == d.w_shape
    if out is None:
        out = alloc_fwd(d, X.device, want_acc)
    if schedule is None:
        rc = lib().daq_conv_fwd_int8(C.byref(d), _ptr(X), _ptr(W), _ptr(out.qx_nhwc), _ptr(out.qx_cnhw), _ptr(out.qw),
                                     _ptr(out.s_x), _ptr(out.s_w), _ptr(out.Y), _ptr(out.acc), _ptr(out.workspace),
                                     out.workspace.numel(), _stream(stream))
        _check(rc, "daq_conv_fwd_int8")
    else:
        rc = lib().daq_conv_fwd_int8_ex(C.byref(d), _ptr(X), _ptr(W), _ptr(out.qx_nhwc), _ptr(out.qx_cnhw), _ptr(out.qw),
                                        _ptr(out.s_x), _ptr(out.s_w), _ptr(out.Y), _ptr(out.acc), schedule,
                                        _ptr(out.workspace), out.workspace.numel(), _stream(stream))
        _check(rc, "daq_conv_fwd_int8_ex")
    return out


def conv_bwd_data_int8(d: ConvDesc, qg: torch.Tensor, s_global: torch.Tensor, qw: torch.Tensor, s_w: torch.Tensor,
                       dX: Optional[torch.Tensor] = None, acc: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if dX is None:
        dX = torch.empty(d.x_shape, dtype=torch.float32, device=qg.device)
    if workspace is None:
        workspace = _ws(workspace_bytes(OP_CONV_BWD_DATA, d), qg.device)
    rc = lib().daq_conv_bwd_data_int8(C.byref(d), _ptr(qg), _ptr(s_global), _ptr(qw), _ptr(s_w), _ptr(dX), _ptr(acc),
                                      _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "daq_conv_bwd_data_int8")
    return dX


def conv_bwd_filter_int8(d: ConvDesc, qx_cnhw: torch.Tensor, s_x: torch.Tensor, vq: torch.Tensor,
                         s_chan: torch.Tensor, dW: Optional[torch.Tensor] = None, acc: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if dW is None:
        dW = torch.empty(d.w_shape, dtype=torch.float32, device=vq.device)
    if workspace is None:
        workspace = _ws(workspace_bytes(OP_CONV_BWD_FILTER, d), vq.device)
    rc = lib().daq_conv_bwd_filter_int8(C.byref(d), _ptr(qx_cnhw), _ptr(s_x), _ptr(vq), _ptr(s_chan), _ptr(dW),
                                        _ptr(acc), _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "daq_conv_bwd_filter_int8")
    return dW


def conv_bwd_data_int8_bf16(d: ConvDesc, qg: torch.Tensor, s_global: torch.Tensor, qw: torch.Tensor, s_w: torch.Tensor,
                            dX: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                            stream=None) -> torch.Tensor:
    """The data gradient stored as bfloat16."""
    if dX is None:
        dX = torch.empty(d.x_shape, dtype=torch.bfloat16, device=qg.device)
    if workspace is None:
        workspace = _ws(workspace_bytes(OP_CONV_BWD_DATA, d), qg.device)
    rc = lib().daq_conv_bwd_data_int8_bf16(C.byref(d), _ptr(qg), _ptr(s_global), _ptr(qw), _ptr(s_w), _ptr(dX),
                                           _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "daq_conv_bwd_data_int8_bf16")
    return dX


def conv_bwd_filter_int8_bf16(d: ConvDesc, qx_cnhw: torch.Tensor, s_x: torch.Tensor, vq: torch.Tensor, s_chan: torch.Tensor,
                              dW: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                              stream=None) -> torch.Tensor:
    """The filter gradient stored as bfloat16."""
    if dW is None:
        dW = torch.empty(d.w_shape, dtype=torch.bfloat16, device=vq.device)
    if workspace is None:
        workspace = _ws(workspace_bytes(OP_CONV_BWD_FILTER, d), vq.device)
    rc = lib().daq_conv_bwd_filter_int8_bf16(C.byref(d), _ptr(qx_cnhw), _ptr(s_x), _ptr(vq), _ptr(s_chan), _ptr(dW),
                                             _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "daq_conv_bwd_filter_int8_bf16")
    return dW


def conv_bwd_data_int8_chan(d: ConvDesc, vq: torch.Tensor, s_chan: torch.Tensor, qw: torch.Tensor, s_w: torch.Tensor,
                            dX: Optional[torch.Tensor] = None, acc: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Depthwise layers: the data gradient from the per-channel copy (ERR_UNSUPPORTED for any other layer)."""
    if dX is None:
        dX = torch.empty(d.x_shape, dtype=torch.float32, device=vq.device)
    if workspace is None:
        workspace = _ws(workspace_bytes(OP_CONV_BWD_DATA, d), vq.device)
    rc = lib().daq_conv_bwd_data_int8_chan(C.byref(d), _ptr(vq), _ptr(s_chan), _ptr(qw), _ptr(s_w), _ptr(dX), _ptr(acc),
                                           _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "daq_conv_bwd_data_int8_chan")
    return dX


def conv_bwd_int8(d: ConvDesc, qx_cnhw: torch.Tensor, s_x: torch.Tensor, vq: torch.Tensor, s_chan: torch.Tensor,
                  qg: torch.Tensor, s_global: torch.Tensor, qw: torch.Tensor, s_w: torch.Tensor,
                  dW: Optional[torch.Tensor] = None, dX: Optional[torch.Tensor] = None,
                  dW_acc: Optional[torch.Tensor] = None, dX_acc: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None):
    """Both gradients of a layer in one call; returns (dW, dX)."""
    if dW is None:
        dW = torch.empty(d.w_shape, dtype=torch.float32, device=vq.device)
    if dX is None:
        dX = torch.empty(d.x_shape, dtype=torch.float32, device=qg.device)
    if workspace is None:
        workspace = _ws(workspace_bytes(OP_CONV_BWD, d), vq.device)
    rc = lib().daq_conv_bwd_int8(C.byref(d), _ptr(qx_cnhw), _ptr(s_x), _ptr(vq), _ptr(s_chan), _ptr(dW), _ptr(dW_acc),
                                 _ptr(qg), _ptr(s_global), _ptr(qw), _ptr(s_w), _ptr(dX), _ptr(dX_acc),
                                 _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "daq_conv_bwd_int8")
    return dW, dX


def clip_search(d: ConvDesc, dY: torch.Tensor, alpha: float, J: int, want_err=True, stream=None):
    """daq_clip_search: (err [Cout, J] fp64 or None, best_s [Cout] fp32, best_j [Cout] int32)."""
    assert dY.is_cuda and dY.dtype == torch.float32 and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    err = torch.empty((d.Cout, J), dtype=torch.float64, device=dY.device) if want_err else None
    best_s = torch.empty(d.Cout, dtype=torch.float32, device=dY.device)
    best_j = torch.empty(d.Cout, dtype=torch.int32, device=dY.device)
    ws = _ws(workspace_bytes(OP_CLIP_SEARCH, d), dY.device)
    rc = lib().daq_clip_search(C.byref(d), _ptr(dY), alpha, J, _ptr(err), _ptr(best_s), _ptr(best_j), _ptr(ws), ws.numel(),
                               _stream(stream))
    _check(rc, "daq_clip_search")
    return err, best_s, best_j


# ------------------------------------------------------------------------------------------------
# 3-D convolution layers
# ------------------------------------------------------------------------------------------------
def conv3d_carriers(d: Conv3dDesc):
    """(kind, cx, cg): the two 2-D problems whose layouts the int8 tensors of the 3-D layer use; kind 1 = the layer is
    that 2-D problem, 0 = layouts only."""
    cx, cg = ConvDesc(), ConvDesc()
    kind = int(lib().daq_conv3d_carriers(C.byref(d), C.byref(cx), C.byref(cg)))
    if kind < 0:
        raise DaqError(ERR_INVALID_ARG, "daq_conv3d_carriers")
    return kind, cx, cg


def conv3d_fwd_int8(d: Conv3dDesc, X: torch.Tensor, W: torch.Tensor, want_acc=False, stream=None) -> Fwd:
    assert X.is_cuda and X.dtype == torch.float32 and X.is_contiguous() and tuple(X.shape) == d.x_shape
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == d.w_shape
    kind, cx, cg = conv3d_carriers(d)
    dev = X.device
    i8 = dict(dtype=torch.int8, device=dev)
    out = Fwd(qx_nhwc=torch.empty(layout_qx_nhwc(cx).bytes, **i8), qx_cnhw=torch.empty(layout_qx_cnhw(cx).bytes, **i8),
              qw=torch.empty(int(lib().daq_conv3d_qw_bytes(C.byref(d))), **i8), s_x=torch.empty(1, device=dev), s_w=torch.empty(1, device=dev),
              Y=torch.empty(d.y_shape, device=dev), acc=torch.empty(d.y_shape, dtype=torch.int32, device=dev) if want_acc else None,
              workspace=_ws(int(lib().daq_conv3d_workspace_bytes(OP_CONV_FWD, C.byref(d))), dev))
    rc = lib().daq_conv3d_fwd_int8(C.byref(d), _ptr(X), _ptr(W), _ptr(out.qx_nhwc), _ptr(out.qx_cnhw), _ptr(out.qw), _ptr(out.s_x),
                                   _ptr(out.s_w), _ptr(out.Y), _ptr(out.acc), _ptr(out.workspace), out.workspace.numel(), _stream(stream))
    _check(rc, "daq_conv3d_fwd_int8")
    return out


def quantize_grad3d(d: Conv3dDesc, dY: torch.Tensor, s_state: torch.Tensor, k=1.0, A=0.8, lam=0.3, mode=ROUND_NEAREST, seed=0,
                    stream=None) -> QuantGrad:
    assert dY.is_cuda and dY.dtype == torch.float32 and dY.is_contiguous() and tuple(dY.shape) == d.y_shape
    kind, cx, cg = conv3d_carriers(d)
    out = alloc_quantize_grad(cg, dY.device)
    out.workspace = _ws(int(lib().daq_conv3d_workspace_bytes(OP_QUANTIZE_GRAD, C.byref(d))), dY.device)
    rc = lib().daq_quantize_grad3d(C.byref(d), _ptr(dY), _ptr(s_state), k, A, lam, mode, seed, None, _ptr(out.vq), _ptr(out.qg),
                                   _ptr(out.s_chan), _ptr(out.s_global), _ptr(out.cls), _ptr(out.stats), _ptr(out.workspace),
                                   out.workspace.numel(), _stream(stream))
    _check(rc, "daq_quantize_grad3d")
    return out


def conv3d_bwd_data_int8(d: Conv3dDesc, qg, s_global, qw, s_w, acc: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    dX = torch.empty(d.x_shape, dtype=torch.float32, device=qg.device)
    ws = _ws(int(lib().daq_conv3d_workspace_bytes(OP_CONV_BWD_DATA, C.byref(d))), qg.device)
    rc = lib().daq_conv3d_bwd_data_int8(C.byref(d), _ptr(qg), _ptr(s_global), _ptr(qw), _ptr(s_w), _ptr(dX), _ptr(acc), _ptr(ws),
                                        ws.numel(), _stream(stream))
    _check(rc, "daq_conv3d_bwd_data_int8")
    return dX


def conv3d_bwd_filter_int8(d: Conv3dDesc, qx_cnhw, s_x, vq, s_chan, acc: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    dW = torch.empty(d.w_shape, dtype=torch.float32, device=vq.device)
    ws = _ws(int(lib().daq_conv3d_workspace_bytes(OP_CONV_BWD_FILTER, C.byref(d))), vq.device)
    rc = lib().daq_conv3d_bwd_filter_int8(C.byref(d), _ptr(qx_cnhw), _ptr(s_x), _ptr(vq), _ptr(s_chan), _ptr(dW), _ptr(acc), _ptr(ws),
                                          ws.numel(), _stream(stream))
    _check(rc, "daq_conv3d_bwd_filter_int8")
    return dW


# ------------------------------------------------------------------------------------------------
# measurement aid
# ------------------------------------------------------------------------------------------------
def prof_begin():
    _check(lib().daq_prof_begin(), "daq_prof_begin")


def prof_end(max_rows: int = 64):
    rows = (ProfRow * max_rows)()
    n = C.c_int32(0)
    _check(lib().daq_prof_end(rows, max_rows, C.byref(n)), "daq_prof_end")
    return {rows[i].name.decode(): (rows[i].total_ms, rows[i].launches) for i in range(n.value)}


def ceiling_mfma_i8(blocks: int, iters: int, sink: torch.Tensor, stream=None) -> float:
    """Enqueue the register-resident int8 matrix-core loop; returns the int8 operations of the launch."""
    ops = C.c_double(0.0)
    _check(lib().daq_ceiling_mfma_i8(blocks, iters, _ptr(sink), C.byref(ops), _stream(stream)), "daq_ceiling_mfma_i8")
    return ops.value


def ceiling_stream(mode: int, src: Optional[torch.Tensor], dst: Optional[torch.Tensor], nbytes: int, blocks: int,
                   sink: torch.Tensor, stream=None) -> None:
    """Enqueue a streaming read (mode 0), write (1) or copy (2) of ``nbytes``."""
    _check(lib().daq_ceiling_stream(mode, _ptr(src), _ptr(dst), nbytes, blocks, _ptr(sink), _stream(stream)),
           "daq_ceiling_stream")
