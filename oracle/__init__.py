"""CPU oracle (TEST INFRASTRUCTURE) for the int8 quantised-convolution path.

A numpy-facing wrapper over ``q8_oracle.c``.  It imports nothing from the GPU
package and the GPU package imports nothing from here.  Only tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may use it.

Notation follows the paper: ``Q``/``D`` are the quantiser and dequantiser of
Eq. Q / Eq. D, ``plus`` is the + rule, ``conv_i8`` the x rule applied to a
convolution, ``requant`` the real-valued tail of Eq. A' with the fused
element-wise sum and ReLU, ``fold_bn`` the batch-norm folding of the
"Model Optimization" section.
"""
import ctypes as C
from dataclasses import dataclass

import numpy as np

from . import build as _build

_lib = C.CDLL(_build.build())

_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_i8p = np.ctypeslib.ndpointer(np.int8, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")


class _Geom(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h",
        "pad_w", "dil_h", "dil_w", "in_c_stride")]


@dataclass
class ConvGeom:
    """Geometry of one convolution: NHWC activations, KRSC weights."""
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 0
    pad_w: int = 0
    dil_h: int = 1
    dil_w: int = 1
    in_c_stride: int = 0  # 0 -> dense (= C)

    def _c(self):
        ics = self.in_c_stride or self.C
        return _Geom(self.N, self.H, self.W, self.C, self.K, self.R, self.S,
                     self.stride_h, self.stride_w, self.pad_h, self.pad_w,
                     self.dil_h, self.dil_w, ics)

    @property
    def Ho(self):
        return _lib.orc_out_h(C.byref(self._c()))

    @property
    def Wo(self):
        return _lib.orc_out_w(C.byref(self._c()))


_lib.orc_maxabs.restype = C.c_float
_lib.orc_maxabs.argtypes = [_f32p, C.c_size_t]
_lib.orc_qfactor.restype = C.c_float
_lib.orc_qfactor.argtypes = [C.c_float, C.c_int]
_lib.orc_quantize.restype = None
_lib.orc_quantize.argtypes = [_f32p, C.c_size_t, C.c_float, C.c_int, _i32p]
_lib.orc_quantize_bias.restype = None
_lib.orc_quantize_bias.argtypes = [_f32p, C.c_size_t, C.c_float, C.c_float, _i32p]
_lib.orc_dequantize.restype = None
_lib.orc_dequantize.argtypes = [_i8p, C.c_size_t, C.c_float, _f32p]
_lib.orc_plus.restype = None
_lib.orc_plus.argtypes = [_i8p, C.c_float, _i8p, C.c_float, C.c_size_t, C.c_int, _i32p]
_lib.orc_fold_bn.restype = None
_lib.orc_fold_bn.argtypes = [_f32p, C.c_void_p, _f32p, _f32p, _f32p, _f32p, C.c_float,
                             C.c_int, C.c_int, _f32p, _f32p]
_lib.orc_out_h.restype = C.c_int
_lib.orc_out_w.restype = C.c_int
_lib.orc_conv_i8.restype = C.c_int
_lib.orc_conv_i8.argtypes = [C.POINTER(_Geom), _i8p, _i8p, C.c_void_p, _i32p]
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
_lib.orc_conv_u8.restype = C.c_int
_lib.orc_conv_u8.argtypes = [C.POINTER(_Geom), _u8p, _i8p, C.c_void_p, _i32p]
_lib.orc_requant_mixed.restype = None
_lib.orc_requant_mixed.argtypes = [_i32p, C.c_size_t, C.c_int, C.c_float, C.c_void_p, C.c_int,
                                   C.c_int, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_int,
                                   C.c_int, C.c_int]
_lib.orc_dequantize_u8.restype = None
_lib.orc_dequantize_u8.argtypes = [_u8p, C.c_size_t, C.c_float, _f32p]
_lib.orc_requant_scales_pc.restype = None
_lib.orc_requant_scales_pc.argtypes = [C.c_float, _f32p, C.c_int, C.c_float, _f32p]
_lib.orc_requant_pc.restype = None
_lib.orc_requant_pc.argtypes = [_i32p, C.c_size_t, C.c_int, _f32p, C.c_void_p, C.c_int, C.c_int,
                                C.c_float, C.c_int, _i8p, C.c_int, C.c_int]
_lib.orc_quantize_bias_pc.restype = None
_lib.orc_quantize_bias_pc.argtypes = [_f32p, C.c_size_t, C.c_float, _f32p, _i32p]
_lib.orc_requant_scale.restype = C.c_float
_lib.orc_requant_scale.argtypes = [C.c_float] * 3
_lib.orc_residual_scale.restype = C.c_float
_lib.orc_residual_scale.argtypes = [C.c_float] * 2
_lib.orc_real_output.restype = None
_lib.orc_real_output.argtypes = [_i32p, C.c_size_t, C.c_int, C.c_float, C.c_float, C.c_void_p,
                                 C.c_int, C.c_int, C.c_float, C.c_int, _f32p, C.c_int, C.c_int]
_lib.orc_requant.restype = None
_lib.orc_requant.argtypes = [_i32p, C.c_size_t, C.c_int, C.c_float, C.c_void_p, C.c_int,
                             C.c_int, C.c_float, C.c_int, _i8p, C.c_int, C.c_int]
_lib.orc_conv_f32.restype = None
_lib.orc_conv_f32.argtypes = [C.POINTER(_Geom), _f32p, _f32p, C.c_void_p, C.c_void_p,
                              C.c_int, _f32p]
_lib.orc_maxpool_i8.restype = None
_lib.orc_maxpool_i8.argtypes = [_i8p] + [C.c_int] * 10 + [_i8p]
_lib.orc_pool_i8.restype = None
_lib.orc_pool_i8.argtypes = [_i8p] + [C.c_int] * 11 + [C.c_float, _i8p, C.c_int, C.c_int]
_lib.orc_num_threads.restype = C.c_int


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads():
    return int(_lib.orc_num_threads())


def maxabs(r):
    r = _f32(r).ravel()
    return np.float32(_lib.orc_maxabs(r, r.size))


def qfactor(max_abs, p):
    return np.float32(_lib.orc_qfactor(np.float32(max_abs), int(p)))


def Q(r, q, p):
    """Eq. Q for p <= 23; returns int8 for p <= 7, else int32."""
    r = _f32(r)
    z = np.empty(r.shape, np.int32)
    _lib.orc_quantize(r.ravel(), r.size, np.float32(q), int(p), z.reshape(-1))
    return z.astype(np.int8) if p <= 7 else z


def Q_u8(r, q):
    """Eq. Q with p = 8 on a non-negative tensor, as uint8 codes (negative values, which the
    clamp would map below zero, are not representable: the caller guarantees r >= 0)."""
    z = Q(r, q, 8)
    assert z.min(initial=0) >= 0
    return z.astype(np.uint8)


def D_u8(z, q):
    z = np.ascontiguousarray(z, dtype=np.uint8)
    r = np.empty(z.shape, np.float32)
    _lib.orc_dequantize_u8(z.ravel(), z.size, np.float32(q), r.reshape(-1))
    return r


def Q31_bias(b, q_x, q_w):
    b = _f32(b)
    z = np.empty(b.shape, np.int32)
    _lib.orc_quantize_bias(b.ravel(), b.size, np.float32(q_x), np.float32(q_w),
                           z.reshape(-1))
    return z


def D(z, q):
    z = np.ascontiguousarray(z, dtype=np.int8)
    r = np.empty(z.shape, np.float32)
    _lib.orc_dequantize(z.ravel(), z.size, np.float32(q), r.reshape(-1))
    return r


def plus(z1, q1, z2, q2, p=7):
    z1 = np.ascontiguousarray(z1, dtype=np.int8)
    z2 = np.ascontiguousarray(z2, dtype=np.int8)
    assert z1.shape == z2.shape
    z = np.empty(z1.shape, np.int32)
    _lib.orc_plus(z1.ravel(), np.float32(q1), z2.ravel(), np.float32(q2), z1.size,
                  int(p), z.reshape(-1))
    return z, np.float32(max(np.float32(q1), np.float32(q2)))


def fold_bn(W, b, gamma, beta, mu, var, eps=1e-5):
    W = _f32(W)
    K = W.shape[0]
    rsc = W.size // K
    b_c = None if b is None else _f32(b)
    W_out = np.empty_like(W)
    b_out = np.empty(K, np.float32)
    _lib.orc_fold_bn(W.reshape(-1), _ptr(b_c), _f32(gamma), _f32(beta), _f32(mu),
                     _f32(var), np.float32(eps), K, rsc, W_out.reshape(-1), b_out)
    return W_out, b_out


def conv_i8(g, z_x, z_w, z_b=None):
    """Integer accumulators [N,Ho,Wo,K] (int32) of the convolution, bias included."""
    z_x = np.ascontiguousarray(z_x, dtype=np.int8)
    z_w = np.ascontiguousarray(z_w, dtype=np.int8)
    ics = g.in_c_stride or g.C
    assert z_x.size == g.N * g.H * g.W * ics, (z_x.shape, g)
    assert z_w.size == g.K * g.R * g.S * g.C
    zb = None if z_b is None else np.ascontiguousarray(z_b, dtype=np.int32)
    if zb is not None:
        assert zb.size == g.K
    acc = np.empty((g.N, g.Ho, g.Wo, g.K), np.int32)
    gc = g._c()
    rc = _lib.orc_conv_i8(C.byref(gc), z_x.ravel(), z_w.ravel(), _ptr(zb), acc.reshape(-1))
    if rc != 0:
        raise OverflowError("accumulator left the int32 range")
    return acc


def conv_u8(g, z_x, z_w, z_b=None):
    """conv_i8 with unsigned 8-bit activation codes (uint8 array)."""
    assert z_x.dtype == np.uint8
    z_x = np.ascontiguousarray(z_x)
    z_w = np.ascontiguousarray(z_w, dtype=np.int8)
    ics = g.in_c_stride or g.C
    assert z_x.size == g.N * g.H * g.W * ics and z_w.size == g.K * g.R * g.S * g.C
    zb = None if z_b is None else np.ascontiguousarray(z_b, dtype=np.int32)
    acc = np.empty((g.N, g.Ho, g.Wo, g.K), np.int32)
    gc = g._c()
    if _lib.orc_conv_u8(C.byref(gc), z_x.ravel(), z_w.ravel(), _ptr(zb), acc.reshape(-1)) != 0:
        raise OverflowError("accumulator left the int32 range")
    return acc


def requant_mixed(acc, m, relu, z_res=None, m_r=0.0, out_unsigned=False, out=None,
                  out_c_off=0):
    """requant where the residual (by its dtype: uint8 = unsigned codes) and the output
    (``out_unsigned``) may be unsigned p = 8 codes.  ``out``: [..., C_total] of the matching
    dtype, written at channels [out_c_off, out_c_off + K)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    K = acc.shape[-1]
    npix = acc.size // K if K else 0
    dt = np.uint8 if out_unsigned else np.int8
    if out is None:
        out = np.empty(acc.shape, dt)
    assert out.dtype == dt and out.flags.c_contiguous and out_c_off + K <= out.shape[-1]
    zr, res_u, rcs = None, 0, 0
    if z_res is not None:
        assert z_res.dtype in (np.uint8, np.int8)
        zr = np.ascontiguousarray(z_res)
        res_u, rcs = int(zr.dtype == np.uint8), zr.shape[-1]
        assert zr.size == npix * rcs and rcs >= K
    _lib.orc_requant_mixed(acc.reshape(-1), npix, K, np.float32(m), _ptr(zr), res_u, rcs, 0,
                           np.float32(m_r), int(bool(relu)), _ptr(out), int(out_unsigned),
                           out.shape[-1], out_c_off)
    return out


def quantize_weights_pc(W, p=7):
    """Per-output-channel weight quantisation: (z_w int8 like W, q_w fp32 [K])."""
    W = _f32(W)
    K = W.shape[0]
    q_w = np.array([qfactor(maxabs(W[k]), p) for k in range(K)], np.float32)
    z_w = np.stack([Q(W[k], q_w[k], p) for k in range(K)])
    return z_w, q_w


def Q31_bias_pc(b, q_x, q_w):
    b = _f32(b)
    q_w = _f32(q_w)
    assert b.shape == q_w.shape
    z = np.empty(b.shape, np.int32)
    _lib.orc_quantize_bias_pc(b, b.size, np.float32(q_x), q_w, z)
    return z


def requant_scales_pc(q_x, q_w, q_out):
    q_w = _f32(q_w)
    m = np.empty(q_w.shape, np.float32)
    _lib.orc_requant_scales_pc(np.float32(q_x), q_w, q_w.size, np.float32(q_out), m)
    return m


def requant_pc(acc, m, relu, z_res=None, m_r=0.0, out=None, out_c_stride=0, out_c_off=0):
    """requant with one scale per output channel (m: fp32 [K])."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    K = acc.shape[-1]
    m = _f32(m)
    assert m.shape == (K,)
    npix = acc.size // K if K else 0
    if out is None:
        out = np.empty(acc.shape, np.int8)
        out_c_stride, out_c_off = K, 0
    assert out.dtype == np.int8 and out.flags.c_contiguous
    assert out.size >= npix * out_c_stride and out_c_off + K <= out_c_stride
    zr, rcs = None, 0
    if z_res is not None:
        zr = np.ascontiguousarray(z_res, dtype=np.int8)
        rcs = K
        assert zr.size == npix * K
    _lib.orc_requant_pc(acc.reshape(-1), npix, K, m, _ptr(zr), rcs, 0, np.float32(m_r),
                        int(bool(relu)), out.reshape(-1), out_c_stride, out_c_off)
    return out


def requant_scale(q_x, q_w, q_out):
    return np.float32(_lib.orc_requant_scale(np.float32(q_x), np.float32(q_w),
                                             np.float32(q_out)))


def residual_scale(q_res, q_out):
    return np.float32(_lib.orc_residual_scale(np.float32(q_res), np.float32(q_out)))


def requant(acc, m, relu, z_res=None, m_r=0.0, res_c_stride=0, res_c_off=0,
            out=None, out_c_stride=0, out_c_off=0):
    """int32 accumulators [..., K] -> int8, optionally into a channel slice of ``out``."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    K = acc.shape[-1]
    npix = acc.size // K if K else 0
    if out is None:
        out = np.empty(acc.shape, np.int8)
        out_c_stride, out_c_off = K, 0
    assert out.dtype == np.int8 and out.flags.c_contiguous
    assert out.size >= npix * out_c_stride and out_c_off + K <= out_c_stride
    zr = None
    if z_res is not None:
        zr = np.ascontiguousarray(z_res, dtype=np.int8)
        res_c_stride = res_c_stride or K
        assert zr.size >= npix * res_c_stride and res_c_off + K <= res_c_stride
    _lib.orc_requant(acc.reshape(-1), npix, K, np.float32(m), _ptr(zr), res_c_stride,
                     res_c_off, np.float32(m_r), int(bool(relu)), out.reshape(-1),
                     out_c_stride, out_c_off)
    return out


def real_output(acc, q_x, q_w, relu, z_res=None, q_res=0.0, res_c_stride=0, res_c_off=0,
                out=None, out_c_stride=0, out_c_off=0):
    """int32 accumulators [..., K] -> fp32 values (Eq. D at q_x*q_w, fused sum, ReLU; no Q)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    K = acc.shape[-1]
    npix = acc.size // K if K else 0
    if out is None:
        out = np.empty(acc.shape, np.float32)
        out_c_stride, out_c_off = K, 0
    assert out.dtype == np.float32 and out.flags.c_contiguous
    assert out.size >= npix * out_c_stride and out_c_off + K <= out_c_stride
    zr = None
    if z_res is not None:
        zr = np.ascontiguousarray(z_res, dtype=np.int8)
        res_c_stride = res_c_stride or K
        assert zr.size >= npix * res_c_stride and res_c_off + K <= res_c_stride
    _lib.orc_real_output(acc.reshape(-1), npix, K, np.float32(q_x), np.float32(q_w), _ptr(zr),
                         res_c_stride, res_c_off, np.float32(q_res), int(bool(relu)),
                         out.reshape(-1), out_c_stride, out_c_off)
    return out


def conv_f32(g, x, w, b=None, res=None, relu=False):
    x, w = _f32(x), _f32(w)
    b_c = None if b is None else _f32(b)
    r_c = None if res is None else _f32(res)
    y = np.empty((g.N, g.Ho, g.Wo, g.K), np.float32)
    gc = g._c()
    _lib.orc_conv_f32(C.byref(gc), x.ravel(), w.ravel(), _ptr(b_c), _ptr(r_c),
                      int(bool(relu)), y.reshape(-1))
    return y


def maxpool_i8(x, R, S, stride, pad, Ho, Wo):
    x = np.ascontiguousarray(x, dtype=np.int8)
    N, H, W, Cc = x.shape
    y = np.empty((N, Ho, Wo, Cc), np.int8)
    _lib.orc_maxpool_i8(x.ravel(), N, H, W, Cc, R, S, stride, pad, Ho, Wo, y.reshape(-1))
    return y


def pool_i8(x, mode, R, S, stride, pad, Ho, Wo, m=1.0, out=None, out_c_off=0):
    """mode 'max' or 'avg'; writes channels [out_c_off, out_c_off + C) of ``out``."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    N, H, W, Cc = x.shape
    if out is None:
        out = np.zeros((N, Ho, Wo, Cc), np.int8)
    assert out.dtype == np.int8 and out.flags.c_contiguous and out.shape[:3] == (N, Ho, Wo)
    assert out_c_off + Cc <= out.shape[3]
    _lib.orc_pool_i8(x.ravel(), N, H, W, Cc, 0 if mode == "max" else 1, R, S, stride, pad, Ho, Wo,
                     np.float32(m), out.reshape(-1), out.shape[3], out_c_off)
    return out


def conv_layer_i8(g, z_x, q_x, z_w, q_w, z_b, q_out, relu, z_res=None, q_res=None):
    """One quantised layer (Eq. A' + fused sum): returns (z_y int8, acc int32)."""
    acc = conv_i8(g, z_x, z_w, z_b)
    m = requant_scale(q_x, q_w, q_out)
    m_r = residual_scale(q_res, q_out) if z_res is not None else np.float32(0)
    return requant(acc, m, relu, z_res, m_r), acc
