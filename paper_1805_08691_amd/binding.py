"""ctypes binding of libq8conv.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used for
device memory and streams, nothing else), passes raw pointers and sizes through the C
ABI of ``include/q8conv.h`` and raises ``Q8Error`` on a non-zero return code.  There is
no fallback: if the shared library has not been built, importing this module fails.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("Q8CONV_LIB") or os.path.join(_HERE, "libq8conv.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_1805_08691_amd.build` "
        "(there is no CPU fallback)")

lib = C.CDLL(LIB_PATH)

EXPORTS = [
    "q8_strerror", "q8_conv_out_h", "q8_conv_out_w", "q8_calibrate_maxabs", "q8_qfactor",
    "q8_quantize", "q8_quantize_pad_channels", "q8_quantize_image", "q8_quantize_bias", "q8_quantize_u8", "q8_dequantize_u8",
    "q8_u8_prepare", "q8_conv_u8", "q8_quantize_weights_per_channel",
    "q8_quantize_bias_per_channel", "q8_requant_scales", "q8_conv_int8_per_channel", "q8_conv_int8_real_output", "q8_conv_pair_supported", "q8_conv_pair_int8", "q8_dequantize",
    "q8_fold_bn", "q8_packed_weight_bytes", "q8_pack_weights", "q8_conv_int8",
    "q8_conv_dual_supported", "q8_conv_dual_int8", "q8_conv_chain_supported", "q8_conv_chain_plan_bytes", "q8_conv_chain_plan",
    "q8_conv_chain_workspace_bytes", "q8_conv_chain_int8",
    "q8_conv_chain_static_workspace_limit", "q8_conv_chain_int8_static",
    "q8_conv_chain_static_status",
    "q8_conv_variant", "q8_conv_num_variants", "q8_conv_variant_name", "q8_conv_int8_variant", "q8_sum_factor",
    "q8_conv_workspace_bytes", "q8_conv_workspace_bytes_variant",
    "q8_conv_image_f32_supported", "q8_conv_image_f32_int8", "q8_conv_int8_dequantized",
    "q8_probe_mfma_i8",
    "q8_conv_f32_ref", "q8_maxpool_i8", "q8_maxpool_f32", "q8_pool_i8", "q8_pool_f32",
]


class Q8Error(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"q8conv error {code}: {lib.q8_strerror(code).decode()}")


class ConvDesc(C.Structure):
    """Mirror of ``q8_conv_desc``."""
    _fields_ = [(n, C.c_int32) for n in (
        "N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "dil_h",
        "dil_w", "relu", "in_c_stride", "out_c_stride", "out_c_off", "res_c_stride",
        "res_c_off")]

    def __init__(self, N, H, W, C, K, R, S, stride_h=1, stride_w=1, pad_h=0, pad_w=0, dil_h=1,
                 dil_w=1, relu=0, in_c_stride=0, out_c_stride=0, out_c_off=0, res_c_stride=0,
                 res_c_off=0):
        super().__init__(N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                         int(relu), in_c_stride, out_c_stride, out_c_off, res_c_stride,
                         res_c_off)

    @property
    def Ho(self):
        return lib.q8_conv_out_h(C.byref(self))

    @property
    def Wo(self):
        return lib.q8_conv_out_w(C.byref(self))


class ChainLayer(C.Structure):
    """Mirror of ``q8_chain_layer``: one layer of a q8_conv_chain_int8 list."""
    _fields_ = [("d", ConvDesc), ("z_x", C.c_void_p), ("z_w_packed", C.c_void_p),
                ("bias_i32", C.c_void_p), ("q_x", C.c_float), ("q_w", C.c_float),
                ("q_out", C.c_float), ("residual", C.c_void_p), ("q_res", C.c_float),
                ("z_y", C.c_void_p), ("src_layer", C.c_int32), ("res_layer", C.c_int32),
                ("variant", C.c_int32)]


_vp, _sz, _f, _i = C.c_void_p, C.c_size_t, C.c_float, C.c_int
_dp = C.POINTER(ConvDesc)
lib.q8_conv_chain_supported.argtypes = [_dp]
lib.q8_conv_dual_supported.argtypes = [_dp, _dp]
lib.q8_conv_dual_int8.argtypes = ([_dp, _vp, _vp, _vp, _f, _f, _f, _vp, _f, _vp] * 2) + [_vp]
lib.q8_conv_chain_plan_bytes.restype = C.c_size_t
lib.q8_conv_chain_plan_bytes.argtypes = [C.POINTER(ChainLayer), _i]
lib.q8_conv_chain_plan.argtypes = [C.POINTER(ChainLayer), _i, _vp, _sz]
lib.q8_conv_chain_workspace_bytes.restype = C.c_size_t
lib.q8_conv_chain_workspace_bytes.argtypes = [_vp]
lib.q8_conv_chain_int8.argtypes = [_vp, _vp, _vp, _sz, _vp]
lib.q8_conv_chain_static_workspace_limit.restype = C.c_size_t
lib.q8_conv_chain_static_workspace_limit.argtypes = []
lib.q8_conv_chain_int8_static.argtypes = [_vp, _vp, _vp]
lib.q8_conv_chain_static_status.argtypes = [C.POINTER(C.c_int32)]
lib.q8_strerror.restype = C.c_char_p
lib.q8_strerror.argtypes = [_i]
lib.q8_conv_out_h.argtypes = [_dp]
lib.q8_conv_out_w.argtypes = [_dp]
lib.q8_calibrate_maxabs.argtypes = [_vp, _sz, _vp, _vp]
lib.q8_qfactor.restype = _f
lib.q8_qfactor.argtypes = [_f, _i]
lib.q8_quantize.argtypes = [_vp, _sz, _f, _i, _vp, _vp]
lib.q8_quantize_pad_channels.argtypes = [_vp, _sz, _i, _i, _f, _i, _vp, _vp]
lib.q8_quantize_image.argtypes = [_vp, _i, _i, _i, _i, _f, _i, _vp, _i, _i, _i, _i, _vp]
lib.q8_quantize_bias.argtypes = [_vp, _sz, _f, _f, _vp, _vp]
lib.q8_dequantize.argtypes = [_vp, _sz, _f, _vp, _vp]
lib.q8_fold_bn.argtypes = [_vp] * 6 + [_f, _i, _i, _vp, _vp, _vp]
lib.q8_packed_weight_bytes.restype = _sz
lib.q8_packed_weight_bytes.argtypes = [_dp]
lib.q8_pack_weights.argtypes = [_dp, _vp, _vp, _vp]
lib.q8_conv_int8.argtypes = [_dp, _vp, _vp, _vp, _f, _f, _f, _vp, _f, _vp, _vp, _vp, C.c_size_t, _vp]
lib.q8_conv_workspace_bytes.argtypes = [_dp]
lib.q8_conv_workspace_bytes.restype = C.c_size_t
lib.q8_conv_workspace_bytes_variant.argtypes = [_dp, _i, _i]
lib.q8_conv_workspace_bytes_variant.restype = C.c_size_t
lib.q8_conv_u8.argtypes = [_dp, _i, _i, _i, _vp, _vp, _vp, _vp, _f, _f, _f, _vp, _f, _vp, _vp, _vp]
lib.q8_u8_prepare.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp]
lib.q8_quantize_weights_per_channel.argtypes = [_vp, _i, _sz, _i, _vp, _vp, _vp]
lib.q8_quantize_bias_per_channel.argtypes = [_vp, _i, _f, _vp, _vp, _vp]
lib.q8_requant_scales.argtypes = [_f, _vp, _i, _f, _vp, _vp]
lib.q8_conv_int8_per_channel.argtypes = [_dp, _vp, _vp, _vp, _vp, _f, _vp, _f, _vp, _vp, _vp]
lib.q8_conv_int8_real_output.argtypes = [_dp, _vp, _vp, _vp, _f, _f, _vp, _f, _vp, _vp]
lib.q8_conv_pair_supported.argtypes = [_dp, _dp]
lib.q8_conv_pair_int8.argtypes = [_dp, _vp, _vp, _vp, _f, _f, _f, _dp, _vp, _vp, _f, _f, _vp, _f, _vp, _vp]
lib.q8_quantize_u8.argtypes = [_vp, _sz, _f, _vp, _vp]
lib.q8_dequantize_u8.argtypes = [_vp, _sz, _f, _vp, _vp]
lib.q8_conv_variant.restype = C.c_char_p
lib.q8_conv_variant.argtypes = [_dp]
lib.q8_conv_num_variants.argtypes = []
lib.q8_conv_variant_name.restype = C.c_char_p
lib.q8_conv_variant_name.argtypes = [_i]
lib.q8_conv_int8_variant.argtypes = [_dp, _vp, _vp, _vp, _f, _f, _f, _vp, _f, _vp, _vp, _i, _i, _vp,
                                     C.c_size_t, _vp]
lib.q8_conv_int8_dequantized.argtypes = [_dp, _vp, _vp, _vp, _f, _f, _f, _vp, _f, _vp, _vp, _vp]
lib.q8_conv_image_f32_supported.argtypes = [_dp, _i, _i, _i, _i, _i, _i]
lib.q8_conv_image_f32_int8.argtypes = [_dp, _vp, _i, _i, _i, _i, _i, _f, _i, _vp, _vp, _f, _f, _i, _vp, _vp]
lib.q8_sum_factor.restype = _f
lib.q8_sum_factor.argtypes = [_f, _f]
lib.q8_probe_mfma_i8.argtypes = [_i, _i, _vp, _vp]
lib.q8_conv_f32_ref.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.q8_maxpool_i8.argtypes = [_vp] + [_i] * 10 + [_vp, _vp]
lib.q8_maxpool_f32.argtypes = [_vp] + [_i] * 10 + [_vp, _vp]


lib.q8_pool_i8.argtypes = [_vp] + [_i] * 11 + [_f, _f, _vp, _i, _i, _vp]
lib.q8_pool_f32.argtypes = [_vp] + [_i] * 11 + [_vp, _i, _i, _vp]


def _check(code):
    if code != 0:
        raise Q8Error(code)


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors, contiguous"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def calibrate_maxabs(x, maxabs):
    """maxabs[0] = max(maxabs[0], max|x|); ``maxabs`` is a 1-element fp32 device tensor."""
    _check(lib.q8_calibrate_maxabs(_ptr(x, torch.float32), x.numel(),
                                   _ptr(maxabs, torch.float32), _stream()))


def qfactor(max_abs, p):
    return lib.q8_qfactor(float(max_abs), int(p))


def quantize(r, q, p, out=None):
    z = out if out is not None else torch.empty(r.shape, dtype=torch.int8, device=r.device)
    _check(lib.q8_quantize(_ptr(r, torch.float32), r.numel(), q, p, _ptr(z, torch.int8),
                           _stream()))
    return z


def quantize_pad_channels(r, c_pad, q, p, out=None):
    """NHWC fp32 [..., C] -> int8 [..., c_pad] with zero channels appended."""
    Cc = r.shape[-1]
    npix = r.numel() // Cc
    z = out if out is not None else torch.empty(r.shape[:-1] + (c_pad,), dtype=torch.int8,
                                                device=r.device)
    _check(lib.q8_quantize_pad_channels(_ptr(r, torch.float32), npix, Cc, c_pad, q, p,
                                        _ptr(z, torch.int8), _stream()))
    return z


def quantize_image(r, q, p, out, top, left):
    """r: [N,H,W,C<=4] fp32; out: zero-framed [N,Hs,Ws,4] int8, interior written at (top, left)."""
    N, H, W, Cc = r.shape
    assert out.shape[0] == N and out.shape[3] == 4
    _check(lib.q8_quantize_image(_ptr(r, torch.float32), N, H, W, Cc, q, p, _ptr(out, torch.int8),
                                 out.shape[1], out.shape[2], top, left, _stream()))
    return out


def quantize_bias(b, q_x, q_w, out=None):
    z = out if out is not None else torch.empty(b.shape, dtype=torch.int32, device=b.device)
    _check(lib.q8_quantize_bias(_ptr(b, torch.float32), b.numel(), q_x, q_w,
                                _ptr(z, torch.int32), _stream()))
    return z


def dequantize(z, q, out=None):
    r = out if out is not None else torch.empty(z.shape, dtype=torch.float32, device=z.device)
    _check(lib.q8_dequantize(_ptr(z, torch.int8), z.numel(), q, _ptr(r, torch.float32),
                             _stream()))
    return r


def fold_bn(W, b, gamma, beta, mu, var, eps=1e-5):
    K = W.shape[0]
    rsc = W.numel() // K if K else 0
    W_out = torch.empty_like(W)
    b_out = torch.empty(K, dtype=torch.float32, device=W.device)
    _check(lib.q8_fold_bn(_ptr(W, torch.float32), _ptr(b, torch.float32),
                          _ptr(gamma, torch.float32), _ptr(beta, torch.float32),
                          _ptr(mu, torch.float32), _ptr(var, torch.float32), eps, K, rsc,
                          _ptr(W_out), _ptr(b_out), _stream()))
    return W_out, b_out


def packed_weight_bytes(desc):
    return lib.q8_packed_weight_bytes(C.byref(desc))


def pack_weights(desc, z_w):
    nbytes = packed_weight_bytes(desc)
    if nbytes == 0:
        raise Q8Error(-2)
    packed = torch.empty(nbytes, dtype=torch.int8, device=z_w.device)
    _check(lib.q8_pack_weights(C.byref(desc), _ptr(z_w, torch.int8), _ptr(packed), _stream()))
    return packed


def conv_workspace_bytes(desc, variant=-1, n_split=0):
    """Workspace with which the library splits this layer's reduction (0: it would not)."""
    if variant >= 0:
        return lib.q8_conv_workspace_bytes_variant(C.byref(desc), int(variant), int(n_split))
    return lib.q8_conv_workspace_bytes(C.byref(desc))


def conv_int8(desc, z_x, z_w_packed, bias_i32, q_x, q_w, q_out, residual=None, q_res=0.0,
              out=None, acc_dump=None, variant=-1, workspace=None, n_split=0):
    """``workspace``: a zeroed uint8 device tensor the library may split the reduction with.
    ``variant`` >= 0 (tests, tuning): that tile variant of the main kernel, ``n_split``
    workgroups per tile where it is a split-reduction variant."""
    if out is None:
        ocs = desc.out_c_stride or desc.K
        out = torch.empty((desc.N, desc.Ho, desc.Wo, ocs), dtype=torch.int8, device=z_x.device)
    args = (C.byref(desc), _ptr(z_x, torch.int8), _ptr(z_w_packed, torch.int8),
            _ptr(bias_i32, torch.int32), q_x, q_w, q_out, _ptr(residual, torch.int8), q_res,
            _ptr(out, torch.int8), _ptr(acc_dump, torch.int32))
    ws = (_ptr(workspace, torch.uint8), 0 if workspace is None else workspace.numel())
    if variant >= 0:
        _check(lib.q8_conv_int8_variant(*args, int(variant), int(n_split), *ws, _stream()))
    else:
        _check(lib.q8_conv_int8(*args, *ws, _stream()))
    return out


def conv_int8_dequantized(desc, z_x, z_w_packed, bias_i32, q_x, q_w, q_out, residual=None, q_res=0.0,
                          out=None, out_f32=None):
    """conv_int8 that also writes Eq. D of its output codes: -> (codes, fp32)."""
    shape = (desc.N, desc.Ho, desc.Wo, desc.out_c_stride or desc.K)
    if out is None:
        out = torch.empty(shape, dtype=torch.int8, device=z_x.device)
    if out_f32 is None:
        out_f32 = torch.empty(shape, dtype=torch.float32, device=z_x.device)
    _check(lib.q8_conv_int8_dequantized(C.byref(desc), _ptr(z_x, torch.int8),
                                        _ptr(z_w_packed, torch.int8), _ptr(bias_i32, torch.int32),
                                        q_x, q_w, q_out, _ptr(residual, torch.int8), q_res,
                                        _ptr(out, torch.int8), _ptr(out_f32, torch.float32),
                                        _stream()))
    return out, out_f32


def conv_image_f32_supported(desc, H, W, Cc, top, left, pool=0):
    return bool(lib.q8_conv_image_f32_supported(C.byref(desc), H, W, Cc, top, left, int(pool)))


def conv_image_f32(desc, r, top, left, q_x, p, z_w_packed, bias_i32, q_w, q_out, pool=0, out=None):
    """Eq. Q on the fp32 image r [N,H,W,C<=4], the layer ``desc`` (given over the zero frame
    that holds r at (top, left)) and, with ``pool``, the 3x3/2 max-pool, as one launch."""
    N, H, W, Cc = r.shape
    assert N == desc.N
    if out is None:
        Ho, Wo = ((desc.Ho - 1) // 2 + 1, (desc.Wo - 1) // 2 + 1) if pool else (desc.Ho, desc.Wo)
        out = torch.empty((N, Ho, Wo, desc.out_c_stride or desc.K), dtype=torch.int8, device=r.device)
    _check(lib.q8_conv_image_f32_int8(C.byref(desc), _ptr(r, torch.float32), H, W, Cc, top, left,
                                      q_x, p, _ptr(z_w_packed, torch.int8),
                                      _ptr(bias_i32, torch.int32), q_w, q_out, int(pool),
                                      _ptr(out, torch.int8), _stream()))
    return out


def quantize_u8(r, q, out=None):
    """Eq. Q, p = 8, on a non-negative tensor; codes stored as code - 128."""
    z = torch.empty(r.shape, dtype=torch.int8, device=r.device) if out is None else out
    _check(lib.q8_quantize_u8(_ptr(r, torch.float32), r.numel(), q, _ptr(z, torch.int8), _stream()))
    return z


def dequantize_u8(z, q, out=None):
    r = torch.empty(z.shape, dtype=torch.float32, device=z.device) if out is None else out
    _check(lib.q8_dequantize_u8(_ptr(z, torch.int8), z.numel(), q, _ptr(r, torch.float32),
                                _stream()))
    return r


def u8_prepare(desc, z_w, bias_i32=None):
    """-> (start values int32 [((R+1)*(S+1))**2, K], one row per rectangle of taps inside the
    image, bias_eff int32 [K]) for a layer reading unsigned codes."""
    taps = torch.empty((((desc.R + 1) * (desc.S + 1)) ** 2, desc.K), dtype=torch.int32,
                       device=z_w.device)
    beff = torch.empty(desc.K, dtype=torch.int32, device=z_w.device)
    _check(lib.q8_u8_prepare(C.byref(desc), _ptr(z_w, torch.int8), _ptr(bias_i32, torch.int32),
                             _ptr(taps, torch.int32), _ptr(beff, torch.int32), _stream()))
    return taps, beff


def conv_u8(desc, in_u8, out_u8, res_u8, z_x, z_w_packed, bias, tap_sums, q_x, q_w, q_out,
            residual=None, q_res=0.0, out=None, acc_dump=None):
    if out is None:
        ocs = desc.out_c_stride or desc.K
        out = torch.empty((desc.N, desc.Ho, desc.Wo, ocs), dtype=torch.int8, device=z_x.device)
    _check(lib.q8_conv_u8(C.byref(desc), int(in_u8), int(out_u8), int(res_u8),
                          _ptr(z_x, torch.int8), _ptr(z_w_packed, torch.int8),
                          _ptr(bias, torch.int32), _ptr(tap_sums, torch.int32), q_x, q_w, q_out,
                          _ptr(residual, torch.int8), q_res, _ptr(out, torch.int8),
                          _ptr(acc_dump, torch.int32), _stream()))
    return out


def quantize_weights_per_channel(W, p=7):
    """W fp32 [K, ...] -> (q_w fp32 [K], z_w int8 like W), one factor per output channel."""
    K = W.shape[0]
    q_w = torch.empty(K, dtype=torch.float32, device=W.device)
    z_w = torch.empty(W.shape, dtype=torch.int8, device=W.device)
    _check(lib.q8_quantize_weights_per_channel(_ptr(W, torch.float32), K, W.numel() // max(K, 1),
                                               p, _ptr(q_w, torch.float32), _ptr(z_w, torch.int8),
                                               _stream()))
    return q_w, z_w


def quantize_bias_per_channel(b, q_x, q_w):
    z = torch.empty(b.shape, dtype=torch.int32, device=b.device)
    _check(lib.q8_quantize_bias_per_channel(_ptr(b, torch.float32), b.numel(), q_x,
                                            _ptr(q_w, torch.float32), _ptr(z, torch.int32),
                                            _stream()))
    return z


def requant_scales(q_x, q_w, q_out):
    m = torch.empty(q_w.shape, dtype=torch.float32, device=q_w.device)
    _check(lib.q8_requant_scales(q_x, _ptr(q_w, torch.float32), q_w.numel(), q_out,
                                 _ptr(m, torch.float32), _stream()))
    return m


def conv_int8_per_channel(desc, z_x, z_w_packed, bias_i32, m, q_out, residual=None, q_res=0.0,
                          out=None, acc_dump=None):
    if out is None:
        ocs = desc.out_c_stride or desc.K
        out = torch.empty((desc.N, desc.Ho, desc.Wo, ocs), dtype=torch.int8, device=z_x.device)
    _check(lib.q8_conv_int8_per_channel(C.byref(desc), _ptr(z_x, torch.int8),
                                        _ptr(z_w_packed, torch.int8), _ptr(bias_i32, torch.int32),
                                        _ptr(m, torch.float32), q_out, _ptr(residual, torch.int8),
                                        q_res, _ptr(out, torch.int8), _ptr(acc_dump, torch.int32),
                                        _stream()))
    return out


def conv_int8_real_output(desc, z_x, w_packed, bias, q_x, q_w, residual=None, q_res=0.0, out=None):
    """The layer's real-valued output (fp32), no requantisation."""
    if out is None:
        out = torch.empty((desc.N, desc.Ho, desc.Wo, desc.out_c_stride or desc.K),
                          dtype=torch.float32, device=z_x.device)
    _check(lib.q8_conv_int8_real_output(C.byref(desc), _ptr(z_x, torch.int8), _ptr(w_packed),
                                        _ptr(bias, torch.int32), q_x, q_w,
                                        _ptr(residual, torch.int8), q_res,
                                        _ptr(out, torch.float32), _stream()))
    return out


def conv_pair_supported(d1, d2):
    return bool(lib.q8_conv_pair_supported(C.byref(d1), C.byref(d2)))


def conv_pair_int8(d1, z_x, w1_packed, bias1, q_x, q_w1, q_mid, d2, w2_packed, bias2, q_w2, q_out,
                   residual=None, q_res=0.0, out=None):
    """A convolution and the 1x1 layer behind it in one launch (the intermediate stays on chip)."""
    if out is None:
        out = torch.empty((d2.N, d2.Ho, d2.Wo, d2.out_c_stride or d2.K), dtype=torch.int8,
                          device=z_x.device)
    _check(lib.q8_conv_pair_int8(C.byref(d1), _ptr(z_x, torch.int8), _ptr(w1_packed),
                                 _ptr(bias1, torch.int32), q_x, q_w1, q_mid, C.byref(d2),
                                 _ptr(w2_packed), _ptr(bias2, torch.int32), q_w2, q_out,
                                 _ptr(residual, torch.int8), q_res, _ptr(out, torch.int8),
                                 _stream()))
    return out


def conv_dual_supported(d1, d2):
    return bool(lib.q8_conv_dual_supported(C.byref(d1), C.byref(d2)))


def conv_dual_int8(a, b):
    """Two independent layers in one launch; ``a`` and ``b`` are tuples (desc, z_x, w_packed,
    bias, q_x, q_w, q_out, residual, q_res, out)."""
    args = []
    for (d, x, w, bias, q_x, q_w, q_out, res, q_res, out) in (a, b):
        args += [C.byref(d), _ptr(x, torch.int8), _ptr(w, torch.int8), _ptr(bias, torch.int32), q_x,
                 q_w, q_out, _ptr(res, torch.int8), q_res, _ptr(out, torch.int8)]
    _check(lib.q8_conv_dual_int8(*args, _stream()))


def conv_chain_supported(desc):
    return bool(lib.q8_conv_chain_supported(C.byref(desc)))


class ConvChain:
    """A planned q8_conv_chain_int8 launch.  ``layers``: list of dicts with the arguments of
    conv_int8 (desc, z_x, w, bias, q_x, q_w, q_out, residual, q_res, out) plus src_layer,
    res_layer (index in the list, or -1) and optionally variant.  Holds the host plan, its
    device copy and the workspace; the tensors named in the plan must stay alive."""

    def __init__(self, layers, device):
        n = len(layers)
        arr = (ChainLayer * n)()
        self.keep = []
        for i, L in enumerate(layers):
            a = arr[i]
            a.d = L["desc"]
            a.z_x = _ptr(L["z_x"], torch.int8)
            a.z_w_packed = _ptr(L["w"], torch.int8)
            a.bias_i32 = _ptr(L["bias"], torch.int32)
            a.q_x, a.q_w, a.q_out = L["q_x"], L["q_w"], L["q_out"]
            a.residual = _ptr(L.get("residual"), torch.int8)
            a.q_res = L.get("q_res", 0.0)
            a.z_y = _ptr(L["out"], torch.int8)
            a.src_layer, a.res_layer = L["src_layer"], L["res_layer"]
            a.variant = L.get("variant", -1)
            self.keep.append((L["z_x"], L["w"], L["bias"], L.get("residual"), L["out"]))
        nbytes = lib.q8_conv_chain_plan_bytes(arr, n)
        if nbytes == 0:
            raise Q8Error(-2)
        self.plan_host = C.create_string_buffer(nbytes)
        _check(lib.q8_conv_chain_plan(arr, n, self.plan_host, nbytes))
        host = torch.frombuffer(self.plan_host, dtype=torch.uint8, count=nbytes)
        self.plan_dev = host.to(device)
        ws_bytes = lib.q8_conv_chain_workspace_bytes(self.plan_host)
        self.ws = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=device)

    def run(self):
        _check(lib.q8_conv_chain_int8(self.plan_host, self.plan_dev.data_ptr(),
                                      self.ws.data_ptr(), self.ws.numel() * 4, _stream()))

    def status(self):
        """Word 0 of the workspace after a synchronisation: 0 = every tile found its inputs."""
        return int(self.ws[0].item())

    def run_static(self):
        """The same launch on the library's own fixed workspace (allocates nothing)."""
        _check(lib.q8_conv_chain_int8_static(self.plan_host, self.plan_dev.data_ptr(), _stream()))

    @staticmethod
    def static_status():
        v = C.c_int32(-1)
        _check(lib.q8_conv_chain_static_status(C.byref(v)))
        return v.value


def conv_variant(desc):
    return lib.q8_conv_variant(C.byref(desc)).decode()


def conv_num_variants():
    return lib.q8_conv_num_variants()


def sum_factor(q1, q2):
    """Eq. +: the factor of a sum of two quantised tensors."""
    return lib.q8_sum_factor(float(q1), float(q2))


def probe_mfma_i8(blocks, iters, sink):
    """Launch the register-resident int8 MFMA loop; returns the int8 ops it performs."""
    _check(lib.q8_probe_mfma_i8(int(blocks), int(iters), _ptr(sink, torch.int32), _stream()))
    return blocks * 4 * 4 * iters * 65536


def conv_f32_ref(desc, x, w, b=None, res=None, out=None):
    if out is None:
        out = torch.empty((desc.N, desc.Ho, desc.Wo, desc.K), dtype=torch.float32,
                          device=x.device)
    _check(lib.q8_conv_f32_ref(C.byref(desc), _ptr(x, torch.float32), _ptr(w, torch.float32),
                               _ptr(b, torch.float32), _ptr(res, torch.float32),
                               _ptr(out, torch.float32), _stream()))
    return out


def _pool(fn, dtype, x, R, S, stride, pad, Ho, Wo):
    N, H, W, Cc = x.shape
    y = torch.empty((N, Ho, Wo, Cc), dtype=dtype, device=x.device)
    _check(fn(_ptr(x, dtype), N, H, W, Cc, R, S, stride, pad, Ho, Wo, _ptr(y), _stream()))
    return y


def maxpool_i8(x, R, S, stride, pad, Ho, Wo):
    return _pool(lib.q8_maxpool_i8, torch.int8, x, R, S, stride, pad, Ho, Wo)


def maxpool_f32(x, R, S, stride, pad, Ho, Wo):
    return _pool(lib.q8_maxpool_f32, torch.float32, x, R, S, stride, pad, Ho, Wo)


def pool_i8(x, mode, R, S, stride, pad, Ho, Wo, q_in=1.0, q_out=1.0, out=None, out_c_off=0):
    """mode 'max' or 'avg'; writes channels [out_c_off, out_c_off + C) of ``out``, rescaled from
    factor ``q_in`` to ``q_out``."""
    N, H, W, Cc = x.shape
    if out is None:
        out = torch.zeros((N, Ho, Wo, Cc), dtype=torch.int8, device=x.device)
    _check(lib.q8_pool_i8(_ptr(x, torch.int8), N, H, W, Cc, 0 if mode == "max" else 1, R, S, stride,
                          pad, Ho, Wo, q_in, q_out, _ptr(out, torch.int8), out.shape[3], out_c_off,
                          _stream()))
    return out


def pool_f32(x, mode, R, S, stride, pad, Ho, Wo, out=None, out_c_off=0):
    N, H, W, Cc = x.shape
    if out is None:
        out = torch.zeros((N, Ho, Wo, Cc), dtype=torch.float32, device=x.device)
    _check(lib.q8_pool_f32(_ptr(x, torch.float32), N, H, W, Cc, 0 if mode == "max" else 1, R, S,
                           stride, pad, Ho, Wo, _ptr(out, torch.float32), out.shape[3], out_c_off,
                           _stream()))
    return out
