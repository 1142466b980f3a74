"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and
rejects bad arguments before anything is launched (so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
B = pytest.importorskip("paper_1805_08691_amd.binding")


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "q8conv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(q8_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 16
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name


def test_strerror():
    assert B.lib.q8_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -99):
        assert len(B.lib.q8_strerror(code)) > 3


def test_qfactor_and_extents():
    assert B.qfactor(0.0, 7) == 1.0
    assert B.qfactor(127.0, 7) == 1.0
    assert B.ConvDesc(1, 224, 224, 3, 64, 7, 7, 2, 2, 3, 3).Ho == 112
    assert B.ConvDesc(1, 19, 19, 512, 1024, 3, 3, 1, 1, 6, 6, 6, 6).Wo == 19
    assert B.ConvDesc(1, 2, 2, 16, 16, 3, 3).Ho == 0


def test_bad_arguments_are_rejected_on_the_host():
    fake = C.c_void_p(0x1000)      # never dereferenced: every call below fails validation first
    L = B.lib
    assert L.q8_calibrate_maxabs(fake, 10, None, None) == -1
    assert L.q8_calibrate_maxabs(None, 10, fake, None) == -1
    assert L.q8_calibrate_maxabs(C.c_void_p(0x1002), 10, fake, None) == -3
    assert L.q8_calibrate_maxabs(None, 0, fake, None) == 0            # empty tensor: no-op
    assert L.q8_quantize(fake, 10, 0.0, 7, fake, None) == -1          # q <= 0
    assert L.q8_quantize_image(fake, 1, 8, 8, 3, 0.5, 7, fake, 8, 9, 1, 0, None) == -1   # frame too low
    assert L.q8_quantize_image(fake, 1, 8, 8, 5, 0.5, 7, fake, 8, 8, 0, 0, None) == -1   # C > 4
    assert L.q8_quantize_image(fake, 1, 8, 8, 3, 0.5, 7, C.c_void_p(0x1002), 8, 8, 0, 0, None) == -3
    assert L.q8_quantize_image(fake, 0, 8, 8, 3, 0.5, 7, fake, 8, 8, 0, 0, None) == 0    # empty batch
    assert L.q8_quantize(fake, 10, float("nan"), 7, fake, None) == -1
    assert L.q8_quantize(fake, 10, float("inf"), 7, fake, None) == -1
    assert L.q8_quantize(fake, 10, 1.0, 8, fake, None) == -1          # p outside 1..7
    assert L.q8_quantize(fake, 10, 1.0, 0, fake, None) == -1
    assert L.q8_quantize(None, 10, 1.0, 7, fake, None) == -1
    assert L.q8_quantize(None, 0, 1.0, 7, None, None) == 0
    assert L.q8_quantize_pad_channels(fake, 10, 5, 4, 1.0, 7, fake, None) == -1
    assert L.q8_quantize_bias(fake, 4, -1.0, 1.0, fake, None) == -1
    assert L.q8_dequantize(fake, 4, 0.0, fake, None) == -1
    assert L.q8_dequantize(None, 4, 1.0, fake, None) == -1
    assert L.q8_fold_bn(fake, None, fake, fake, fake, fake, 1e-5, -1, 4, fake, fake, None) == -1
    assert L.q8_fold_bn(fake, None, None, fake, fake, fake, 1e-5, 2, 4, fake, fake, None) == -1
    assert L.q8_fold_bn(fake, None, fake, fake, fake, fake, 1e-5, 0, 4, fake, fake, None) == 0

    d = B.ConvDesc(1, 8, 8, 16, 16, 3, 3, pad_h=1, pad_w=1)
    ok = (fake, fake, None, 1.0, 1.0, 1.0, None, 0.0, fake, None, None)
    assert L.q8_conv_int8(None, *ok) == -1
    bad = B.ConvDesc(1, 8, 8, 16, 16, 3, 3, stride_h=0)
    assert L.q8_conv_int8(C.byref(bad), *ok) == -1
    odd = B.ConvDesc(1, 8, 8, 24, 16, 3, 3)          # C neither <= 4 nor a multiple of 16
    assert L.q8_conv_int8(C.byref(odd), *ok) == -2
    assert B.packed_weight_bytes(odd) == 0
    assert L.q8_conv_int8(C.byref(d), fake, fake, None, 0.0, 1.0, 1.0, None, 0.0, fake, None,
                          None) == -1
    assert L.q8_conv_int8(C.byref(d), None, fake, None, 1.0, 1.0, 1.0, None, 0.0, fake, None,
                          None) == -1
    assert L.q8_conv_int8(C.byref(d), C.c_void_p(0x1004), fake, None, 1.0, 1.0, 1.0, None, 0.0,
                          fake, None, None) == -3     # activations not 16-byte aligned
    narrow = B.ConvDesc(1, 8, 8, 16, 16, 3, 3, out_c_stride=8)
    assert L.q8_conv_int8(C.byref(narrow), *ok) == -1  # K does not fit the output stride
    resq = (fake, fake, None, 1.0, 1.0, 1.0, fake, 0.0, fake, None, None)
    assert L.q8_conv_int8(C.byref(d), *resq) == -1     # residual with q_res <= 0
    empty = B.ConvDesc(0, 8, 8, 16, 16, 3, 3)
    assert L.q8_conv_int8(C.byref(empty), None, None, None, 1.0, 1.0, 1.0, None, 0.0, None, None,
                          None) == 0                   # empty batch: nothing to do
    # sizes beyond the kernels' 32-bit offsets are refused on the host, nothing is launched
    big_x = B.ConvDesc(4096, 512, 512, 64, 64, 3, 3, pad_h=1, pad_w=1)        # activations > 2 GiB
    assert L.q8_conv_int8(C.byref(big_x), *ok) == -2
    big_m = B.ConvDesc(40000, 256, 256, 16, 64, 1, 1)                          # N*Ho*Wo > 2^31
    assert L.q8_conv_int8(C.byref(big_m), *ok) == -2
    big_w = B.ConvDesc(1, 8, 8, 16384, 16384, 3, 3, pad_h=1, pad_w=1)          # filters > 2 GiB
    assert L.q8_conv_int8(C.byref(big_w), *ok) == -2
    # layer pairs: what the pair build cannot take is reported, not attempted
    p1 = B.ConvDesc(2, 14, 14, 64, 128, 3, 3, pad_h=1, pad_w=1, relu=1)
    p2_ok = B.ConvDesc(2, 14, 14, 128, 512, 1, 1)
    assert L.q8_conv_pair_supported(C.byref(p1), C.byref(p2_ok)) == 1
    for bad2 in (B.ConvDesc(2, 14, 14, 128, 4096, 1, 1),          # its filters do not fit in LDS
                 B.ConvDesc(2, 14, 14, 128, 192, 1, 1),           # K2 not a multiple of K1
                 B.ConvDesc(2, 14, 14, 128, 512, 3, 3, pad_h=1, pad_w=1),
                 B.ConvDesc(2, 7, 7, 128, 512, 1, 1),             # not the first layer's output
                 B.ConvDesc(2, 14, 14, 128, 512, 1, 1, stride_h=2, stride_w=2)):
        assert L.q8_conv_pair_supported(C.byref(p1), C.byref(bad2)) == 0
    assert L.q8_conv_pair_supported(C.byref(B.ConvDesc(2, 14, 14, 64, 96, 3, 3)), C.byref(p2_ok)) == 0
    pair_args = (fake, fake, None, 1.0, 1.0, 1.0)
    assert L.q8_conv_pair_int8(C.byref(p1), *pair_args, C.byref(B.ConvDesc(2, 14, 14, 128, 4096, 1, 1)),
                               fake, None, 1.0, 1.0, None, 0.0, fake, None) == -2
    assert L.q8_conv_pair_int8(C.byref(p1), *pair_args, C.byref(p2_ok), None, None, 1.0, 1.0, None, 0.0,
                               fake, None) == -1                     # no second filters
    assert L.q8_conv_pair_int8(C.byref(p1), *pair_args, C.byref(p2_ok), fake, None, 1.0, 0.0, None, 0.0,
                               fake, None) == -1                     # q_out <= 0
    # unsigned activation codes
    wide = B.ConvDesc(1, 8, 8, 16, 64, 3, 3, pad_h=1, pad_w=1, relu=1)
    u8 = (fake, fake, fake, fake, 1.0, 1.0, 1.0, None, 0.0, fake, None, None)
    assert L.q8_conv_u8(C.byref(d), 1, 1, 0, *u8) == -2          # K <= 32: not in the extended build
    norelu = B.ConvDesc(1, 8, 8, 16, 64, 3, 3, pad_h=1, pad_w=1, relu=0)
    assert L.q8_conv_u8(C.byref(norelu), 1, 1, 0, *u8) == -1     # unsigned output without ReLU
    assert L.q8_conv_u8(C.byref(wide), 1, 1, 1, *u8) == -1       # unsigned residual, none given
    assert L.q8_conv_u8(C.byref(wide), 1, 1, 0, fake, fake, None, fake, 1.0, 1.0, 1.0, None, 0.0,
                        fake, None, None) == -1                  # unsigned input needs bias_eff
    assert L.q8_conv_u8(C.byref(wide), 1, 1, 0, fake, fake, fake, None, 1.0, 1.0, 1.0, None, 0.0,
                        fake, None, None) == -1                  # padding needs the tap sums
    assert L.q8_u8_prepare(C.byref(wide), None, None, fake, fake, None) == -1
    assert L.q8_u8_prepare(C.byref(B.ConvDesc(1, 8, 8, 3, 64, 3, 3)), fake, None, fake, fake,
                           None) == -2
    assert L.q8_quantize_u8(fake, 4, 0.0, fake, None) == -1
    assert L.q8_dequantize_u8(None, 4, 1.0, fake, None) == -1
    assert L.q8_dequantize_u8(None, 0, 1.0, None, None) == 0
    # per-channel weight factors
    pc = (fake, fake, None, fake, 1.0, None, 0.0, fake, None, None)
    assert L.q8_conv_int8_per_channel(C.byref(wide), fake, fake, None, None, 1.0, None, 0.0, fake,
                                      None, None) == -1          # no scale vector
    assert L.q8_conv_int8_per_channel(C.byref(d), *pc) == -2     # K <= 32: not in the extended build
    assert L.q8_conv_int8_per_channel(C.byref(wide), fake, fake, None, C.c_void_p(0x1004), 1.0,
                                      None, 0.0, fake, None, None) == -3
    # real-valued (fp32) output
    ro = (fake, fake, None, 1.0, 1.0, None, 0.0)
    assert L.q8_conv_int8_real_output(C.byref(d), *ro, None, None) == -1        # no output
    assert L.q8_conv_int8_real_output(C.byref(d), *ro, C.c_void_p(0x1002), None) == -3
    assert L.q8_conv_int8_real_output(C.byref(d), fake, fake, None, 1.0, 0.0, None, 0.0, fake,
                                      None) == -1                              # q_w <= 0
    assert L.q8_conv_int8_real_output(C.byref(d), fake, fake, None, 1.0, 1.0, fake, 0.0, fake,
                                      None) == -1                              # residual, q_res <= 0
    assert L.q8_conv_int8_real_output(C.byref(empty), None, None, None, 1.0, 1.0, None, 0.0, None,
                                      None) == 0
    assert L.q8_probe_mfma_i8(0, 10, fake, None) == -1
    assert L.q8_probe_mfma_i8(4, 10, None, None) == -1
    assert L.q8_quantize_weights_per_channel(fake, 4, 16, 9, fake, fake, None) == -1   # p
    assert L.q8_quantize_weights_per_channel(None, 4, 16, 7, fake, fake, None) == -1
    assert L.q8_quantize_weights_per_channel(None, 0, 16, 7, None, None, None) == 0
    assert L.q8_quantize_bias_per_channel(fake, 4, 0.0, fake, fake, None) == -1
    assert L.q8_requant_scales(1.0, fake, 4, 0.0, fake, None) == -1
    assert B.packed_weight_bytes(d) == 16 * 3 * 3 * 16
    assert B.packed_weight_bytes(B.ConvDesc(1, 8, 8, 3, 64, 7, 7)) == 64 * 7 * 2 * 16
    assert L.q8_maxpool_i8(fake, 1, 8, 8, 4, 3, 3, 2, 3, 4, 4, fake, None) == -1   # pad >= window
