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
    ok = (fake, fake, None, 1.0, 1.0, 1.0, None, 0.0, fake, None, None, 0, None)   # no workspace
    assert L.q8_conv_int8(None, *ok) == -1
    bad = B.ConvDesc(1, 8, 8, 16, 16, 3, 3, stride_h=0)
    assert L.q8_conv_int8(C.byref(bad), *ok) == -1
    odd = B.ConvDesc(1, 8, 8, 24, 16, 3, 3)          # C neither <= 4 nor a multiple of 16
    assert L.q8_conv_int8(C.byref(odd), *ok) == -2
    assert B.packed_weight_bytes(odd) == 0
    assert L.q8_conv_int8(C.byref(d), fake, fake, None, 0.0, 1.0, 1.0, None, 0.0, fake, None,
                          None, 0, None) == -1
    assert L.q8_conv_int8(C.byref(d), None, fake, None, 1.0, 1.0, 1.0, None, 0.0, fake, None,
                          None, 0, None) == -1
    assert L.q8_conv_int8(C.byref(d), C.c_void_p(0x1004), fake, None, 1.0, 1.0, 1.0, None, 0.0,
                          fake, None, None, 0, None) == -3     # activations not 16-byte aligned
    narrow = B.ConvDesc(1, 8, 8, 16, 16, 3, 3, out_c_stride=8)
    assert L.q8_conv_int8(C.byref(narrow), *ok) == -1  # K does not fit the output stride
    resq = (fake, fake, None, 1.0, 1.0, 1.0, fake, 0.0, fake, None, None, 0, None)
    assert L.q8_conv_int8(C.byref(d), *resq) == -1     # residual with q_res <= 0
    empty = B.ConvDesc(0, 8, 8, 16, 16, 3, 3)
    assert L.q8_conv_int8(C.byref(empty), None, None, None, 1.0, 1.0, 1.0, None, 0.0, None, None,
                          None, 0, None) == 0          # empty batch: nothing to do
    # split reduction: the workspace is checked on the host
    deep = B.ConvDesc(2, 7, 7, 512, 512, 3, 3, pad_h=1, pad_w=1)
    names = [L.q8_conv_variant_name(v).decode() for v in range(L.q8_conv_num_variants())]
    sv = next(v for v, nm in enumerate(names) if "split" in nm)
    need = L.q8_conv_workspace_bytes_variant(C.byref(deep), sv, 4)
    assert need > 4 * 98 * 49 // 128 * 4            # counters plus four partial tiles per tile
    assert L.q8_conv_workspace_bytes_variant(C.byref(deep), sv, 1) == 0     # nothing to share
    assert L.q8_conv_workspace_bytes_variant(C.byref(deep), 0, 4) == 0      # not a split build
    assert L.q8_conv_workspace_bytes_variant(C.byref(odd), sv, 4) == 0
    assert L.q8_conv_workspace_bytes(C.byref(deep)) <= need
    sp = (fake, fake, None, 1.0, 1.0, 1.0, None, 0.0, fake, None, sv, 4)
    assert L.q8_conv_int8_variant(C.byref(deep), *sp, None, 0, None) == -1             # none given
    assert L.q8_conv_int8_variant(C.byref(deep), *sp, C.c_void_p(0x1010), need, None) == -3
    assert L.q8_conv_int8_variant(C.byref(deep), *sp, fake, need - 1, None) == -5      # too small
    assert L.q8_conv_int8_variant(C.byref(deep), *sp[:-1], 65, fake, need, None) == -1 # factor
    assert L.q8_conv_int8_variant(C.byref(deep), *sp[:-2], len(names), 2, fake, need, None) == -1
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


# ------------------------------------------------------------------ layer lists (host side)
def _chain_layers(n_img=16, bad=None):
    """A bottleneck block (1x1 256->64, 3x3 64->64, 1x1 64->256 + residual) as a layer list on
    made-up, distinct, aligned device addresses (nothing is dereferenced on the host)."""
    base = 0x7F0000000000
    t = {"x": base, "a": base + (1 << 28), "b": base + (2 << 28), "y": base + (3 << 28)}
    geo = [(256, 64, 1, "x", "a", None), (64, 64, 3, "a", "b", None), (64, 256, 1, "b", "y", "x")]
    arr = (B.ChainLayer * 3)()
    for i, (Cc, K, R, src, dst, res) in enumerate(geo):
        a = arr[i]
        a.d = B.ConvDesc(n_img, 28, 28, Cc, K, R, R, 1, 1, R // 2, R // 2, relu=1)
        a.z_x, a.z_y = t[src], t[dst]
        a.z_w_packed, a.bias_i32 = 0x100000 + i * 0x100000, 0x10000 + i * 0x1000
        a.q_x = a.q_w = a.q_out = a.q_res = 0.5
        a.residual = t[res] if res else None
        a.src_layer = i - 1 if i else -1
        a.res_layer = -1
        a.variant = -1
    if bad:
        bad(arr)
    return arr


def test_fused_head_and_dequantized_output_host_checks():
    """q8_conv_image_f32_supported and the argument checks of q8_conv_image_f32_int8 /
    q8_conv_int8_dequantized run on the host: nothing is launched here."""
    L = B.lib
    fake = C.c_void_p(0x1000)
    # ResNet-50's first layer over its zero frame, with and without the max-pool
    d = B.ConvDesc(32, 230, 230, 3, 64, 7, 7, 2, 2, 0, 0, 1, 1, relu=1, in_c_stride=4)
    assert B.conv_image_f32_supported(d, 224, 224, 3, 3, 3, 0)
    assert B.conv_image_f32_supported(d, 224, 224, 3, 3, 3, 1)
    assert not B.conv_image_f32_supported(d, 228, 224, 3, 3, 3, 1)      # does not fit the frame
    assert not B.conv_image_f32_supported(d, 224, 224, 4, 3, 3, 1)      # C != d.C
    # outside the family: 3 filter columns; rows of more than 128 output pixels; K > 64;
    # the pool needs a vertical stride of 2
    assert not B.conv_image_f32_supported(
        B.ConvDesc(1, 301, 301, 3, 32, 3, 3, 2, 2, 0, 0, 1, 1, in_c_stride=4), 299, 299, 3, 1, 1, 0)
    assert not B.conv_image_f32_supported(
        B.ConvDesc(1, 200, 240, 3, 64, 7, 7, 1, 1, 0, 0, 1, 1, in_c_stride=4), 194, 234, 3, 3, 3, 0)
    assert not B.conv_image_f32_supported(
        B.ConvDesc(1, 70, 70, 3, 96, 7, 7, 2, 2, 0, 0, 1, 1, in_c_stride=4), 64, 64, 3, 3, 3, 0)
    d1 = B.ConvDesc(1, 70, 70, 3, 64, 7, 7, 1, 2, 0, 0, 1, 1, in_c_stride=4)
    assert B.conv_image_f32_supported(d1, 64, 64, 3, 3, 3, 0)
    assert not B.conv_image_f32_supported(d1, 64, 64, 3, 3, 3, 1)
    args = lambda dd, r, H, W, Cc, top, left, q, p, pool, y: L.q8_conv_image_f32_int8(
        C.byref(dd), r, H, W, Cc, top, left, q, p, fake, None, 0.01, 0.5, pool, y, None)
    assert args(d, fake, 224, 224, 3, 3, 3, 0.02, 7, 2, fake) == -1       # pool flag
    assert args(d, fake, 224, 224, 3, 3, 3, 0.02, 8, 1, fake) == -1       # p out of range
    assert args(d, fake, 230, 224, 3, 3, 3, 0.02, 7, 1, fake) == -1       # image beyond the frame
    assert args(d, None, 224, 224, 3, 3, 3, 0.02, 7, 1, fake) == -1       # no image
    assert args(d, C.c_void_p(0x1002), 224, 224, 3, 3, 3, 0.02, 7, 1, fake) == -3   # misaligned
    assert args(d, fake, 224, 224, 3, 3, 3, -1.0, 7, 1, fake) == -1       # factor
    d3 = B.ConvDesc(1, 30, 30, 3, 64, 3, 3, 1, 1, 0, 0, 1, 1, in_c_stride=4)
    assert args(d3, fake, 28, 28, 3, 1, 1, 0.02, 7, 0, fake) == -2        # not in the family
    dd = B.ConvDesc(2, 7, 7, 512, 2048, 1, 1)
    deq = lambda r_y: L.q8_conv_int8_dequantized(C.byref(dd), fake, fake, None, 0.02, 0.01, 0.5, None,
                                                 0.0, fake, r_y, None)
    assert deq(None) == -1
    assert deq(C.c_void_p(0x1002)) == -3


def test_chain_plan_accepts_a_block_and_sizes_its_workspace():
    arr = _chain_layers()
    n = B.lib.q8_conv_chain_plan_bytes(arr, 3)
    assert n > 0 and n % 256 == 0
    buf = C.create_string_buffer(n)
    assert B.lib.q8_conv_chain_plan(arr, 3, buf, n) == 0
    assert B.lib.q8_conv_chain_plan(arr, 3, buf, n - 1) == -1          # plan buffer too small
    ws = B.lib.q8_conv_chain_workspace_bytes(buf)
    # status line + per XCD a queue head line and one counter per pixel tile of every layer
    assert ws >= 4 * (32 + 8 * 32) and ws % 128 == 0
    fake = C.c_void_p(0x7F1000000000)
    assert B.lib.q8_conv_chain_int8(buf, fake, fake, ws - 4, None) == -5    # workspace too small
    assert B.lib.q8_conv_chain_int8(buf, C.c_void_p(0x7F1000000010), fake, ws, None) == -3
    assert B.lib.q8_conv_chain_int8(buf, None, fake, ws, None) == -1
    assert B.lib.q8_conv_chain_workspace_bytes(C.create_string_buffer(256)) == 0   # not a plan
    assert B.lib.q8_conv_chain_int8(C.create_string_buffer(256), fake, fake, 1 << 20, None) == -1
    assert B.lib.q8_conv_chain_int8_static(C.create_string_buffer(256), fake, None) == -1
    assert B.lib.q8_conv_chain_static_workspace_limit() == 1 << 20
    assert B.lib.q8_strerror(-5) != B.lib.q8_strerror(-99)


def test_chain_plan_rejects_inconsistent_lists():
    def plan_rc(bad):
        arr = _chain_layers(bad=bad)
        return B.lib.q8_conv_chain_plan_bytes(arr, 3)

    def forward_ref(arr): arr[1].src_layer = 2                     # reads a later layer
    def wrong_src(arr): arr[2].src_layer = 0                       # z_x is not that layer's z_y
    def alias(arr): arr[1].z_y = arr[0].z_y                        # a tensor written twice
    def clobber_input(arr): arr[2].z_y = arr[0].z_x                # writes what the list reads
    def odd_c(arr): arr[0].d.C = 48                                # not a chain geometry
    def sliced(arr): arr[2].d.out_c_off = 16
    def batches(arr): arr[1].d.N = 3
    def res_without_tensor(arr): arr[1].res_layer = 0
    for bad in (forward_ref, wrong_src, alias, clobber_input, odd_c, sliced, batches,
                res_without_tensor):
        assert plan_rc(bad) == 0, bad.__name__
    assert B.lib.q8_conv_chain_plan_bytes(None, 3) == 0
    assert B.lib.q8_conv_chain_plan_bytes(_chain_layers(), 0) == 0
    assert B.lib.q8_conv_chain_supported(C.byref(B.ConvDesc(8, 14, 14, 256, 256, 3, 3, 1, 1, 1, 1))) == 1
    assert B.lib.q8_conv_chain_supported(C.byref(B.ConvDesc(8, 14, 14, 48, 256, 3, 3, 1, 1, 1, 1))) == 0
    assert B.lib.q8_conv_chain_supported(C.byref(B.ConvDesc(8, 14, 14, 64, 16, 1, 1))) == 0


def test_chain_plan_splits_the_batch_over_eight_queues():
    import struct
    for n_img, want in ((16, [2] * 8), (13, [2, 2, 2, 2, 2, 1, 1, 1]), (3, [1, 1, 1, 0, 0, 0, 0, 0])):
        arr = _chain_layers(n_img)
        n = B.lib.q8_conv_chain_plan_bytes(arr, 3)
        buf = C.create_string_buffer(n)
        assert B.lib.q8_conv_chain_plan(arr, 3, buf, n) == 0
        hd = struct.unpack_from("<I7i8i", bytes(buf), 0)
        assert hd[1] == 3
        n_items = hd[8:16]
        # queue entries of an XCD are proportional to its images (28x28 = 784 pixels each)
        per_image = [i // w if w else 0 for i, w in zip(n_items, want)]
        assert [bool(i) for i in n_items] == [bool(w) for w in want]
        assert len({p for p, w in zip(per_image, want) if w == want[0]}) == 1
