"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs.

Bar: bit-exact for int8 codes, int32 accumulators, int32 bias, max-abs and the folded fp32
weights (each is a fixed sequence of IEEE operations); dequantised values within 1e-5
relative (they are in fact bit-equal: one fp32 multiply).
"""
import numpy as np
import pytest
import torch

import oracle as orc
from oracle import net as onet
from paper_1805_08691_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import paper_1805_08691_amd.binding as b
    assert torch.cuda.is_available()
    return b


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


# ------------------------------------------------------------------ calibration / Q / D
@pytest.mark.parametrize("n", [0, 1, 3, 5, 63, 1024, 4099, 1_000_003, 8_388_608 + 7])
@pytest.mark.parametrize("offset", [0, 1, 3])
def test_maxabs(B, n, offset):
    rng = np.random.default_rng(n + offset)
    x = rng.standard_normal(n + offset).astype(np.float32)
    if n > 10:
        x[offset + int(rng.integers(0, n))] = -7.25     # a single extreme, negative
    xd = dev(x)[offset:]
    slot = torch.zeros(1, device="cuda")
    B.calibrate_maxabs(xd, slot)
    assert host(slot)[0] == orc.maxabs(x[offset:])
    # running maximum over a second batch
    x2 = (x * np.float32(0.5)).astype(np.float32)
    x2[-1:] = 9.5
    B.calibrate_maxabs(dev(x2)[offset:], slot)
    assert host(slot)[0] == max(orc.maxabs(x[offset:]), orc.maxabs(x2[offset:]))


@pytest.mark.parametrize("n", [0, 1, 2, 7, 1023, 65536 + 5, 3_000_001])
@pytest.mark.parametrize("offset", [0, 1, 2])
@pytest.mark.parametrize("p", [7, 4])
def test_quantize(B, n, offset, p):
    rng = np.random.default_rng(100 + n + offset)
    x = (rng.standard_normal(n + offset) * 2).astype(np.float32)
    q = np.float32(0.0371)
    if n > 64:      # exact ties and saturating values
        k = np.arange(-40, 24)
        x[offset:offset + 64] = (k.astype(np.float32) + np.float32(0.5)) * q
        x[offset + 64 - 4:offset + 64] = [1e6, -1e6, 127.5 * q, -128.5 * q]
    z = B.quantize(dev(x)[offset:], float(q), p)
    assert np.array_equal(host(z), orc.Q(x[offset:], q, p))


def test_quantize_pad_channels(B):
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 9, 11, 3)).astype(np.float32)
    q = orc.qfactor(orc.maxabs(x), 7)
    z = host(B.quantize_pad_channels(dev(x), 4, float(q), 7))
    assert z.shape == (2, 9, 11, 4)
    assert np.array_equal(z[..., :3], orc.Q(x, q, 7)) and np.all(z[..., 3] == 0)
    z = host(B.quantize_pad_channels(dev(x), 16, float(q), 7))
    assert np.array_equal(z[..., :3], orc.Q(x, q, 7)) and np.all(z[..., 3:] == 0)


@pytest.mark.parametrize("n", [0, 1, 5, 1024, 1_000_003])
@pytest.mark.parametrize("offset", [0, 1])
def test_dequantize(B, n, offset):
    rng = np.random.default_rng(200 + n)
    z = rng.integers(-128, 128, n + offset).astype(np.int8)
    q = np.float32(0.0123)
    r = host(B.dequantize(dev(z)[offset:], float(q)))
    want = orc.D(z[offset:], q)
    assert np.array_equal(r, want)
    assert np.all(np.abs(r - want) <= 1e-5 * np.abs(want))


def test_elementwise_passes_beyond_2_31_elements(B):
    """Max-abs, Eq. Q and Eq. D on a tensor of more than 2^31 elements (64-bit indexing): a
    constant with a few planted values, checked on those and on sums over the whole tensor."""
    n = 2**31 + 1029
    x = torch.full((n,), 0.25, dtype=torch.float32, device="cuda")
    planted = {0: 3.0, 12345: -0.75, 2**31 - 1: 1.25, 2**31: -1.75, 2**31 + 3: 12.75, n - 1: -77.5}
    for i, v in planted.items():
        x[i] = v
    slot = torch.zeros(1, dtype=torch.float32, device="cuda")
    B.calibrate_maxabs(x, slot)
    assert float(host(slot)[0]) == 77.5                     # the extreme is the very last element
    q = np.float32(0.5)
    z = B.quantize(x, float(q), 7)
    idx = sorted(planted)
    want = orc.Q(np.array([planted[i] for i in idx], np.float32), q, 7)
    assert [int(z[i]) for i in idx] == want.tolist()        # incl. the tie 25.5 -> 26, clamp at -128
    assert int(orc.Q(np.array([0.25], np.float32), q, 7)[0]) == 0
    assert int(z.sum(dtype=torch.int64)) == int(want.astype(np.int64).sum())   # every other code is 0
    del x
    r = B.dequantize(z, float(q))
    assert [float(r[i]) for i in idx] == orc.D(want, q).tolist()
    assert int(torch.count_nonzero(r)) == int(np.count_nonzero(want))


def test_quantize_bias(B):
    rng = np.random.default_rng(9)
    b = (rng.standard_normal(1000) * 0.1).astype(np.float32)
    b[:4] = [1e9, -1e9, 0.0, 1e-12]
    for q_x, q_w in [(0.0137, 0.00091), (1.0, 1.0), (3e-3, 2.5e-4)]:
        z = host(B.quantize_bias(dev(b), q_x, q_w))
        assert np.array_equal(z, orc.Q31_bias(b, q_x, q_w))


@pytest.mark.parametrize("K,RSC", [(1, 1), (3, 7), (64, 576), (130, 1030)])
def test_fold_bn(B, K, RSC):
    rng = np.random.default_rng(K * 1000 + RSC)
    W = rng.standard_normal((K, RSC)).astype(np.float32)
    b = rng.standard_normal(K).astype(np.float32)
    gamma = rng.uniform(.5, 1.5, K).astype(np.float32)
    beta = (rng.standard_normal(K) * .1).astype(np.float32)
    mu = (rng.standard_normal(K) * .1).astype(np.float32)
    var = rng.uniform(.5, 1.5, K).astype(np.float32)
    Wf, bf = B.fold_bn(dev(W), dev(b), dev(gamma), dev(beta), dev(mu), dev(var), 1e-5)
    Wo, bo = orc.fold_bn(W, b, gamma, beta, mu, var, 1e-5)
    assert np.array_equal(host(Wf), Wo) and np.array_equal(host(bf), bo)
    Wf, bf = B.fold_bn(dev(W), None, dev(gamma), dev(beta), dev(mu), dev(var), 1e-5)
    Wo, bo = orc.fold_bn(W, None, gamma, beta, mu, var, 1e-5)
    assert np.array_equal(host(Wf), Wo) and np.array_equal(host(bf), bo)


# ------------------------------------------------------------------ convolution
CONV_CASES = [
    # several tiles and ragged tails in pixels, channels and reduction
    dict(N=2, H=14, W=14, C=32, K=48, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=3, H=13, W=11, C=64, K=64, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=1, H=56, W=56, C=64, K=64, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=2, H=28, W=28, C=128, K=160, R=1, S=1),
    dict(N=2, H=28, W=28, C=256, K=128, R=1, S=1, stride_h=2, stride_w=2),
    dict(N=1, H=17, W=17, C=128, K=192, R=1, S=7, pad_w=3),
    dict(N=1, H=17, W=17, C=128, K=192, R=7, S=1, pad_h=3),
    dict(N=1, H=19, W=19, C=64, K=96, R=3, S=3, dil_h=6, dil_w=6, pad_h=6, pad_w=6),
    dict(N=2, H=12, W=12, C=48, K=64, R=5, S=5, pad_h=2, pad_w=2),
    dict(N=1, H=35, W=35, C=80, K=24, R=3, S=3, stride_h=2, stride_w=2),
    dict(N=1, H=10, W=10, C=16, K=126, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=2, H=9, W=9, C=16, K=17, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=1, H=3, W=3, C=256, K=16, R=3, S=3),
    dict(N=4, H=1, W=1, C=256, K=84, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=2, H=37, W=41, C=3, K=64, R=7, S=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3),
    dict(N=2, H=37, W=40, C=3, K=64, R=7, S=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3),  # rows of
    dict(N=3, H=9, W=12, C=3, K=64, R=3, S=3, pad_h=1, pad_w=1),     # whole 4-pixel groups
    dict(N=1, H=20, W=20, C=3, K=32, R=3, S=3, stride_h=2, stride_w=2),
    dict(N=1, H=16, W=16, C=4, K=8, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=1, H=7, W=7, C=512, K=2048 // 8, R=1, S=1),
    # more than 32 taps over 16-channel chunks: the register-staged kernel
    dict(N=1, H=15, W=15, C=16, K=40, R=7, S=7, pad_h=3, pad_w=3),
    dict(N=2, H=13, W=9, C=32, K=72, R=6, S=6, stride_h=2, stride_w=1, pad_h=2, pad_w=3),
    # a fully connected layer (Eq. A covers it): 1x1 convolution on a 1x1 map, M = batch
    dict(N=64, H=1, W=1, C=2048, K=1000, R=1, S=1),
]


def _run_conv_case(B, geom, relu, with_res, with_bias, seed, out_pad=0, out_off=0, variant=-1,
                   dump_acc=True, n_split=0, workspace=None):
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(seed)
    Cs = 4 if g.C < 4 else g.C                      # stored channels of the input
    x = rng.integers(-128, 128, (g.N, g.H, g.W, Cs)).astype(np.int8)
    w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
    b = rng.integers(-20000, 20000, g.K).astype(np.int32) if with_bias else None
    Ho, Wo = g.Ho, g.Wo
    q_x, q_w = np.float32(0.021), np.float32(0.0017)
    fan = g.R * g.S * g.C
    # accumulators have std ~ 74^2 sqrt(fan): aim at ~40 output codes std, a few saturate
    q_out = np.float32(q_x * q_w * 5476.0 * np.sqrt(fan) / 40.0)
    q_res = np.float32(0.3) * q_out
    res = rng.integers(-128, 128, (g.N, Ho, Wo, g.K)).astype(np.int8) if with_res else None

    go = orc.ConvGeom(**{**geom, "in_c_stride": Cs})
    acc_o = orc.conv_i8(go, x, w, b)
    m = orc.requant_scale(q_x, q_w, q_out)
    m_r = orc.residual_scale(q_res, q_out) if with_res else 0.0
    out_cs = g.K + out_pad
    want = np.full((g.N, Ho, Wo, out_cs), 77, np.int8)
    orc.requant(acc_o, m, relu, res, m_r, out=want, out_c_stride=out_cs, out_c_off=out_off)

    d = B.ConvDesc(g.N, g.H, g.W, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, g.pad_h, g.pad_w,
                   g.dil_h, g.dil_w, relu=relu, in_c_stride=Cs, out_c_stride=out_cs,
                   out_c_off=out_off)
    packed = B.pack_weights(d, dev(w))
    out = torch.full((g.N, Ho, Wo, out_cs), 77, dtype=torch.int8, device="cuda")
    dump = torch.zeros((g.N, Ho, Wo, g.K), dtype=torch.int32, device="cuda")
    B.conv_int8(d, dev(x), packed, None if b is None else dev(b), float(q_x), float(q_w),
                float(q_out), None if res is None else dev(res), float(q_res), out=out,
                acc_dump=dump if dump_acc else None, variant=variant, n_split=n_split,
                workspace=workspace)
    if dump_acc:
        assert np.array_equal(host(dump), acc_o), "int32 accumulators differ"
    got = host(out)
    assert np.array_equal(got, want), "int8 outputs differ"
    frac_sat = np.mean(np.abs(want[..., out_off:out_off + g.K].astype(int)) >= 127)
    assert frac_sat < 0.5


@pytest.mark.parametrize("idx", range(len(CONV_CASES)))
def test_conv_shapes(B, idx):
    geom = CONV_CASES[idx]
    _run_conv_case(B, geom, relu=True, with_res=False, with_bias=True, seed=idx)
    _run_conv_case(B, geom, relu=(idx % 2 == 0), with_res=True, with_bias=(idx % 3 != 0),
                   seed=1000 + idx)


VARIANT_CASES = [
    dict(N=2, H=14, W=14, C=64, K=160, R=3, S=3, pad_h=1, pad_w=1),      # uniform taps, tails
    dict(N=1, H=17, W=17, C=48, K=272, R=1, S=7, pad_w=3),               # per-lane taps, tails
    dict(N=3, H=28, W=28, C=128, K=64, R=1, S=1, stride_h=2, stride_w=2),
    dict(N=1, H=33, W=31, C=256, K=384, R=1, S=1),                       # complete + ragged tiles
    dict(N=2, H=43, W=47, C=3, K=96, R=7, S=7, stride_h=2, stride_w=2),  # unpadded 4-channel image
]


def test_conv_every_kernel_variant(B):
    """Every tile / ring variant of the main kernel gives the same bits (integer sums are
    order-independent; the epilogue is one fixed fp32 sequence)."""
    n = B.conv_num_variants()
    assert n >= 10
    for v in range(n):
        for k, geom in enumerate(VARIANT_CASES):
            _run_conv_case(B, geom, relu=bool(k % 2), with_res=bool((k + v) % 2),
                           with_bias=True, seed=100 * v + k, variant=v)


HALO_CASES = [   # 3x3, stride 1, padding 1, C % 64 == 0: the shapes the 3x3 tile family takes
    dict(N=3, H=7, W=7, C=64, K=64),          # several images inside one pixel tile
    dict(N=5, H=7, W=7, C=512, K=128),        # eight channel chunks, ragged last pixel tile
    dict(N=2, H=14, W=14, C=128, K=128),
    dict(N=1, H=28, W=28, C=64, K=256),
    dict(N=2, H=9, W=31, C=192, K=96),        # three chunks, K ends inside a channel tile
    dict(N=1, H=5, W=63, C=64, K=64),         # the widest map of the narrow patch buffers
    dict(N=1, H=3, W=100, C=64, K=128),       # only the wide patch buffers take it
    dict(N=1, H=2, W=300, C=64, K=64),        # only the widest one
    dict(N=1, H=1, W=1, C=64, K=64),          # one pixel: only the centre tap is inside
    dict(N=2, H=1, W=17, C=64, K=64),         # one row: no tap above or below
]


@pytest.mark.parametrize("idx", range(len(HALO_CASES)))
def test_conv_3x3_tile_family(B, idx):
    """Every build of the 3x3 tile family (activation patch with halo staged once per channel
    chunk, nine taps as nine row offsets) against the oracle; a build whose patch buffer is too
    narrow for the map hands the layer to the generic kernel, which must give the same bits."""
    geom = dict(R=3, S=3, pad_h=1, pad_w=1, **HALO_CASES[idx])
    n = B.conv_num_variants()
    names = [B.lib.q8_conv_variant_name(v).decode() for v in range(n)]
    halo = [v for v in range(n) if "halo3" in names[v]]
    assert len(halo) >= 4
    for k, v in enumerate(halo):
        _run_conv_case(B, geom, relu=bool(k % 2), with_res=bool((k + idx) % 2), with_bias=True,
                       seed=1000 * idx + v, variant=v)


P3_CASES = [     # 3x3, stride 1, padding 1, C = 64, K <= 64: what the persistent 3x3 family takes
    dict(N=2, H=56, W=56, C=64, K=64),        # several tiles per workgroup? no: one pass, ragged end
    dict(N=40, H=28, W=28, C=64, K=64),       # more tiles than resident workgroups: two passes
    dict(N=3, H=7, W=7, C=64, K=64),          # several images inside one pixel tile
    dict(N=1, H=5, W=63, C=64, K=48),         # the widest map of the narrow patch, K short of the tile
    dict(N=1, H=3, W=100, C=64, K=64),        # only the wide patch takes it
    dict(N=1, H=1, W=1, C=64, K=16),          # one pixel
    dict(N=2, H=1, W=17, C=64, K=32),         # one row: no tap above or below
    dict(N=2, H=19, W=301, C=64, K=64),       # a wide map: only the block-tiled build takes it
    dict(N=3, H=9, W=16, C=64, K=16),         # blocks: a ragged last block row, exact columns
]


@pytest.mark.parametrize("idx", range(len(P3_CASES)))
def test_conv_persistent_3x3_family(B, idx):
    """Every build of the persistent 3x3 family (all filters resident in LDS, workgroups walk
    over pixel tiles with the next tile's activation patch in flight) against the oracle; a
    build whose patch is too narrow for the map hands the layer to the generic kernel."""
    geom = dict(R=3, S=3, pad_h=1, pad_w=1, **P3_CASES[idx])
    n = B.conv_num_variants()
    names = [B.lib.q8_conv_variant_name(v).decode() for v in range(n)]
    p3 = [v for v in range(n) if "p3_kernel" in names[v] or "p3b_kernel" in names[v]]
    assert len(p3) >= 3
    for k, v in enumerate(p3):
        _run_conv_case(B, geom, relu=bool(k % 2), with_res=False, with_bias=True,
                       seed=5000 * idx + v, variant=v, out_pad=16 * (k % 2), out_off=16 * (k % 2),
                       dump_acc=False)


STEM_CASES = [   # unpadded 4-channel images, 5..8 taps per filter row: the image-row family
    dict(N=2, H=43, W=47, C=3, K=64, R=7, S=7, stride_h=2, stride_w=2),
    dict(N=3, H=230, W=230, C=3, K=64, R=7, S=7, stride_h=2, stride_w=2),   # ResNet-50's first layer
    dict(N=3, H=20, W=240, C=4, K=48, R=5, S=8, stride_h=1, stride_w=2),    # the widest image, K short
    dict(N=1, H=12, W=100, C=3, K=16, R=3, S=5),                            # stride 1
    dict(N=2, H=40, W=60, C=2, K=32, R=8, S=6, stride_h=4, stride_w=2),     # 8 + 4 rows in the ring
    dict(N=37, H=19, W=33, C=1, K=64, R=7, S=7, stride_h=2, stride_w=2),    # many images, short strips
    dict(N=1, H=9, W=200, C=3, K=64, R=3, S=5),                             # rows too long: generic kernel
]


@pytest.mark.parametrize("idx", range(len(STEM_CASES)))
def test_conv_image_row_family(B, idx):
    """The image-row family (filters resident, a ring of image rows in LDS as the activation
    operand, workgroups walking down strips of output rows) against the oracle, with and
    without ReLU and with a strided output; ResNet-50's first layer also picks it by itself."""
    geom = STEM_CASES[idx]
    n = B.conv_num_variants()
    names = [B.lib.q8_conv_variant_name(v).decode() for v in range(n)]
    stem = [v for v in range(n) if "stem_kernel" in names[v]]
    assert len(stem) == 1
    for k in range(2):
        _run_conv_case(B, geom, relu=bool(k), with_res=False, with_bias=bool(k), seed=7000 + 10 * idx + k,
                       variant=stem[0], out_pad=16 * k, out_off=16 * k, dump_acc=False)
    if idx == 1:
        g = orc.ConvGeom(**geom)
        d = B.ConvDesc(g.N, g.H, g.W, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, 0, 0, 1, 1,
                       relu=1, in_c_stride=4)
        assert "stem_kernel" in B.conv_variant(d)
        _run_conv_case(B, geom, relu=True, with_res=False, with_bias=True, seed=7777, dump_acc=False)


HEAD_CASES = [   # image (N, H, W, C), filter, strides, padding = the zero frame around the image
    dict(N=2, H=37, W=41, C=3, K=64, R=7, S=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3),
    dict(N=3, H=224, W=224, C=3, K=64, R=7, S=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3),  # ResNet-50
    dict(N=1, H=24, W=20, C=1, K=48, R=5, S=5, stride_h=2, stride_w=2, pad_h=2, pad_w=2),
    dict(N=2, H=33, W=232, C=4, K=32, R=8, S=8, stride_h=2, stride_w=2, pad_h=4, pad_w=4),   # widest frame
    dict(N=35, H=19, W=33, C=2, K=16, R=3, S=6, stride_h=2, stride_w=1, pad_h=1, pad_w=2),
    dict(N=1, H=3, W=9, C=3, K=64, R=7, S=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3),       # one or two rows
    dict(N=2, H=18, W=30, C=3, K=64, R=5, S=7, stride_h=1, stride_w=1, pad_h=2, pad_w=3),     # stride 1: no pool
]


@pytest.mark.parametrize("idx", range(len(HEAD_CASES)))
def test_conv_image_f32_head(B, idx):
    """Eq. Q on the real-valued image, the first layer and the 3x3 / 2 max-pool as one launch
    against the oracle's three steps (quantise, padded convolution + requantisation, max-pool
    of the codes); values next to rounding ties and beyond the code range are in the image."""
    geom = HEAD_CASES[idx]
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(900 + idx)
    r = rng.standard_normal((g.N, g.H, g.W, g.C)).astype(np.float32)
    q_x = orc.qfactor(np.float32(2.9), 7)                       # |r| > 2.9 saturates
    flat = r.reshape(-1)
    where = rng.choice(flat.size, flat.size // 7, replace=False)
    ties = ((rng.integers(-130, 130, where.size).astype(np.float32) + np.float32(0.5)) * q_x).astype(np.float32)
    toward = np.float32([-np.inf, 0.0, np.inf])[rng.integers(0, 3, where.size)]
    flat[where] = np.nextafter(ties, toward)                    # a tie or an fp32 neighbour of it
    z_x = orc.Q(r, q_x, 7)
    w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
    b = rng.integers(-2000, 2000, g.K).astype(np.int32)
    q_w = np.float32(0.004)
    q_out = np.float32(q_x * q_w * 74 * 40 * np.sqrt(g.R * g.S * g.C) / 40.0)
    Hs, Ws = g.H + 2 * g.pad_h, g.W + 2 * g.pad_w
    d = B.ConvDesc(g.N, Hs, Ws, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, 0, 0, 1, 1,
                   relu=1, in_c_stride=4)
    packed = B.pack_weights(d, dev(w))
    for relu in (1, 0):
        d.relu = relu
        conv = orc.requant(orc.conv_i8(g, z_x, w, b), orc.requant_scale(q_x, q_w, q_out), bool(relu))
        for pool in (0, 1):
            ok = B.conv_image_f32_supported(d, g.H, g.W, g.C, g.pad_h, g.pad_w, pool)
            assert ok == (not (pool and g.stride_h != 2))
            if not ok:
                continue
            want = orc.maxpool_i8(conv, 3, 3, 2, 1, (g.Ho - 1) // 2 + 1, (g.Wo - 1) // 2 + 1) if pool else conv
            out = torch.full(want.shape, 77, dtype=torch.int8, device="cuda")
            B.conv_image_f32(d, dev(r), g.pad_h, g.pad_w, float(q_x), 7, packed, dev(b), float(q_w),
                             float(q_out), pool=pool, out=out)
            assert np.array_equal(host(out), want), f"relu={relu} pool={pool}"


@pytest.mark.parametrize("geom", [
    dict(N=2, H=7, W=7, C=512, K=2048, R=1, S=1),                          # ResNet-50's last layer
    dict(N=1, H=9, W=11, C=64, K=40, R=3, S=3, pad_h=1, pad_w=1),          # K ends inside a group
    dict(N=3, H=5, W=5, C=3, K=24, R=3, S=3, pad_h=1, pad_w=1),            # the small-channel kernel
])
def test_conv_with_dequantized_output(B, geom):
    """Eq. A' and Eq. D in one launch: the codes equal the oracle's, and the fp32 tensor is
    Eq. D of those codes (one fp32 multiplication, bit for bit); channels outside the
    layer's slice of a wider tensor are left alone."""
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(4242 + g.K)
    Cs = 4 if g.C < 4 else g.C
    x = rng.integers(-128, 128, (g.N, g.H, g.W, Cs)).astype(np.int8)
    w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
    b = rng.integers(-20000, 20000, g.K).astype(np.int32)
    res = rng.integers(-128, 128, (g.N, g.Ho, g.Wo, g.K)).astype(np.int8)
    q_x, q_w = np.float32(0.021), np.float32(0.0017)
    q_out = np.float32(q_x * q_w * 5476.0 * np.sqrt(g.R * g.S * g.C) / 40.0)
    q_res = np.float32(0.3) * q_out
    go = orc.ConvGeom(**{**geom, "in_c_stride": Cs})
    acc = orc.conv_i8(go, x, w, b)
    for with_res, pad in ((True, 0), (False, 8)):
        ocs = g.K + pad
        want = np.full((g.N, g.Ho, g.Wo, ocs), 77, np.int8)
        orc.requant(acc, orc.requant_scale(q_x, q_w, q_out), True, res if with_res else None,
                    orc.residual_scale(q_res, q_out) if with_res else 0.0, out=want,
                    out_c_stride=ocs, out_c_off=pad)
        d = B.ConvDesc(g.N, g.H, g.W, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, g.pad_h, g.pad_w,
                       g.dil_h, g.dil_w, relu=1, in_c_stride=Cs, out_c_stride=ocs, out_c_off=pad)
        out = torch.full(want.shape, 77, dtype=torch.int8, device="cuda")
        out_f = torch.full(want.shape, -5.0, dtype=torch.float32, device="cuda")
        B.conv_int8_dequantized(d, dev(x), B.pack_weights(d, dev(w)), dev(b), float(q_x), float(q_w),
                                float(q_out), dev(res) if with_res else None, float(q_res),
                                out=out, out_f32=out_f)
        assert np.array_equal(host(out), want)
        want_f = np.full(want.shape, -5.0, np.float32)
        want_f[..., pad:] = orc.D(want[..., pad:], q_out)
        assert np.array_equal(host(out_f), want_f)


def test_conv_image_f32_head_rejects(B):
    """Host checks of the fused head: a layer outside the family is unsupported, an image that
    does not fit its frame is invalid."""
    d = B.ConvDesc(1, 30, 30, 3, 64, 3, 3, 1, 1, 0, 0, 1, 1, relu=1, in_c_stride=4)   # 3 columns
    assert not B.conv_image_f32_supported(d, 28, 28, 3, 1, 1, 0)
    d = B.ConvDesc(1, 30, 30, 3, 64, 7, 7, 2, 2, 0, 0, 1, 1, relu=1, in_c_stride=4)
    assert B.conv_image_f32_supported(d, 24, 24, 3, 3, 3, 1)
    assert not B.conv_image_f32_supported(d, 28, 24, 3, 3, 3, 1)                     # 3 + 28 > 30
    assert not B.conv_image_f32_supported(d, 24, 24, 4, 3, 3, 1)                     # C != d.C
    r = torch.zeros((1, 28, 24, 3), dtype=torch.float32, device="cuda")
    w = torch.zeros((64, 7, 7, 3), dtype=torch.int8, device="cuda")
    with pytest.raises(B.Q8Error):
        B.conv_image_f32(d, r, 3, 3, 0.02, 7, B.pack_weights(d, w), None, 0.01, 0.5)


SPLIT_CASES = [   # long reductions over few output tiles: what a split reduction is for
    dict(N=5, H=7, W=7, C=512, K=512, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=3, H=14, W=14, C=1024, K=256, R=1, S=1),
    dict(N=2, H=9, W=11, C=192, K=96, R=3, S=3, pad_h=1, pad_w=1),        # ragged tiles
    dict(N=1, H=14, W=14, C=1024, K=512, R=1, S=1, stride_h=2, stride_w=2),
    dict(N=2, H=8, W=8, C=128, K=128, R=3, S=3, pad_h=2, pad_w=2, dil_h=2, dil_w=2),
    dict(N=1, H=6, W=6, C=64, K=64, R=1, S=1),                             # one step: never split
]


@pytest.mark.parametrize("idx", range(len(SPLIT_CASES)))
def test_conv_split_reduction(B, idx):
    """Eq. x: the accumulator is an integer sum, so splitting the reduction over 2, 3, 5 or 7
    workgroups per tile (partial tiles through the caller's workspace, the last workgroup to
    arrive adds them up) gives the oracle's accumulators and codes bit for bit, with every
    split build.  One workspace, zeroed once, serves all calls: each leaves its counters zero."""
    geom = SPLIT_CASES[idx]
    g = orc.ConvGeom(**geom)
    d = B.ConvDesc(g.N, g.H, g.W, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, g.pad_h, g.pad_w,
                   g.dil_h, g.dil_w)
    n = B.conv_num_variants()
    names = [B.lib.q8_conv_variant_name(v).decode() for v in range(n)]
    split = [v for v in range(n) if "split" in names[v]]
    assert len(split) >= 4
    factors = (2, 3, 5, 7)
    need = max(B.conv_workspace_bytes(d, v, f) for v in split for f in factors)
    ws = torch.zeros(max(need, 256), dtype=torch.uint8, device="cuda")
    for k, v in enumerate(split):
        for f in factors:
            _run_conv_case(B, geom, relu=bool((k + f) % 2), with_res=bool(k % 2), with_bias=True,
                           seed=7000 + 100 * idx + 10 * k + f, variant=v, n_split=f, workspace=ws)
    if need:
        words = B.conv_workspace_bytes(d, split[0], 2)      # (an upper bound on the counters)
        assert not host(ws[:min(words, 4096)]).view(np.int32)[:16].any()


PW_CASES = [     # 1x1, stride 1, no padding, C in {64, 128, 256}: what the pointwise family takes
    dict(N=2, H=56, W=56, C=64, K=256),       # many pixel tiles per workgroup, ragged last tile
    dict(N=1, H=28, W=28, C=128, K=512),
    dict(N=3, H=19, W=23, C=256, K=64),
    dict(N=1, H=9, W=9, C=64, K=64),          # fewer pixel tiles than workgroups
    dict(N=2, H=31, W=17, C=128, K=96),       # K ends inside a channel tile
    dict(N=40, H=28, W=28, C=64, K=128),      # more pixel tiles than one round of workgroups
    dict(N=1, H=1, W=1, C=256, K=320),
]


@pytest.mark.parametrize("idx", range(len(PW_CASES)))
def test_conv_pointwise_tile_family(B, idx):
    """Every build of the pointwise tile family (persistent workgroups, filters resident in LDS,
    the next pixel tile's operands in flight while the current one is computed) against the
    oracle; a build made for another channel count hands the layer to the generic kernel."""
    geom = dict(R=1, S=1, **PW_CASES[idx])
    n = B.conv_num_variants()
    names = [B.lib.q8_conv_variant_name(v).decode() for v in range(n)]
    pw = [v for v in range(n) if "pw_kernel" in names[v]]
    assert len(pw) >= 4
    for k, v in enumerate(pw):
        for with_res in (False, True):
            _run_conv_case(B, geom, relu=bool((k + with_res) % 2), with_res=with_res,
                           with_bias=True, seed=3000 * idx + 2 * v + with_res, variant=v,
                           out_pad=16 * (k % 2), out_off=16 * (k % 2), dump_acc=False)


@pytest.mark.parametrize("q", [0.03, 0.0078125, 1.0 / 3.0, 0.0123456789, 5.5e-3])
def test_quantize_image_next_to_ties(B, q):
    """Eq. Q on values whose quotient r/q lies on, and within a few ulps of, every tie k + 1/2
    and every integer k of the code range (and beyond its ends): the image kernel, which only
    divides where a product with 1/q cannot decide the rounding, must give the oracle's codes."""
    q = np.float32(q)
    ks = np.arange(-131, 131, dtype=np.float64)
    centres = np.concatenate([ks + 0.5, ks]) * np.float64(q)
    vals = []
    for c in centres.astype(np.float32):
        v = c
        for _ in range(6):
            v = np.nextafter(v, np.float32(-np.inf), dtype=np.float32)
        for _ in range(13):
            vals.append(v)
            v = np.nextafter(v, np.float32(np.inf), dtype=np.float32)
    vals = np.array(vals, dtype=np.float32)
    n_pix = -(-vals.size // 3)
    W = 8
    Hh = -(-n_pix // W)
    r = np.zeros((1, Hh, W, 3), np.float32)
    r.reshape(-1)[:vals.size] = vals
    want = orc.Q(r, q, 7)
    ties = np.abs(np.abs(vals.astype(np.float64) / np.float64(q)) % 1.0 - 0.5) < 1e-4
    assert ties.sum() > 2000                                 # the cases are what they claim to be
    frame = torch.zeros((1, Hh, W, 4), dtype=torch.int8, device="cuda")
    B.quantize_image(dev(r), float(q), 7, frame, 0, 0)
    got = host(frame)
    assert np.array_equal(got[..., :3], want)
    assert not got[..., 3].any()


@pytest.mark.parametrize("geom", [
    dict(N=2, H=37, W=41, C=3, K=64, R=7, S=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3),
    dict(N=1, H=39, W=39, C=3, K=64, R=3, S=3, stride_h=2, stride_w=2),
    dict(N=2, H=30, W=31, C=3, K=64, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=1, H=24, W=20, C=1, K=40, R=5, S=5, pad_h=2, pad_w=2),
    dict(N=1, H=12, W=12, C=4, K=48, R=3, S=9, pad_h=1, pad_w=4),
])
def test_conv_image_in_zero_frame(B, geom):
    """A C <= 4 image quantised into a zero frame that holds the layer's padding, the layer
    then run without padding, equals the oracle's padded convolution of the bare image."""
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(g.H * 100 + g.W)
    r = rng.standard_normal((g.N, g.H, g.W, g.C)).astype(np.float32)
    q_x = orc.qfactor(orc.maxabs(r), 7)
    z_x = orc.Q(r, q_x, 7)
    w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
    b = rng.integers(-2000, 2000, g.K).astype(np.int32)
    q_w = np.float32(0.004)
    q_out = np.float32(q_x * q_w * 74 * 40 * np.sqrt(g.R * g.S * g.C) / 40.0)
    acc_o = orc.conv_i8(g, z_x, w, b)
    want = orc.requant(acc_o, orc.requant_scale(q_x, q_w, q_out), True)

    Hs, Ws = g.H + 2 * g.pad_h, g.W + 2 * g.pad_w
    frame = torch.zeros((g.N, Hs, Ws, 4), dtype=torch.int8, device="cuda")
    B.quantize_image(dev(r), float(q_x), 7, frame, g.pad_h, g.pad_w)
    f = host(frame)
    assert np.array_equal(f[:, g.pad_h:g.pad_h + g.H, g.pad_w:g.pad_w + g.W, :g.C], z_x)
    f[:, g.pad_h:g.pad_h + g.H, g.pad_w:g.pad_w + g.W, :g.C] = 0
    assert not f.any()
    d = B.ConvDesc(g.N, Hs, Ws, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, 0, 0, 1, 1,
                   relu=1, in_c_stride=4)
    assert (d.Ho, d.Wo) == (g.Ho, g.Wo)
    assert "ring" in B.conv_variant(d)
    dump = torch.zeros((g.N, g.Ho, g.Wo, g.K), dtype=torch.int32, device="cuda")
    got = B.conv_int8(d, frame, B.pack_weights(d, dev(w)), dev(b), float(q_x), float(q_w),
                      float(q_out), acc_dump=dump)
    assert np.array_equal(host(dump), acc_o)
    assert np.array_equal(host(got), want)


# ------------------------------------------------------------------ unsigned activations
def _stored(u8):
    """unsigned codes -> the stored form (code - 128 in an int8 byte)."""
    return (u8.astype(np.int16) - 128).astype(np.int8)


def test_quantize_dequantize_u8(B):
    rng = np.random.default_rng(81)
    r = np.abs(rng.standard_normal(100_003)).astype(np.float32) * 3
    r[:4] = [0.0, 1e-9, 1e9, 2.5]
    q = orc.qfactor(np.float32(9.0), 8)              # some values saturate at 255
    want = orc.Q_u8(r, q)
    got = host(B.quantize_u8(dev(r), float(q)))
    assert np.array_equal(got, _stored(want))
    back = host(B.dequantize_u8(dev(got), float(q)))
    assert np.array_equal(back, orc.D_u8(want, q))


U8_CASES = [
    # geometry, in_u8, out_u8, res ("u8", "s8" or None), relu
    (dict(N=2, H=14, W=14, C=64, K=160, R=3, S=3, pad_h=1, pad_w=1), 1, 1, "u8", 1),
    (dict(N=2, H=14, W=14, C=64, K=160, R=3, S=3, pad_h=1, pad_w=1), 1, 0, "s8", 0),
    (dict(N=1, H=15, W=13, C=32, K=64, R=3, S=3, pad_h=1, pad_w=1, stride_h=2, stride_w=2), 1, 1, None, 1),
    (dict(N=3, H=9, W=9, C=128, K=256, R=1, S=1), 1, 1, "s8", 1),
    (dict(N=3, H=9, W=9, C=128, K=256, R=1, S=1), 0, 1, "u8", 1),
    (dict(N=1, H=17, W=17, C=48, K=96, R=1, S=7, pad_w=3), 1, 0, None, 1),
    (dict(N=1, H=12, W=12, C=16, K=72, R=3, S=3, dil_h=2, dil_w=2, pad_h=2, pad_w=2), 1, 1, "u8", 1),
    (dict(N=1, H=7, W=7, C=64, K=64, R=5, S=5, pad_h=2, pad_w=2), 1, 1, None, 1),   # mostly border
    (dict(N=2, H=28, W=28, C=64, K=128, R=3, S=3, pad_h=1, pad_w=1), 1, 1, "u8", 1),  # complete tiles
]


@pytest.mark.parametrize("idx", range(len(U8_CASES)))
def test_conv_unsigned_activations(B, idx):
    """Eq. A' on unsigned p = 8 codes (the paper's form for non-negative tensors) through
    the signed matrix instruction: accumulators and outputs equal the oracle's, which
    works on the codes 0..255 themselves."""
    geom, in_u8, out_u8, res_kind, relu = U8_CASES[idx]
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(500 + idx)
    w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
    b = rng.integers(-20000, 20000, g.K).astype(np.int32)
    if in_u8:
        x = rng.integers(0, 256, (g.N, g.H, g.W, g.C)).astype(np.uint8)
        acc_o = orc.conv_u8(g, x, w, b)
        x_st = _stored(x)
    else:
        x = rng.integers(-128, 128, (g.N, g.H, g.W, g.C)).astype(np.int8)
        acc_o = orc.conv_i8(g, x, w, b)
        x_st = x
    Ho, Wo = g.Ho, g.Wo
    q_x, q_w = np.float32(0.011), np.float32(0.0017)
    fan = g.R * g.S * g.C
    q_out = np.float32(q_x * q_w * 74.0 * (147.0 if in_u8 else 74.0) * np.sqrt(fan) / 60.0)
    q_res = np.float32(0.4) * q_out
    res = res_st = None
    if res_kind == "u8":
        res = rng.integers(0, 256, (g.N, Ho, Wo, g.K)).astype(np.uint8)
        res_st = _stored(res)
    elif res_kind == "s8":
        res = res_st = rng.integers(-128, 128, (g.N, Ho, Wo, g.K)).astype(np.int8)
    m = orc.requant_scale(q_x, q_w, q_out)
    m_r = orc.residual_scale(q_res, q_out) if res is not None else 0.0
    want = orc.requant_mixed(acc_o, m, relu, res, m_r, out_unsigned=bool(out_u8))

    d = B.ConvDesc(g.N, g.H, g.W, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, g.pad_h, g.pad_w,
                   g.dil_h, g.dil_w, relu=relu)
    packed = B.pack_weights(d, dev(w))
    if in_u8:
        taps, bias = B.u8_prepare(d, dev(w), dev(b))
        tw = w.astype(np.int64).sum(axis=3)                               # [K, R, S]
        # one row per rectangle [r_lo, r_hi) x [s_lo, s_hi) of taps inside the image
        tab = host(taps).reshape(g.R + 1, g.R + 1, g.S + 1, g.S + 1, g.K)
        for r_lo, r_hi, s_lo, s_hi in [(0, g.R, 0, g.S), (1, g.R, 0, g.S), (0, g.R - 1, 0, g.S - 1),
                                       (0, 1, 0, 1), (g.R, 0, 0, g.S), (0, 0, 0, 0)]:
            inside = tw[:, r_lo:r_hi, s_lo:s_hi].sum(axis=(1, 2)) if r_hi > r_lo and s_hi > s_lo else 0
            assert np.array_equal(tab[r_lo, r_hi, s_lo, s_hi], b + 128 * inside)
        assert np.array_equal(host(bias), b + 128 * tw.sum(axis=(1, 2)))
    else:
        taps, bias = None, dev(b)
    dump = torch.zeros((g.N, Ho, Wo, g.K), dtype=torch.int32, device="cuda")
    for use_dump in (True, False):             # general epilogue, then the fast one
        got = B.conv_u8(d, in_u8, out_u8, res_kind == "u8", dev(x_st), packed, bias, taps,
                        float(q_x), float(q_w), float(q_out),
                        None if res_st is None else dev(res_st), float(q_res),
                        acc_dump=dump if use_dump else None)
        if use_dump:
            assert np.array_equal(host(dump), acc_o), "int32 accumulators differ"
        got = host(got)
        if out_u8:
            assert np.array_equal(got.astype(np.int16) + 128, want.astype(np.int16))
        else:
            assert np.array_equal(got, want)
    sat = np.mean((want == (255 if out_u8 else 127)))
    assert sat < 0.5


# ------------------------------------------------------------------ per-channel weights
def test_per_channel_weight_preparation(B):
    rng = np.random.default_rng(91)
    K = 70
    W = (rng.standard_normal((K, 3, 3, 16)) * rng.uniform(0.01, 3.0, K)[:, None, None, None])
    W = W.astype(np.float32)
    W[5] = 0                                            # an all-zero filter
    b = rng.standard_normal(K).astype(np.float32)
    z_o, q_o = orc.quantize_weights_pc(W)
    q_g, z_g = B.quantize_weights_per_channel(dev(W))
    assert np.array_equal(host(q_g), q_o) and np.array_equal(host(z_g), z_o)
    q_x, q_out = np.float32(0.0231), np.float32(0.177)
    assert np.array_equal(host(B.quantize_bias_per_channel(dev(b), float(q_x), q_g)),
                          orc.Q31_bias_pc(b, q_x, q_o))
    assert np.array_equal(host(B.requant_scales(float(q_x), q_g, float(q_out))),
                          orc.requant_scales_pc(q_x, q_o, q_out))


@pytest.mark.parametrize("geom,with_res", [
    (dict(N=2, H=14, W=14, C=64, K=160, R=3, S=3, pad_h=1, pad_w=1), True),
    (dict(N=2, H=28, W=28, C=64, K=128, R=1, S=1), False),
    (dict(N=1, H=17, W=17, C=48, K=72, R=1, S=7, pad_w=3), True),
    (dict(N=2, H=30, W=30, C=3, K=64, R=3, S=3, in_c_stride=4), False),     # unpadded image
])
def test_conv_per_channel_scales(B, geom, with_res):
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(g.K + g.C)
    Cs = g.in_c_stride or g.C
    x = rng.integers(-128, 128, (g.N, g.H, g.W, Cs)).astype(np.int8)
    w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
    b = rng.integers(-20000, 20000, g.K).astype(np.int32)
    acc_o = orc.conv_i8(g, x, w, b)
    base = 40.0 / (5476.0 * np.sqrt(g.R * g.S * g.C))
    m = (base * rng.uniform(0.3, 3.0, g.K)).astype(np.float32)
    res = rng.integers(-128, 128, acc_o.shape).astype(np.int8) if with_res else None
    m_r = np.float32(0.3)
    want = orc.requant_pc(acc_o, m, True, res, m_r)
    d = B.ConvDesc(g.N, g.H, g.W, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, g.pad_h, g.pad_w,
                   g.dil_h, g.dil_w, relu=1, in_c_stride=Cs)
    packed = B.pack_weights(d, dev(w))
    dump = torch.zeros(acc_o.shape, dtype=torch.int32, device="cuda")
    for use_dump in (True, False):             # general epilogue, then the fast one
        got = B.conv_int8_per_channel(d, dev(x), packed, dev(b), dev(m), 1.0,
                                      None if res is None else dev(res), float(m_r),
                                      acc_dump=dump if use_dump else None)
        if use_dump:
            assert np.array_equal(host(dump), acc_o)
        assert np.array_equal(host(got), want)


def _random_geometries(seed, count):
    """Seeded small geometries with everything unequal: strides, pads, dilations, odd extents,
    K and C off the tile sizes."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        g = dict(N=int(rng.integers(1, 4)), H=int(rng.integers(5, 24)), W=int(rng.integers(5, 24)),
                 C=16 * int(rng.integers(1, 7)), K=int(rng.integers(1, 200)), R=R, S=S,
                 stride_h=int(rng.integers(1, 4)), stride_w=int(rng.integers(1, 4)),
                 pad_h=int(rng.integers(0, R)), pad_w=int(rng.integers(0, S)),
                 dil_h=int(rng.integers(1, 3)), dil_w=int(rng.integers(1, 3)))
        geom = orc.ConvGeom(**g)
        if geom.Ho >= 1 and geom.Wo >= 1:
            out.append(g)
    return out


@pytest.mark.parametrize("geom", _random_geometries(1805, 24))
def test_conv_random_geometries(B, geom):
    """int32 accumulators and int8 outputs for seeded random geometries, signed and (where
    the extended build takes the shape) with unsigned input codes."""
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(g.K * 31 + g.C + g.H)
    x = rng.integers(-128, 128, (g.N, g.H, g.W, g.C)).astype(np.int8)
    w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
    b = rng.integers(-20000, 20000, g.K).astype(np.int32)
    res = rng.integers(-128, 128, (g.N, g.Ho, g.Wo, g.K)).astype(np.int8)
    q_x, q_w = np.float32(0.021), np.float32(0.0017)
    q_out = np.float32(q_x * q_w * 5476.0 * np.sqrt(g.R * g.S * g.C) / 40.0)
    q_res = np.float32(0.3) * q_out
    d = B.ConvDesc(g.N, g.H, g.W, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, g.pad_h, g.pad_w,
                   g.dil_h, g.dil_w, relu=1)
    packed = B.pack_weights(d, dev(w))
    m, m_r = orc.requant_scale(q_x, q_w, q_out), orc.residual_scale(q_res, q_out)
    acc_o = orc.conv_i8(g, x, w, b)
    want = orc.requant(acc_o, m, True, res, m_r)
    dump = torch.zeros((g.N, g.Ho, g.Wo, g.K), dtype=torch.int32, device="cuda")
    for use_dump in (True, False):
        got = B.conv_int8(d, dev(x), packed, dev(b), float(q_x), float(q_w), float(q_out), dev(res),
                          float(q_res), acc_dump=dump if use_dump else None)
        if use_dump:
            assert np.array_equal(host(dump), acc_o)
        assert np.array_equal(host(got), want)
    if g.K > 32 and g.R * g.S <= 32:          # unsigned input codes, border start table
        xu = rng.integers(0, 256, (g.N, g.H, g.W, g.C)).astype(np.uint8)
        acc_u = orc.conv_u8(g, xu, w, b)
        want_u = orc.requant_mixed(acc_u, m, True, res, m_r, out_unsigned=True)
        taps, bias = B.u8_prepare(d, dev(w), dev(b))
        got = B.conv_u8(d, 1, 1, 0, dev(_stored(xu)), packed, bias, taps, float(q_x), float(q_w),
                        float(q_out), dev(res), float(q_res), acc_dump=dump)
        assert np.array_equal(host(dump), acc_u)
        assert np.array_equal(host(got).astype(np.int16) + 128, want_u.astype(np.int16))


PAIR_CASES = [
    # first layer, K2, residual, ReLU of the second layer
    (dict(N=2, H=14, W=14, C=64, K=64, R=3, S=3, pad_h=1, pad_w=1), 256, True, True),
    (dict(N=3, H=13, W=11, C=64, K=64, R=3, S=3, pad_h=1, pad_w=1), 128, False, True),   # ragged pixels
    (dict(N=2, H=28, W=28, C=128, K=128, R=3, S=3, pad_h=1, pad_w=1), 512, True, True),
    (dict(N=1, H=9, W=7, C=128, K=128, R=3, S=3, pad_h=1, pad_w=1), 128, True, False),
    (dict(N=2, H=20, W=20, C=64, K=64, R=1, S=1), 64, False, False),                      # 1x1 -> 1x1
    (dict(N=1, H=31, W=31, C=192, K=128, R=3, S=3, stride_h=2, stride_w=2), 384, False, True),
]


@pytest.mark.parametrize("geom,K2,with_res,relu2", PAIR_CASES)
def test_conv_pair_equals_two_layers(B, geom, K2, with_res, relu2):
    """The fused 3x3 -> 1x1 launch gives the bits of the oracle's two layers."""
    g1 = orc.ConvGeom(**geom)
    rng = np.random.default_rng(g1.K + K2 + g1.H)
    x = rng.integers(-128, 128, (g1.N, g1.H, g1.W, g1.C)).astype(np.int8)
    w1 = rng.integers(-128, 128, (g1.K, g1.R, g1.S, g1.C)).astype(np.int8)
    b1 = rng.integers(-20000, 20000, g1.K).astype(np.int32)
    Ho, Wo = g1.Ho, g1.Wo
    g2 = orc.ConvGeom(N=g1.N, H=Ho, W=Wo, C=g1.K, K=K2, R=1, S=1)
    w2 = rng.integers(-128, 128, (K2, 1, 1, g1.K)).astype(np.int8)
    b2 = rng.integers(-20000, 20000, K2).astype(np.int32)
    q_x, q_w1, q_w2 = np.float32(0.021), np.float32(0.0017), np.float32(0.0023)
    q_mid = np.float32(q_x * q_w1 * 5476.0 * np.sqrt(g1.R * g1.S * g1.C) / 40.0)
    q_out = np.float32(q_mid * q_w2 * 3000.0 * np.sqrt(g1.K) / 40.0)
    q_res = np.float32(0.4) * q_out
    res = rng.integers(-128, 128, (g1.N, Ho, Wo, K2)).astype(np.int8) if with_res else None
    mid = orc.requant(orc.conv_i8(g1, x, w1, b1), orc.requant_scale(q_x, q_w1, q_mid), True)
    want = orc.requant(orc.conv_i8(g2, mid, w2, b2), orc.requant_scale(q_mid, q_w2, q_out), relu2,
                       res, orc.residual_scale(q_res, q_out) if with_res else 0.0)
    assert 0.02 < np.mean(mid != 0) and np.mean(np.abs(want.astype(int)) >= 127) < 0.5

    d1 = B.ConvDesc(g1.N, g1.H, g1.W, g1.C, g1.K, g1.R, g1.S, g1.stride_h, g1.stride_w, g1.pad_h,
                    g1.pad_w, relu=1)
    d2 = B.ConvDesc(g1.N, Ho, Wo, g1.K, K2, 1, 1, relu=int(relu2))
    assert B.conv_pair_supported(d1, d2)
    got = B.conv_pair_int8(d1, dev(x), B.pack_weights(d1, dev(w1)), dev(b1), float(q_x), float(q_w1),
                           float(q_mid), d2, B.pack_weights(d2, dev(w2)), dev(b2), float(q_w2),
                           float(q_out), None if res is None else dev(res), float(q_res))
    assert np.array_equal(host(got), want)
    # and the two launches it replaces give the same
    mid_g = B.conv_int8(d1, dev(x), B.pack_weights(d1, dev(w1)), dev(b1), float(q_x), float(q_w1),
                        float(q_mid))
    two = B.conv_int8(d2, mid_g, B.pack_weights(d2, dev(w2)), dev(b2), float(q_mid), float(q_w2),
                      float(q_out), None if res is None else dev(res), float(q_res))
    assert np.array_equal(host(two), want)


REAL_OUTPUT_CASES = [
    # geometry, residual, ReLU, extra channels of the output tensor, channel offset
    (dict(N=2, H=14, W=14, C=64, K=160, R=3, S=3, pad_h=1, pad_w=1), True, True, 0, 0),
    (dict(N=2, H=7, W=7, C=512, K=256, R=1, S=1), True, True, 0, 0),          # complete tiles
    (dict(N=1, H=19, W=19, C=64, K=84, R=3, S=3, pad_h=1, pad_w=1), False, False, 0, 0),  # SSD head
    (dict(N=1, H=17, W=17, C=48, K=72, R=1, S=7, pad_w=3), False, True, 12, 4),
    (dict(N=2, H=9, W=9, C=16, K=17, R=3, S=3, pad_h=1, pad_w=1), True, False, 5, 3),  # K <= 32: a channel tile mostly beyond K
    (dict(N=64, H=1, W=1, C=2048, K=1000, R=1, S=1), False, False, 0, 0),     # classifier logits
    (dict(N=0, H=5, W=5, C=16, K=16, R=1, S=1), False, False, 0, 0),
]


@pytest.mark.parametrize("geom,with_res,relu,out_pad,out_off", REAL_OUTPUT_CASES)
def test_conv_real_valued_output(B, geom, with_res, relu, out_pad, out_off):
    """A layer that leaves the quantised domain writes fp32 directly: the same bits as the
    oracle's fixed fp32 sequence (well inside the 1e-5 relative bound)."""
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(g.K * 7 + g.C)
    x = rng.integers(-128, 128, (g.N, g.H, g.W, g.C)).astype(np.int8)
    w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
    b = rng.integers(-20000, 20000, g.K).astype(np.int32)
    q_x, q_w, q_res = np.float32(0.021), np.float32(0.0017), np.float32(0.083)
    Ho, Wo = g.Ho, g.Wo
    res = rng.integers(-128, 128, (g.N, Ho, Wo, g.K)).astype(np.int8) if with_res else None
    out_cs = g.K + out_pad
    want = np.full((g.N, Ho, Wo, out_cs), np.float32(-7.5))
    if g.N:
        acc_o = orc.conv_i8(g, x, w, b)
        orc.real_output(acc_o, q_x, q_w, relu, res, q_res, out=want, out_c_stride=out_cs,
                        out_c_off=out_off)
    d = B.ConvDesc(g.N, g.H, g.W, g.C, g.K, g.R, g.S, g.stride_h, g.stride_w, g.pad_h, g.pad_w,
                   g.dil_h, g.dil_w, relu=int(relu), out_c_stride=out_cs, out_c_off=out_off)
    out = torch.full((g.N, Ho, Wo, out_cs), -7.5, dtype=torch.float32, device="cuda")
    B.conv_int8_real_output(d, dev(x), B.pack_weights(d, dev(w)), dev(b), float(q_x), float(q_w),
                            None if res is None else dev(res), float(q_res), out=out)
    got = host(out)
    assert np.array_equal(got, want)
    if g.N:
        # and it is the value the int8 tail would have quantised: D(Q(y')) is within q/2 of it
        q_out = np.float32(np.abs(want[..., out_off:out_off + g.K]).max() / 127)
        z = orc.requant(acc_o, orc.requant_scale(q_x, q_w, q_out), relu, res,
                        orc.residual_scale(q_res, q_out) if with_res else 0.0)
        err = np.abs(orc.D(z, q_out) - want[..., out_off:out_off + g.K])
        assert err.max() <= 0.5001 * q_out


@pytest.mark.parametrize("xv,wv", [(-128, -128), (127, -128), (-128, 127), (0, 0)])
def test_conv_extreme_and_degenerate_values(B, xv, wv):
    """Constant tensors at the ends of the int8 range with the longest reduction of the
    benchmark networks (R*S*C = 4608): accumulators of +-7.5e7, beyond 2^24, so the int32 ->
    fp32 conversion of the epilogue rounds; and all-zero operands (the output is the bias)."""
    g = orc.ConvGeom(N=1, H=9, W=9, C=512, K=80, R=3, S=3, pad_h=1, pad_w=1)
    x = np.full((1, 9, 9, 512), xv, np.int8)
    w = np.full((80, 3, 3, 512), wv, np.int8)
    b = (np.arange(80, dtype=np.int32) - 40) * 1001
    acc_o = orc.conv_i8(g, x, w, b)
    if xv and wv:
        assert np.abs(acc_o).max() > 2**24
    q_x, q_w = np.float32(0.013), np.float32(0.0021)
    q_out = np.float32(float(q_x) * float(q_w) * max(float(np.abs(acc_o).max()), 1.0) / 100.0)
    want = orc.requant(acc_o, orc.requant_scale(q_x, q_w, q_out), False)
    d = B.ConvDesc(1, 9, 9, 512, 80, 3, 3, pad_h=1, pad_w=1)
    dump = torch.zeros(acc_o.shape, dtype=torch.int32, device="cuda")
    got = B.conv_int8(d, dev(x), B.pack_weights(d, dev(w)), dev(b), float(q_x), float(q_w),
                      float(q_out), acc_dump=dump)
    assert np.array_equal(host(dump), acc_o)
    assert np.array_equal(host(got), want)
    got = B.conv_int8(d, dev(x), B.pack_weights(d, dev(w)), dev(b), float(q_x), float(q_w),
                      float(q_out))                      # the fast epilogue
    assert np.array_equal(host(got), want)


def test_conv_near_the_32_bit_offset_limit(B):
    """An activation tensor of just under 2 GiB (the kernels' 32-bit offsets end there): a
    3x3 layer over it, checked on sampled output pixels (first, last, image borders, random)
    whose 3x3 neighbourhoods the oracle convolves one by one."""
    N, H, W, C, K = 8, 2044, 2044, 64, 64
    assert 2**31 - 2**24 < N * H * W * C < 2**31
    gen = torch.Generator(device="cuda").manual_seed(1805)
    x = torch.randint(-128, 128, (N, H, W, C), dtype=torch.int8, device="cuda", generator=gen)
    rng = np.random.default_rng(8691)
    w = rng.integers(-128, 128, (K, 3, 3, C)).astype(np.int8)
    b = rng.integers(-20000, 20000, K).astype(np.int32)
    q_x, q_w = np.float32(0.021), np.float32(0.0017)
    q_out = np.float32(q_x * q_w * 5476.0 * np.sqrt(9 * C) / 40.0)
    d = B.ConvDesc(N, H, W, C, K, 3, 3, pad_h=1, pad_w=1, relu=1)
    y = B.conv_int8(d, x, B.pack_weights(d, dev(w)), dev(b), float(q_x), float(q_w), float(q_out))
    picks = [(0, 0, 0), (N - 1, H - 1, W - 1), (N - 1, H - 1, 0), (N - 1, 0, W - 1), (3, 1000, 0),
             (7, 2043, 1022)]
    picks += [tuple(int(v) for v in (rng.integers(0, N), rng.integers(0, H), rng.integers(0, W)))
              for _ in range(58)]
    # the 3x3 neighbourhood of each picked pixel, zeros outside the image
    nb = np.zeros((len(picks), 3, 3, C), np.int8)
    for i, (n, h, ww) in enumerate(picks):
        for r in range(3):
            for s2 in range(3):
                hi, wi = h - 1 + r, ww - 1 + s2
                if 0 <= hi < H and 0 <= wi < W:
                    nb[i, r, s2] = host(x[n, hi, wi])
    g1 = orc.ConvGeom(N=len(picks), H=3, W=3, C=C, K=K, R=3, S=3)
    want = orc.requant(orc.conv_i8(g1, nb, w, b), orc.requant_scale(q_x, q_w, q_out), True)
    got = np.stack([host(y[n, h, ww]) for n, h, ww in picks])
    assert np.array_equal(got, want.reshape(len(picks), K))
    assert len(np.unique(want)) > 32


@pytest.mark.parametrize("out_pad,out_off", [(16, 0), (16, 16), (36, 4), (7, 3)])
def test_conv_channel_slice_of_concat(B, out_pad, out_off):
    geom = dict(N=2, H=9, W=9, C=32, K=40, R=3, S=3, pad_h=1, pad_w=1)
    _run_conv_case(B, geom, relu=True, with_res=False, with_bias=True, seed=5,
                   out_pad=out_pad, out_off=out_off)


def test_conv_input_channel_stride(B):
    # a conv that reads the first 32 channels of a 48-channel tensor
    rng = np.random.default_rng(3)
    g = orc.ConvGeom(N=2, H=10, W=10, C=32, K=32, R=3, S=3, pad_h=1, pad_w=1, in_c_stride=48)
    x = rng.integers(-128, 128, (2, 10, 10, 48)).astype(np.int8)
    w = rng.integers(-128, 128, (32, 3, 3, 32)).astype(np.int8)
    acc_o = orc.conv_i8(g, x, w)
    d = B.ConvDesc(2, 10, 10, 32, 32, 3, 3, pad_h=1, pad_w=1, in_c_stride=48)
    dump = torch.zeros((2, 10, 10, 32), dtype=torch.int32, device="cuda")
    B.conv_int8(d, dev(x), B.pack_weights(d, dev(w)), None, 1.0, 1.0, 1000.0, acc_dump=dump)
    assert np.array_equal(host(dump), acc_o)


def test_conv_batch_elements_are_independent(B):
    rng = np.random.default_rng(4)
    x = rng.integers(-128, 128, (5, 14, 14, 64)).astype(np.int8)
    w = rng.integers(-128, 128, (64, 3, 3, 64)).astype(np.int8)
    d5 = B.ConvDesc(5, 14, 14, 64, 64, 3, 3, pad_h=1, pad_w=1, relu=1)
    d1 = B.ConvDesc(1, 14, 14, 64, 64, 3, 3, pad_h=1, pad_w=1, relu=1)
    wp = B.pack_weights(d5, dev(w))
    full = host(B.conv_int8(d5, dev(x), wp, None, 0.02, 0.002, 0.08))
    for i in (0, 2, 4):
        one = host(B.conv_int8(d1, dev(x[i:i + 1]), wp, None, 0.02, 0.002, 0.08))
        assert np.array_equal(one[0], full[i])


@pytest.mark.parametrize("shape,win", [((2, 23, 23, 64), (3, 2, 1)), ((1, 10, 9, 48), (2, 2, 0)),
                                       ((2, 11, 11, 6), (3, 2, 1)), ((1, 19, 19, 32), (3, 1, 1))])
def test_maxpool_helper(B, shape, win):
    R, stride, pad = win
    rng = np.random.default_rng(sum(shape))
    x = rng.integers(-128, 128, shape).astype(np.int8)
    Ho = (shape[1] + 2 * pad - R) // stride + 1
    Wo = (shape[2] + 2 * pad - R) // stride + 1
    got = host(B.maxpool_i8(dev(x), R, R, stride, pad, Ho, Wo))
    assert np.array_equal(got, orc.maxpool_i8(x, R, R, stride, pad, Ho, Wo))


# ------------------------------------------------------------------ whole configurations
@pytest.mark.parametrize("mode", ["max", "avg"])
@pytest.mark.parametrize("shape,win,m,slice_", [
    ((2, 35, 35, 192), (3, 1, 1), 1.0, (0, 0)),        # Inception pooled branch
    ((1, 17, 17, 768), (3, 2, 0), 0.73, (1280, 512)),  # into a concatenation, rescaled
    ((2, 9, 10, 20), (2, 2, 0), 1.9, (23, 3)),         # odd widths, saturating scale
    ((1, 8, 8, 3), (8, 8, 0), 1.0, (0, 0)),            # whole-image window
    ((1, 19, 19, 64), (3, 1, 1), 0.5, (64, 0)),        # ties of .5 after the scale
])
def test_pool_i8(B, mode, shape, win, m, slice_):
    rng = np.random.default_rng(sum(shape) + win[0])
    x = rng.integers(-128, 128, size=shape, dtype=np.int8)
    R, stride, pad = win
    Ho = (shape[1] + 2 * pad - R) // stride + 1
    Wo = (shape[2] + 2 * pad - R) // stride + 1
    Cd, off = slice_
    Cd = Cd or shape[3]
    base = rng.integers(-128, 128, size=(shape[0], Ho, Wo, Cd), dtype=np.int8)
    # the library forms the rescale itself from the two factors, one fp32 division
    q_out = np.float32(0.0071)
    q_in = np.float32(m) * q_out
    m_used = orc.residual_scale(q_in, q_out)
    assert abs(float(m_used) - m) <= 1e-6 * m
    want = orc.pool_i8(x, mode, R, R, stride, pad, Ho, Wo, m_used, out=base.copy(), out_c_off=off)
    got = B.pool_i8(dev(x), mode, R, R, stride, pad, Ho, Wo, float(q_in), float(q_out),
                    out=dev(base), out_c_off=off)
    assert np.array_equal(host(got), want)


def test_pool_f32(B):
    import torch
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 17, 15, 24)).astype(np.float32)
    xt = torch.from_numpy(x).permute(0, 3, 1, 2)
    for mode, ref in (("max", torch.nn.functional.max_pool2d(xt, 3, 2, 1)),
                      ("avg", torch.nn.functional.avg_pool2d(xt, 3, 2, 1, count_include_pad=True))):
        got = host(B.pool_f32(dev(x), mode, 3, 3, 2, 1, 9, 8))
        want = ref.permute(0, 2, 3, 1).numpy()
        assert np.allclose(got, want, rtol=1e-6, atol=1e-6), mode


def _oracle_pipeline(cfg_id, batch, calib_library):
    cfg = wl.CONFIGS[cfg_id]
    net = cfg["make"]()
    params = {op.name: wl.conv_params(cfg_id, i, op) for i, op in enumerate(net.convs())}
    x = wl.input_batch(cfg_id, net, batch, 0, relu=cfg["relu_input"])
    folded = onet.fold_all(net, params)
    q = onet.calibrate(net, folded, [x], use_library=calib_library)
    qparams = onet.quantize_params(net, folded, q)
    z_in = orc.Q(x, q[net.input], 7)
    acts, accs = onet.forward_i8(net, qparams, q, z_in, keep_acc=True)
    return net, params, x, folded, q, qparams, z_in, acts, accs


def _gpu_pipeline_checks(B, cfg_id, batch, calib_library):
    from paper_1805_08691_amd.engine import Engine
    net, params, x, folded, q, qparams, z_in, acts, accs = _oracle_pipeline(
        cfg_id, batch, calib_library)
    eng = Engine(net, batch)
    eng.load_params(params)
    eng.fold()
    for name, (Wf, bf) in folded.items():          # Eq. BN: bit-exact
        assert np.array_equal(host(eng.folded[name][0]), Wf)
        assert np.array_equal(host(eng.folded[name][1]), bf)
    eng.set_factors(q)                             # frozen factor table from the oracle side
    eng.quantize_weights()
    for name, qp in qparams.items():               # q_w, int8 filters, int32 bias: bit-exact
        assert np.float32(eng.qw[name]) == qp["q_w"]
        assert np.array_equal(host(eng.zw_dense[name]), qp["z_w"])
        assert np.array_equal(host(eng.wq[name][1]), qp["z_b"])
    eng.allocate()
    xd = dev(x)
    slot = torch.zeros(1, device="cuda")           # the input factor from the GPU's own max-abs
    B.calibrate_maxabs(xd, slot)
    assert np.float32(B.qfactor(float(host(slot)[0]), 7)) == q[net.input]
    eng.quantize_input(xd)
    assert np.array_equal(host(eng.act[net.input]), z_in)
    dumps = {op.name: torch.zeros((batch, net.tensors[op.dst].H, net.tensors[op.dst].W, op.K),
                                  dtype=torch.int32, device="cuda") for op in net.convs()}
    eng.run_layers(acc_dump=dumps)
    for op in net.convs():
        assert np.array_equal(host(dumps[op.name]), accs[op.name]), op.name
        assert np.array_equal(host(eng.act[op.dst]), acts[op.dst]), op.name
    for o in net.outputs:                          # Eq. D on what leaves the int8 domain
        r = host(B.dequantize(eng.act[o], float(q[o])))
        want = orc.D(acts[o], q[o])
        assert np.all(np.abs(r - want) <= 1e-5 * np.abs(want))
        assert len(np.unique(acts[o])) > 32        # not degenerate
    return eng, net, xd, acts


def test_config1_single_conv(B):
    _gpu_pipeline_checks(B, 1, 1, calib_library=False)


def test_config2_bottleneck_block(B):
    eng, net, xd, acts = _gpu_pipeline_checks(B, 2, 32, calib_library=True)
    # the same through a captured HIP graph, replayed with eager work in between
    eng.capture(xd)
    for _ in range(3):
        for t in eng.act.values():
            if t is not eng.act[net.input]:
                t.fill_(55)
        torch.cuda.synchronize()
        eng.graph.replay()
        for o in net.outputs:
            assert np.array_equal(host(eng.act[o]), acts[o])


def test_run_step_one_and_two_pipelines_and_serial(B):
    """The step the benchmark times (quantise, layers, dequantise) gives the oracle's values
    whether the batch runs whole, as two concurrent half-batch pipelines, or as the same
    launches one pipeline after the other; an odd batch splits unevenly."""
    from paper_1805_08691_amd.engine import Engine
    cfg_id, batch = 2, 7
    net, params, x, folded, q, qparams, z_in, acts, accs = _oracle_pipeline(cfg_id, batch, True)
    o = net.outputs[0]
    want = orc.D(acts[o], q[o])
    for n_streams, serial, fuse_deq in ((1, False, False), (2, False, False), (2, True, False),
                                        (3, False, False), (2, False, True), (1, False, True)):
        eng = Engine(net, batch, n_streams=n_streams, fuse_dequant=fuse_deq)
        eng.load_params(params)
        eng.fold()
        eng.set_factors(q)
        eng.quantize_weights()
        eng.allocate()
        if n_streams == 2:
            assert eng.parts == [(0, 4), (4, 3)]
        if n_streams == 3:
            assert eng.parts == [(0, 3), (3, 2), (5, 2)]
        out = torch.full(eng.act[o].shape, -1.0, dtype=torch.float32, device="cuda")
        eng.run_step(dev(x), {o: out}, serial=serial)
        torch.cuda.synchronize()
        assert np.array_equal(host(eng.act[o]), acts[o]), (n_streams, serial)
        assert bool(eng._dequant_writer(o)) == fuse_deq
        got = host(out)
        assert np.all(np.abs(got - want) <= 1e-5 * np.abs(want)), (n_streams, serial, fuse_deq)
        assert np.array_equal(got, host(eng.dequantize(o)))       # fused or not: the same bits


def _sampled_images_check(B, cfg_id, batch, picks, n_cal, cal_batch, n_streams=2, unsigned=False,
                          per_channel=False, real_outputs=False, own_sum_factor=False,
                          fuse_pairs=False, chain=False, chain_variants=None, fuse_duals=False,
                          fuse_head=False):
    """Whole network at ``batch`` in the launch configuration the benchmark times; the
    oracle evaluates the images in ``picks`` (batch elements are independent once the
    factor table is frozen) and every tensor of the chain is compared bit for bit."""
    from paper_1805_08691_amd.engine import Engine
    net = wl.CONFIGS[cfg_id]["make"]()
    params = {op.name: wl.conv_params(cfg_id, i, op) for i, op in enumerate(net.convs())}
    folded = onet.fold_all(net, params)
    U = onet.unsigned_tensors(net) if unsigned else set()
    q = onet.calibrate(net, folded, (wl.input_batch(cfg_id, net, cal_batch, 100 + i)
                                     for i in range(n_cal)), unsigned=U,
                       own_sum_factor=own_sum_factor)
    qparams = onet.quantize_params(net, folded, q, per_channel=per_channel)
    x = wl.input_batch(cfg_id, net, batch, 0)
    z_in = orc.Q(x[picks], q[net.input], 7)
    plain = not (unsigned or per_channel or real_outputs or own_sum_factor)
    if plain:
        acts, accs = onet.forward_i8(net, qparams, q, z_in, keep_acc=True)
    else:
        acts = onet.forward_i8(net, qparams, q, z_in, unsigned=U)

    def codes(name, a):       # the GPU's bytes as the oracle's codes
        return (a.astype(np.int16) + 128).astype(np.uint8) if name in U else a

    eng = Engine(net, batch, n_streams=n_streams, unsigned_activations=unsigned,
                 per_channel_weights=per_channel, real_outputs=real_outputs,
                 fuse_pairs=fuse_pairs, chain=chain, fuse_duals=fuse_duals, fuse_head=fuse_head)
    assert bool(eng.head) == fuse_head
    assert bool(eng.duals) == fuse_duals
    assert eng.unsigned == U
    assert bool(eng.pairs) == fuse_pairs
    unwritten = {op.dst for op in net.convs() if op.name in eng.pairs}   # stay on chip
    if eng.head and eng.head[1]:
        unwritten.add(eng.head[0].dst)       # pooled inside the first layer's launch
    # outputs that leave the quantised domain as fp32 straight from their convolution
    real_want = {}
    if real_outputs:
        assert eng.real, "this network has no output a convolution writes whole"
        for op in net.convs():
            if op.dst in eng.real:
                qp = qparams[op.name]
                acc = orc.conv_i8(onet.geom(op, net.tensors, len(picks)), acts[op.src], qp["z_w"],
                                  qp["z_b"])
                real_want[op.dst] = orc.real_output(
                    acc, q[op.src], qp["q_w"], op.relu, acts[op.res] if op.res else None,
                    q[op.res] if op.res else 0.0)
    eng.load_params(params)
    eng.fold()
    eng.set_factors(q)
    eng.quantize_weights()
    for name, qp in qparams.items():
        if per_channel:
            assert np.array_equal(host(eng.qw[name]), qp["q_w"]), name
        else:
            assert np.float32(eng.qw[name]) == qp["q_w"], name
        bias = host(eng.wq[name][1])
        if name in eng.taps:       # reads unsigned codes: 128 * (filter sum) is folded in
            bias = bias - 128 * qp["z_w"].astype(np.int64).reshape(bias.size, -1).sum(axis=1)
        assert np.array_equal(bias, qp["z_b"]), name
    xd = dev(x)
    if chain:
        eng.allocate()
        chains = eng.build_chains(chain_variants)
        assert chains, "no run of chainable layers in this network"
    outs = eng.forward(xd)
    if chain:
        torch.cuda.synchronize()
        assert [c.status() for _, _, c in eng.chains] == [0] * len(eng.chains)
    if eng.head:
        # the head's launches quantised the image on the way in; the stand-alone Eq. Q (which
        # the small-batch check below starts from) is checked here all the same
        assert not host(eng.act[net.input]).any()
        eng.quantize_input(xd)
    zi = host(eng.input_codes())
    if z_in.shape[-1] == 3:              # an image: stored with a zero fourth channel
        assert np.array_equal(zi[picks][..., :3], z_in) and np.all(zi[..., 3] == 0)
    else:
        assert np.array_equal(zi[picks], z_in)
    if eng.in_frame:                     # the frame around the image holds zeros
        top, left = eng.in_frame[:2]
        full = host(eng.act[net.input])
        assert not full[:, :top].any() and not full[:, top + z_in.shape[1]:].any()
        assert not full[:, :, :left].any() and not full[:, :, left + z_in.shape[2]:].any()
    for op in net.ops:
        if op.dst in eng.real or op.dst in unwritten:
            continue
        got = codes(op.dst, host(eng.act[op.dst])[picks])
        assert got.dtype == acts[op.dst].dtype and np.array_equal(got, acts[op.dst]), op.name
    for o, out in zip(net.outputs, outs):
        r = host(eng.dequantize(o))[picks]
        if o in eng.real:
            assert np.array_equal(r, real_want[o]), o
            # the int8 path's D(Q(.)) of the same value is within half a step of it
            # (where the int8 range holds it)
            inside = np.abs(r) <= 127 * q[o]
            assert np.all(np.abs(orc.D(acts[o], q[o]) - r)[inside] <= 0.5001 * q[o]), o
            continue
        want = orc.D_u8(acts[o], q[o]) if o in U else orc.D(acts[o], q[o])
        assert np.all(np.abs(r - want) <= 1e-5 * np.abs(want)), o
    if plain and not chain:
        # the int32 accumulators of every layer on the sampled images (run as a small batch of
        # their own from the same int8 input codes), against the oracle's
        small = Engine(net, len(picks), fuse_pairs=fuse_pairs)
        small.load_params(params)
        small.fold()
        small.set_factors(q)
        small.quantize_weights()
        small.allocate()
        small.input_codes().copy_(eng.input_codes()[picks])
        dumps = {op.name: torch.zeros((len(picks), net.tensors[op.dst].H, net.tensors[op.dst].W,
                                       op.K), dtype=torch.int32, device="cuda")
                 for op in net.convs()}
        some = {k: v for i, (k, v) in enumerate(dumps.items()) if i % 2 == 0} if fuse_pairs else dumps
        small.run_layers(acc_dump=some)
        for name in some:
            assert np.array_equal(host(dumps[name]), accs[name]), name
        for op in net.ops:
            assert np.array_equal(host(small.act[op.dst]), acts[op.dst]), op.name
        del small, dumps
    # replays of the captured HIP graph, with eager work between them: same bits each time
    eng.capture(xd)
    for rep in range(3):
        for o in net.outputs:
            eng.act[o].fill_(3 + rep)
        torch.cuda.synchronize()
        for o in eng.real:
            eng.act_f32[o].fill_(3 + rep)
        eng.graph.replay()
        for o in net.outputs:
            if o in eng.real:
                assert np.array_equal(host(eng.act_f32[o])[picks], real_want[o]), (o, rep)
            else:
                assert np.array_equal(codes(o, host(eng.act[o])[picks]), acts[o]), (o, rep)


@pytest.mark.parametrize("n_streams", [2, 1])
def test_config3_resnet50_batch64_sampled_images(B, n_streams):
    # n_streams = 2 is the launch configuration the benchmark times (two half-batch
    # pipelines); images 31 and 32 sit on either side of the split
    _sampled_images_check(B, 3, 64, [0, 31, 32, 63], n_cal=8, cal_batch=8, n_streams=n_streams)


def test_resnet50_unsigned_activations(B):
    # ResNet-50 with unsigned p = 8 codes on every ReLU output (the paper's precision for
    # non-negative activations), batch 64 in the benchmark's launch configuration
    _sampled_images_check(B, 3, 64, [0, 31, 32, 63], n_cal=4, cal_batch=8, unsigned=True)


def test_resnet50_per_channel_weights(B):
    _sampled_images_check(B, 3, 64, [0, 31, 32, 63], n_cal=4, cal_batch=8, per_channel=True)


def test_resnet50_after_sparsity_removal(B):
    # the paper's graph transformation of the stride-2 stage entries (config 6): strided
    # 1x1 layers with a residual that a 1x1 stride-2 pooling subsampled
    _sampled_images_check(B, 6, 16, [0, 7, 8, 15], n_cal=2, cal_batch=8)


def test_config4_inception_v3_batch64_sampled_images(B):
    # odd extents (299 -> 149 -> 147 -> 73 -> 71 -> 35 -> 17 -> 8), 1x7 / 7x1 filters,
    # pooled branches, channel-slice writes into concatenations
    _sampled_images_check(B, 4, 64, [0, 21, 63], n_cal=4, cal_batch=8)


@pytest.mark.parametrize("batch,picks", [(1, [0]), (64, [0, 32, 63])])
def test_config5_ssd300_vgg16_sampled_images(B, batch, picks):
    # 3x3 stack at 300x300, ceil-mode pooling, dilation 6, head convolutions with
    # K in {16, 24, 84, 126}, twelve int8 outputs
    _sampled_images_check(B, 5, batch, picks, n_cal=2, cal_batch=4)


def test_resnet50_with_fused_layer_pairs(B):
    # every bottleneck's 3x3 -> 1x1 whose 3x3 has 64 or 128 filters runs as one launch, in
    # the benchmark's launch configuration
    _sampled_images_check(B, 3, 64, [0, 31, 32, 63], n_cal=4, cal_batch=8, fuse_pairs=True)


def test_resnet50_with_fused_head(B):
    # Eq. Q on the image, the 7x7 / 2 layer and the 3x3 / 2 max-pool as one launch per half
    # batch: the launch configuration the benchmark times
    _sampled_images_check(B, 3, 64, [0, 31, 32, 63], n_cal=4, cal_batch=8, fuse_head=True)
    _sampled_images_check(B, 3, 5, [0, 2, 4], n_cal=2, cal_batch=8, fuse_head=True, n_streams=1)


def test_resnet50_with_dual_launches(B):
    # the projection branch and the first 1x1 of each of the four stages as one launch, in the
    # benchmark's launch configuration (two half-batch pipelines), also together with the fused
    # 3x3 -> 1x1 pairs
    _sampled_images_check(B, 3, 64, [0, 31, 32, 63], n_cal=4, cal_batch=8, fuse_duals=True)
    _sampled_images_check(B, 3, 16, [0, 7, 8, 15], n_cal=2, cal_batch=8, fuse_duals=True,
                          fuse_pairs=True)


def test_resnet50_as_one_chained_launch(B):
    # the 52 convolutions behind the first pooling as ONE persistent launch (the batch split
    # over the eight XCDs, tiles started by completion counters); images on both sides of
    # every boundary between two XCDs' shares are among the picks
    _sampled_images_check(B, 3, 64, [0, 7, 8, 31, 32, 55, 56, 63], n_cal=4, cal_batch=8,
                          n_streams=1, chain=True)


@pytest.mark.parametrize("batch", [13, 3])
def test_chained_launch_with_uneven_and_empty_shares(B, batch):
    # 13 images: shares of 2 and 1; 3 images: five XCDs have no work at all
    _sampled_images_check(B, 3, batch, list(range(batch)), n_cal=2, cal_batch=8, n_streams=1,
                          chain=True)


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
def test_chained_launch_with_every_tile_variant(B, variant):
    # the bottleneck block of config 2 with one tile shape forced on all three layers:
    # ragged pixel tiles (25 images: shares of 4 and 3) and the residual dependency
    net = wl.CONFIGS[2]["make"]()
    _sampled_images_check(B, 2, 25, [0, 3, 4, 12, 24], n_cal=1, cal_batch=4, n_streams=1,
                          chain=True, chain_variants={op.name: variant for op in net.convs()})


def test_resnet50_sums_at_their_own_calibrated_factor(B):
    # the variant of the sum rule: q of a fused sum from its own max-abs, not max(q1, q2)
    _sampled_images_check(B, 3, 8, [0, 3, 4, 7], n_cal=2, cal_batch=8, own_sum_factor=True)


def test_networks_with_real_valued_outputs(B):
    # the last convolution (ResNet-50: fused sum + ReLU) and the twelve SSD head
    # convolutions write fp32 directly instead of int8 codes plus a dequantise pass
    _sampled_images_check(B, 3, 8, [0, 3, 4, 7], n_cal=2, cal_batch=8, real_outputs=True)
    _sampled_images_check(B, 5, 1, [0], n_cal=2, cal_batch=4, real_outputs=True)


def test_gpu_calibration_matches_oracle_closely(B):
    # the GPU's own calibration (fp32 forward in a different summation order) gives
    # factors equal to the oracle's up to fp32 rounding of the activations
    from paper_1805_08691_amd.engine import Engine
    cfg_id, batch = 2, 4
    cfg = wl.CONFIGS[cfg_id]
    net = cfg["make"]()
    params = {op.name: wl.conv_params(cfg_id, i, op) for i, op in enumerate(net.convs())}
    xs = [wl.input_batch(cfg_id, net, batch, i, relu=True) for i in range(2)]
    folded = onet.fold_all(net, params)
    q_o = onet.calibrate(net, folded, xs, use_library=False)
    eng = Engine(net, batch)
    eng.load_params(params)
    eng.fold()
    q_g = eng.calibrate([dev(x) for x in xs])
    assert set(q_g) == set(q_o)
    for k in q_o:
        assert abs(q_g[k] - float(q_o[k])) <= 1e-5 * float(q_o[k]), k
