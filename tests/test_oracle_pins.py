"""Pins of the CPU oracle against what the paper's equations and plain mathematics fix.

None of these tests needs a GPU and none compares the oracle with itself: expected
values are hand-worked from Eq. Q / Eq. D / Eq. + / Eq. BN, computed with exact
Python integers and Fractions (tests/exact.py), by brute-force Python loops, or by an
independent library routine (torch float64 convolution / pooling on the CPU).
"""
from fractions import Fraction

import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st

import golden_io
import oracle as orc
from exact import clamp, fl32, fl64, round_half_even

F = Fraction


# ----------------------------------------------------------------------------------------
# Eq. Q: rounding is half-to-even, clamp bounds are -2^p and 2^p - 1
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["unit_factor", "half_factor", "p8_bounds", "p3_bounds",
                                  "calibration"])
def test_Q_handworked(case):
    c = golden_io.load("eq_Q.txt")[case]
    assert orc.Q(c["r"], c["q"], int(c["p"])).tolist() == [int(v) for v in c["z"]]


def test_Q31_bias_bounds_and_values():
    # factor = q_x*q_w = 0.25: b/0.25 = [4, 2, -2 (tie 2.5 -> 2), ...]; +-3e9 saturate.
    z = orc.Q31_bias([1.0, 0.5, -0.625, 0.625, 0.875], 0.5, 0.5)
    assert z.tolist() == [4, 2, -2, 2, 4]
    z = orc.Q31_bias([3e9, -3e9], 1.0, 1.0)
    assert z.tolist() == [2147483647, -2147483648]


def test_Q31_bias_matches_exact_rational_fp64():
    rng = np.random.default_rng(5)
    b = rng.normal(0, 0.1, 64).astype(np.float32)
    q_x, q_w = np.float32(0.0137), np.float32(0.00091)
    got = orc.Q31_bias(b, q_x, q_w)
    q = fl64(F(float(q_x)) * F(float(q_w)))
    want = [clamp(round_half_even(fl64(F(float(v)) / q)), -2**31, 2**31 - 1) for v in b]
    assert got.tolist() == want


def test_calibration_example():
    # max|x| = 2.54, p = 7 -> q = 0.02; the largest element maps to -(2^p - 1)
    x = np.array([0.1, -2.54, 1.0, 2.0], np.float32)
    m = orc.maxabs(x)
    assert m == np.float32(2.54)
    q = orc.qfactor(m, 7)
    assert q == np.float32(2.54) / np.float32(127)
    assert orc.Q(x, q, 7).tolist() == [5, -127, 50, 100]
    assert orc.qfactor(0.0, 7) == np.float32(1.0)       # all-zero tensor reading
    assert orc.maxabs(np.zeros(0, np.float32)) == 0.0
    assert orc.qfactor(255.0, 8) == np.float32(1.0)
    assert orc.qfactor(np.float32(2**31 - 1), 31) == np.float32(1.0)


def test_maxabs_invariants():
    rng = np.random.default_rng(1)
    x = rng.normal(size=4099).astype(np.float32)
    m = orc.maxabs(x)
    assert m == np.abs(x).max()
    assert orc.maxabs(rng.permutation(x)) == m
    assert orc.maxabs(-x) == m
    parts = np.array_split(x, 7)
    assert max(orc.maxabs(p) for p in parts) == m      # running max == max of concat
    q = orc.qfactor(m, 7)
    z = orc.Q(x, q, 7)
    assert abs(int(z[np.argmax(np.abs(x))])) == 127 and np.abs(z.astype(int)).max() == 127


@settings(max_examples=300, deadline=None)
@given(st.floats(min_value=2.0**-20, max_value=2.0**20, width=32),
       st.lists(st.floats(min_value=-1.0, max_value=1.0, width=32), min_size=1, max_size=32),
       st.sampled_from([3, 7, 8]))
def test_DQ_error_bound(q, us, p):
    # Inside the representable range |D(Q(r)) - r| <= q/2, up to the fp32 rounding of r/q.
    q = np.float32(q)
    lim = float(q) * (2**p - 1)
    r = (np.array(us, np.float32) * np.float32(lim)).astype(np.float32)
    r = r[np.abs(r.astype(np.float64)) <= lim]
    if r.size == 0:
        return
    z = orc.Q(r, q, p).astype(np.int64)
    err = np.abs(float(q) * z.astype(np.float64) - r.astype(np.float64))
    assert np.all(err <= float(q) * (0.5 + 2**p * 2.0**-23))
    assert z.max() <= 2**p - 1 and z.min() >= -2**p


def test_Q_matches_exact_rational():
    rng = np.random.default_rng(11)
    r = rng.normal(0, 3, 400).astype(np.float32)
    q = np.float32(0.0371)
    got = orc.Q(r, q, 7).tolist()
    want = [clamp(round_half_even(fl32(F(float(v)) / F(float(q)))), -128, 127) for v in r]
    assert got == want


def test_QD_roundtrip_all_codes():
    z = np.arange(-128, 128).astype(np.int8)
    rng = np.random.default_rng(2)
    for q in [1.0, 0.5, 0.02, 3.0] + list(rng.uniform(1e-3, 10, 20)):
        r = orc.D(z, q)
        assert r.dtype == np.float32
        assert np.array_equal(r, np.float32(q) * z.astype(np.float32))
        assert np.array_equal(orc.Q(r, q, 7), z)


def test_D_handworked():
    assert orc.D(np.array([-128, -1, 0, 3, 127], np.int8), 0.25).tolist() == \
        [-32.0, -0.25, 0.0, 0.75, 31.75]


# ----------------------------------------------------------------------------------------
# Eq. +  (literal) and the fused epilogue
# ----------------------------------------------------------------------------------------
def test_plus_handworked():
    c = golden_io.load("eq_plus.txt")["two_factors"]
    z, q = orc.plus([int(v) for v in c["z1"]], c["q1"], [int(v) for v in c["z2"]], c["q2"])
    assert q == np.float32(c["q"])
    assert z.tolist() == [int(v) for v in c["z"]]
    # adding the zero tensor at a smaller-or-equal factor leaves z unchanged
    a = np.arange(-128, 128).astype(np.int8)
    z, q = orc.plus(a, 0.75, np.zeros_like(a), 0.3)
    assert q == np.float32(0.75) and np.array_equal(z, a.astype(np.int32))
    # commutative
    rng = np.random.default_rng(3)
    b = rng.integers(-128, 128, 256).astype(np.int8)
    z1, _ = orc.plus(a, 0.11, b, 0.07)
    z2, _ = orc.plus(b, 0.07, a, 0.11)
    assert np.array_equal(z1, z2)


def test_requant_handworked():
    c = golden_io.load("eq_Aprime_tail.txt")["half_scale"]
    acc = np.array(c["acc"], np.int32).reshape(1, -1)
    assert orc.requant(acc, c["m"], relu=False).ravel().tolist() == [int(v) for v in c["z"]]
    assert orc.requant(acc, c["m"], relu=True).ravel().tolist() == [int(v) for v in c["z_relu"]]


def test_requant_int32_to_fp32_conversion_is_rne():
    # 2^24+1 is not an fp32 value: ties-to-even gives 2^24; 2^24+3 -> 2^24+4.
    acc = np.array([16777217, 16777219, -16777217, -16777219], np.int32).reshape(1, 4)
    m = np.float32(2.0**-18)
    got = orc.requant(acc, m, relu=False).ravel().tolist()
    want = [round_half_even(F(v) * F(2)**-18) for v in (16777216, 16777220, -16777216, -16777220)]
    assert got == want == [64, 64, -64, -64]
    # a case where the conversion changes the final code: (2^24+2^0)*2^-17 region
    acc = np.array([2**25 + 2, 2**25 + 6], np.int32).reshape(1, 2)   # -> 2^25, 2^25+8
    m = np.float32(2.0**-3)            # exact scaling, clamp hides value -> use windowed test below
    assert orc.requant(acc, m, relu=False).ravel().tolist() == [127, 127]


def _requant_exact(acc, m, relu, z_res=None, m_r=None):
    t = fl32(F(int(acc)))
    t = fl32(t * F(float(m)))
    if z_res is not None:
        u = fl32(F(int(z_res)) * F(float(m_r)))
        t = fl32(t + u)
    if relu and t < 0:
        t = F(0)
    t = clamp(t, F(-128), F(127))
    return round_half_even(t)


def test_requant_sweep_against_exact_rational():
    rng = np.random.default_rng(7)
    for m in [np.float32(0.0123), np.float32(1 / 3), np.float32(2.5e-6), np.float32(0.5)]:
        centre = int(60 / float(m))
        lo = max(centre - 300, -2**31)
        hi = min(centre + 300, 2**31 - 1)
        accs = np.concatenate([np.arange(lo, hi), -np.arange(lo, hi),
                               rng.integers(-2**31, 2**31 - 1, 200)]).astype(np.int32)
        for relu in (False, True):
            got = orc.requant(accs.reshape(-1, 1), m, relu).ravel().tolist()
            want = [_requant_exact(a, m, relu) for a in accs]
            assert got == want


def test_requant_residual_against_exact_rational():
    rng = np.random.default_rng(8)
    acc = rng.integers(-40000, 40000, size=(50, 8)).astype(np.int32)
    res = rng.integers(-128, 128, size=(50, 8)).astype(np.int8)
    m, m_r = np.float32(0.00231), np.float32(0.6180339)
    for relu in (False, True):
        got = orc.requant(acc, m, relu, res, m_r)
        want = [[_requant_exact(acc[i, k], m, relu, res[i, k], m_r) for k in range(8)]
                for i in range(50)]
        assert got.tolist() == want


def test_requant_scales_are_two_fp32_ops():
    q_x, q_w, q_o = np.float32(0.0173), np.float32(0.00219), np.float32(0.0411)
    want = fl32(fl32(F(float(q_x)) * F(float(q_w))) / F(float(q_o)))
    assert F(float(orc.requant_scale(q_x, q_w, q_o))) == want
    want = fl32(F(float(q_x)) / F(float(q_o)))
    assert F(float(orc.residual_scale(q_x, q_o))) == want


def test_requant_channel_slice_addressing():
    rng = np.random.default_rng(9)
    acc = rng.integers(-3000, 3000, size=(6, 5)).astype(np.int32)
    res_wide = rng.integers(-128, 128, size=(6, 16)).astype(np.int8)
    out = np.full((6, 12), 99, np.int8)
    orc.requant(acc, 0.05, True, res_wide, 0.5, res_c_stride=16, res_c_off=3, out=out,
                out_c_stride=12, out_c_off=4)
    dense = orc.requant(acc, 0.05, True, np.ascontiguousarray(res_wide[:, 3:8]), 0.5)
    assert np.array_equal(out[:, 4:9], dense)
    assert np.all(out[:, :4] == 99) and np.all(out[:, 9:] == 99)


def test_fused_sum_vs_literal_two_step_differs_by_at_most_one():
    # Fused: one rounding of (acc*m + res*m_r).  Literal: round the conv to int8 at q1,
    # then apply Eq. + at max(q1, q2).  The arguments of the final Round differ by <= 1/2.
    rng = np.random.default_rng(10)
    acc = rng.integers(-60000, 60000, size=(400, 4)).astype(np.int32)
    res = rng.integers(-128, 128, size=(400, 4)).astype(np.int8)
    q_x, q_w = np.float32(0.02), np.float32(0.003)
    for q1, q2 in [(0.9, 0.7), (0.5, 1.1)]:
        q1, q2 = np.float32(q1), np.float32(q2)
        q_out = max(q1, q2)
        fused = orc.requant(acc, orc.requant_scale(q_x, q_w, q_out), False, res,
                            orc.residual_scale(q2, q_out)).astype(int)
        z1 = orc.requant(acc, orc.requant_scale(q_x, q_w, q1), False)
        lit, q = orc.plus(z1, q1, res, q2)
        assert q == q_out
        assert np.abs(fused - lit).max() <= 1


# ----------------------------------------------------------------------------------------
# Eq. BN
# ----------------------------------------------------------------------------------------
def test_fold_bn_closed_form_and_identity():
    W = np.arange(24, dtype=np.float32).reshape(2, 2, 2, 3) - 7
    b = np.array([1.0, -2.0], np.float32)
    gamma = np.array([3.0, -1.0], np.float32)
    beta = np.array([0.5, 0.25], np.float32)
    mu = np.array([0.5, 1.0], np.float32)
    var = np.array([4.0, 4.0], np.float32)
    Wf, bf = orc.fold_bn(W, b, gamma, beta, mu, var, eps=0.0)   # s = gamma / 2
    assert np.array_equal(Wf[0], 1.5 * W[0]) and np.array_equal(Wf[1], -0.5 * W[1])
    assert bf.tolist() == [1.5 * 0.5 + 0.5, -0.5 * -3.0 + 0.25]
    Wi, bi = orc.fold_bn(W, b, np.ones(2), np.zeros(2), np.zeros(2), np.ones(2), eps=0.0)
    assert np.array_equal(Wi, W) and np.array_equal(bi, b)
    Wn, bn = orc.fold_bn(W, None, gamma, beta, mu, var, eps=0.0)  # missing bias == zero bias
    W0, b0 = orc.fold_bn(W, np.zeros(2), gamma, beta, mu, var, eps=0.0)
    assert np.array_equal(Wn, W0) and np.array_equal(bn, b0)


def test_fold_bn_equals_conv_then_bn_fp64():
    rng = np.random.default_rng(12)
    N, H, Wd, Cc, K, R, S = 2, 6, 5, 3, 4, 3, 3
    x = rng.normal(size=(N, H, Wd, Cc))
    W = rng.normal(size=(K, R, S, Cc)).astype(np.float32)
    b = rng.normal(size=K).astype(np.float32)
    gamma = rng.uniform(.5, 1.5, K).astype(np.float32)
    beta = rng.normal(0, .1, K).astype(np.float32)
    mu = rng.normal(0, .1, K).astype(np.float32)
    var = rng.uniform(.5, 1.5, K).astype(np.float32)
    eps = 1e-5
    Wf, bf = orc.fold_bn(W, b, gamma, beta, mu, var, eps)

    def conv64(w, bias):
        xt = torch.from_numpy(x).permute(0, 3, 1, 2)
        wt = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)
        return torch.nn.functional.conv2d(xt, wt, torch.from_numpy(bias.astype(np.float64)),
                                          padding=1).permute(0, 2, 3, 1).numpy()
    y = conv64(W, b)
    bn = gamma.astype(np.float64) * (y - mu) / np.sqrt(var.astype(np.float64) + eps) + beta
    folded = conv64(Wf, bf)
    assert np.allclose(folded, bn, rtol=1e-5, atol=1e-5)
    # a wrong sign on mu or a dropped beta must fail the line above: check the margin
    assert not np.allclose(conv64(Wf, bf - beta), bn, rtol=1e-5, atol=1e-5)


# ----------------------------------------------------------------------------------------
# x rule: the integer convolution
# ----------------------------------------------------------------------------------------
def _brute_conv(g, x, w, b):
    ics = g.in_c_stride or g.C
    x = x.reshape(g.N, g.H, g.W, ics)
    w = w.reshape(g.K, g.R, g.S, g.C)
    Ho = (g.H + 2 * g.pad_h - g.dil_h * (g.R - 1) - 1) // g.stride_h + 1
    Wo = (g.W + 2 * g.pad_w - g.dil_w * (g.S - 1) - 1) // g.stride_w + 1
    out = [[[[0] * g.K for _ in range(Wo)] for _ in range(Ho)] for _ in range(g.N)]
    for n in range(g.N):
        for ho in range(Ho):
            for wo in range(Wo):
                for k in range(g.K):
                    a = int(b[k]) if b is not None else 0
                    for r in range(g.R):
                        for s in range(g.S):
                            hi = ho * g.stride_h - g.pad_h + r * g.dil_h
                            wi = wo * g.stride_w - g.pad_w + s * g.dil_w
                            if 0 <= hi < g.H and 0 <= wi < g.W:
                                for c in range(g.C):
                                    a += int(x[n, hi, wi, c]) * int(w[k, r, s, c])
                    out[n][ho][wo][k] = a
    return np.array(out, np.int64).reshape(g.N, Ho, Wo, g.K)


def test_conv_toy_handworked():
    # 3x3 single-channel image 1..9, 2x2 filter [[1,0],[0,-1]], no padding:
    # every output is x[i,j] - x[i+1,j+1] = -4.
    g = orc.ConvGeom(N=1, H=3, W=3, C=1, K=1, R=2, S=2)
    x = np.arange(1, 10, dtype=np.int8)
    w = np.array([1, 0, 0, -1], np.int8)
    assert orc.conv_i8(g, x, w).ravel().tolist() == [-4, -4, -4, -4]
    # with bias 10 and padding 1 the corner output sees only the -1 tap on x[0,0]
    g = orc.ConvGeom(N=1, H=3, W=3, C=1, K=1, R=2, S=2, pad_h=1, pad_w=1)
    acc = orc.conv_i8(g, x, w, np.array([10], np.int32))
    assert acc.shape == (1, 4, 4, 1)
    assert acc[0, 0, 0, 0] == 10 - 1 and acc[0, 3, 3, 0] == 10 + 9
    assert acc[0, 1, 1, 0] == 10 + 1 - 5


@pytest.mark.parametrize("geom", [
    dict(N=2, H=5, W=4, C=3, K=2, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=1, H=7, W=6, C=2, K=3, R=3, S=2, stride_h=2, stride_w=1, pad_h=0, pad_w=1),
    dict(N=1, H=9, W=9, C=1, K=2, R=3, S=3, dil_h=2, dil_w=3, pad_h=2, pad_w=3),
    dict(N=2, H=4, W=4, C=4, K=4, R=1, S=1, stride_h=2, stride_w=2),
    dict(N=1, H=5, W=8, C=2, K=1, R=1, S=7, pad_w=3),
    dict(N=1, H=8, W=5, C=2, K=1, R=7, S=1, pad_h=3),
    dict(N=1, H=6, W=6, C=3, K=2, R=3, S=3, pad_h=1, pad_w=1, in_c_stride=5),
])
def test_conv_brute_force_toys(geom):
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(hash(tuple(geom.items())) % 2**32)
    ics = g.in_c_stride or g.C
    x = rng.integers(-128, 128, g.N * g.H * g.W * ics).astype(np.int8)
    w = rng.integers(-128, 128, g.K * g.R * g.S * g.C).astype(np.int8)
    b = rng.integers(-10**6, 10**6, g.K).astype(np.int32)
    assert np.array_equal(orc.conv_i8(g, x, w, b), _brute_conv(g, x, w, b))
    assert np.array_equal(orc.conv_i8(g, x, w, None), _brute_conv(g, x, w, None))


def _torch_conv_int(g, x, w, b):
    xt = torch.from_numpy(x.reshape(g.N, g.H, g.W, g.C).astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(w.reshape(g.K, g.R, g.S, g.C).astype(np.float64)).permute(0, 3, 1, 2)
    bt = None if b is None else torch.from_numpy(b.astype(np.float64))
    y = torch.nn.functional.conv2d(xt, wt, bt, stride=(g.stride_h, g.stride_w),
                                   padding=(g.pad_h, g.pad_w), dilation=(g.dil_h, g.dil_w))
    return y.permute(0, 2, 3, 1).numpy().astype(np.int64)


@pytest.mark.parametrize("geom", [
    dict(N=2, H=14, W=14, C=32, K=24, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=1, H=17, W=17, C=16, K=20, R=1, S=7, pad_w=3),
    dict(N=1, H=17, W=17, C=16, K=20, R=7, S=1, pad_h=3),
    dict(N=1, H=23, W=23, C=3, K=8, R=7, S=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3),
    dict(N=1, H=19, W=19, C=8, K=8, R=3, S=3, dil_h=6, dil_w=6, pad_h=6, pad_w=6),
    dict(N=2, H=10, W=10, C=48, K=64, R=5, S=5, pad_h=2, pad_w=2),
    dict(N=1, H=35, W=35, C=16, K=12, R=3, S=3, stride_h=2, stride_w=2),
    dict(N=3, H=8, W=8, C=64, K=16, R=1, S=1, stride_h=2, stride_w=2),
])
def test_conv_against_float64_library_convolution(geom):
    # sums stay far below 2^53, so the float64 library convolution is exact
    g = orc.ConvGeom(**geom)
    rng = np.random.default_rng(42)
    x = rng.integers(-128, 128, g.N * g.H * g.W * g.C).astype(np.int8)
    w = rng.integers(-128, 128, g.K * g.R * g.S * g.C).astype(np.int8)
    b = rng.integers(-10**5, 10**5, g.K).astype(np.int32)
    acc = orc.conv_i8(g, x, w, b)
    ref = _torch_conv_int(g, x, w, b)
    assert acc.shape == ref.shape
    assert np.array_equal(acc, ref)


def test_conv_1x1_is_matrix_product_and_padding_channels_is_neutral():
    rng = np.random.default_rng(13)
    g = orc.ConvGeom(N=2, H=5, W=5, C=24, K=10, R=1, S=1)
    x = rng.integers(-128, 128, (50, 24)).astype(np.int8)
    w = rng.integers(-128, 128, (10, 24)).astype(np.int8)
    acc = orc.conv_i8(g, x, w)
    assert np.array_equal(acc.reshape(50, 10), x.astype(np.int64) @ w.astype(np.int64).T)
    # zero-padding the channel axis (C -> C+8) leaves the result unchanged
    xp = np.concatenate([x, np.zeros((50, 8), np.int8)], 1)
    wp = np.concatenate([w, rng.integers(-128, 128, (10, 8)).astype(np.int8)], 1)
    g2 = orc.ConvGeom(N=2, H=5, W=5, C=32, K=10, R=1, S=1)
    assert np.array_equal(orc.conv_i8(g2, xp, wp), acc)


def test_conv_overflow_is_reported():
    g = orc.ConvGeom(N=1, H=1, W=1, C=4, K=1, R=1, S=1)
    x = np.full(4, 127, np.int8)
    w = np.full(4, 127, np.int8)
    with pytest.raises(OverflowError):
        orc.conv_i8(g, x, w, np.array([2**31 - 1], np.int32))


def test_output_extent_formula():
    assert (orc.ConvGeom(1, 224, 224, 3, 1, 7, 7, 2, 2, 3, 3).Ho) == 112
    assert (orc.ConvGeom(1, 19, 19, 8, 1, 3, 3, 1, 1, 6, 6, 6, 6).Ho) == 19
    assert (orc.ConvGeom(1, 35, 35, 8, 1, 3, 3, 2, 2).Wo) == 17
    assert (orc.ConvGeom(1, 3, 3, 8, 1, 3, 3).Wo) == 1
    assert (orc.ConvGeom(1, 2, 2, 8, 1, 3, 3).Wo) == 0


# ----------------------------------------------------------------------------------------
# Whole layer, Eq. A' + fused sum, with power-of-two factors: every fp32 step is exact,
# so the result equals the exact-rational value of the paper's formula.
# ----------------------------------------------------------------------------------------
def test_layer_exact_with_power_of_two_factors():
    rng = np.random.default_rng(14)
    g = orc.ConvGeom(N=1, H=6, W=6, C=8, K=5, R=3, S=3, pad_h=1, pad_w=1)
    z_x = rng.integers(-128, 128, (1, 6, 6, 8)).astype(np.int8)
    z_w = rng.integers(-128, 128, (5, 3, 3, 8)).astype(np.int8)
    z_b = rng.integers(-5000, 5000, 5).astype(np.int32)
    z_r = rng.integers(-128, 128, (1, 6, 6, 5)).astype(np.int8)
    q_x, q_w, q_r, q_o = 2.0**-5, 2.0**-9, 2.0**-3, 2.0**-2
    z_y, acc = orc.conv_layer_i8(g, z_x, q_x, z_w, q_w, z_b, q_o, True, z_r, q_r)
    ref_acc = _brute_conv(g, z_x, z_w, z_b)
    assert np.array_equal(acc, ref_acc)
    want = np.empty_like(z_y)
    for idx in np.ndindex(*ref_acc.shape):
        real = F(q_x) * F(q_w) * int(ref_acc[idx]) + F(q_r) * int(z_r[idx])
        real = max(real, F(0))
        want[idx] = clamp(round_half_even(real / F(q_o)), -128, 127)
    assert np.array_equal(z_y, want)
    assert len(np.unique(z_y)) > 20          # the case is not degenerate (all saturated)


# ----------------------------------------------------------------------------------------
# helpers that only chain shapes
# ----------------------------------------------------------------------------------------
def test_conv_f32_against_float64_library():
    rng = np.random.default_rng(15)
    g = orc.ConvGeom(N=2, H=9, W=8, C=5, K=6, R=3, S=3, stride_h=2, stride_w=1, pad_h=1, pad_w=1)
    x = rng.normal(size=(2, 9, 8, 5)).astype(np.float32)
    w = rng.normal(size=(6, 3, 3, 5)).astype(np.float32)
    b = rng.normal(size=6).astype(np.float32)
    y = orc.conv_f32(g, x, w, b, None, relu=True)
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)
    ref = torch.nn.functional.conv2d(xt, wt, torch.from_numpy(b.astype(np.float64)),
                                     stride=(2, 1), padding=1).clamp_min(0)
    ref = ref.permute(0, 2, 3, 1).numpy()
    assert np.allclose(y, ref, rtol=1e-6, atol=1e-6)
    res = rng.normal(size=y.shape).astype(np.float32)
    y2 = orc.conv_f32(g, x, w, b, res, relu=False)
    ref2 = torch.nn.functional.conv2d(xt, wt, torch.from_numpy(b.astype(np.float64)),
                                      stride=(2, 1), padding=1).permute(0, 2, 3, 1).numpy() + res
    assert np.allclose(y2, ref2, rtol=1e-6, atol=1e-6)


def test_maxpool_against_library():
    rng = np.random.default_rng(16)
    x = rng.integers(-128, 128, (2, 11, 11, 6)).astype(np.int8)
    y = orc.maxpool_i8(x, 3, 3, 2, 1, 6, 6)
    ref = torch.nn.functional.max_pool2d(
        torch.from_numpy(x.astype(np.float32)).permute(0, 3, 1, 2), 3, 2, 1)
    assert np.array_equal(y, ref.permute(0, 2, 3, 1).numpy().astype(np.int8))


def _pool_exact(x, mode, R, stride, pad, Ho, Wo, m):
    """Pooling written out with Python integers and exact fractions: window max / window
    sum, the stated fp32 roundings (1/(R*S), sum * that, * m), clamp, round half to even."""
    N, H, W, Cc = x.shape
    inv = fl32(Fraction(1, R * R))
    mf = Fraction(float(np.float32(m)))
    out = np.zeros((N, Ho, Wo, Cc), np.int64)
    for n in range(N):
        for ho in range(Ho):
            for wo in range(Wo):
                for c in range(Cc):
                    vals = [int(x[n, hi, wi, c])
                            for hi in range(ho * stride - pad, ho * stride - pad + R)
                            for wi in range(wo * stride - pad, wo * stride - pad + R)
                            if 0 <= hi < H and 0 <= wi < W]
                    if mode == "max":
                        t = Fraction(max(vals))
                    else:
                        t = fl32(Fraction(sum(vals)) * inv)
                    t = fl32(t * mf)
                    out[n, ho, wo, c] = round_half_even(clamp(t, Fraction(-128), Fraction(127)))
    return out


@pytest.mark.parametrize("mode", ["max", "avg"])
@pytest.mark.parametrize("m", [1.0, 0.5, 0.737, 1.9])
def test_pool_i8_against_exact_arithmetic(mode, m):
    rng = np.random.default_rng(31)
    x = rng.integers(-128, 128, (2, 7, 6, 3)).astype(np.int8)
    for R, stride, pad in ((3, 1, 1), (3, 2, 0), (2, 2, 0)):
        Ho = (7 + 2 * pad - R) // stride + 1
        Wo = (6 + 2 * pad - R) // stride + 1
        got = orc.pool_i8(x, mode, R, R, stride, pad, Ho, Wo, m)
        assert np.array_equal(got, _pool_exact(x, mode, R, stride, pad, Ho, Wo, m)), (R, stride)


def test_pool_i8_against_library_and_slices():
    rng = np.random.default_rng(32)
    x = rng.integers(-128, 128, (2, 12, 11, 5)).astype(np.int8)
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    # max with m = 1 is the library's max pooling exactly, ceil-mode extent included
    ref = torch.nn.functional.max_pool2d(xt, 2, 2, 0, ceil_mode=True).permute(0, 2, 3, 1).numpy()
    assert ref.shape[1:3] == (6, 6)
    assert np.array_equal(orc.pool_i8(x, "max", 2, 2, 2, 0, 6, 6), ref.astype(np.int8))
    # avg: within half a code (+ fp32 slack) of the library's real-valued average,
    # padding counted in the divisor
    ref = torch.nn.functional.avg_pool2d(xt, 3, 1, 1, count_include_pad=True)
    ref = ref.permute(0, 2, 3, 1).numpy()
    got = orc.pool_i8(x, "avg", 3, 3, 1, 1, 12, 11)
    assert np.max(np.abs(got - ref)) <= 0.5 + 1e-4
    # channel-slice write leaves the other channels alone
    base = rng.integers(-128, 128, (2, 12, 11, 9)).astype(np.int8)
    out = orc.pool_i8(x, "avg", 3, 3, 1, 1, 12, 11, out=base.copy(), out_c_off=3)
    assert np.array_equal(out[..., 3:8], got)
    assert np.array_equal(out[..., :3], base[..., :3]) and np.array_equal(out[..., 8:], base[..., 8:])
    # saturation on both sides
    big = np.full((1, 3, 3, 1), 127, np.int8)
    assert orc.pool_i8(big, "max", 3, 3, 1, 0, 1, 1, 2.0)[0, 0, 0, 0] == 127
    assert orc.pool_i8(-big - 1, "avg", 3, 3, 1, 0, 1, 1, 2.0)[0, 0, 0, 0] == -128


def test_sparsity_removal_keeps_the_values_that_are_read():
    """The paper's ResNet graph transformation (the producer of a stride-2 1x1 layer's input
    computes only the pixels that are read, the skip branch is subsampled by a 1x1 stride-2
    pooling): with one factor table both graphs give the same codes wherever the
    transformed graph has a value, and the same network output."""
    from oracle import net as onet
    from paper_1805_08691_amd import workloads as wl
    plain, sparse = wl.resnet50(image=64), wl.resnet50(image=64, sparsity_removal=True)
    assert [o.name for o in plain.convs()] == [o.name for o in sparse.convs()]
    assert sparse.macs_per_image() < plain.macs_per_image()
    params = {op.name: wl.conv_params(3, i, op) for i, op in enumerate(plain.convs())}
    folded = onet.fold_all(plain, params)
    q = onet.calibrate(plain, folded, [wl.input_batch(3, plain, 2, 100)])
    for op in sparse.ops:                         # tensors only the transformed graph has
        if op.kind == "pool" and op.dst not in q:
            q[op.dst] = q[op.src]
    qparams = onet.quantize_params(plain, folded, q)
    z_in = orc.Q(wl.input_batch(3, plain, 1, 0), q[plain.input], 7)
    a = onet.forward_i8(plain, qparams, q, z_in)
    b = onet.forward_i8(sparse, qparams, q, z_in)
    assert np.array_equal(a[plain.outputs[0]], b[sparse.outputs[0]])
    halved = 0
    for name, t in b.items():
        if name not in a:
            continue
        if t.shape == a[name].shape:
            assert np.array_equal(t, a[name]), name
        else:
            assert np.array_equal(t, a[name][:, ::2, ::2]), name
            halved += 1
    assert halved == 3


# ----------------------------------------------------------------------------------------
# unsigned p = 8 activation codes (calibration paragraph: non-negative tensors)
# ----------------------------------------------------------------------------------------
def test_conv_u8_against_float64_library_convolution():
    rng = np.random.default_rng(41)
    for geom in (dict(N=2, H=9, W=8, C=5, K=7, R=3, S=3, pad_h=1, pad_w=1),
                 dict(N=1, H=11, W=11, C=4, K=3, R=3, S=2, stride_h=2, stride_w=1, pad_h=1, pad_w=0,
                      dil_h=2)):
        g = orc.ConvGeom(**geom)
        x = rng.integers(0, 256, (g.N, g.H, g.W, g.C)).astype(np.uint8)
        w = rng.integers(-128, 128, (g.K, g.R, g.S, g.C)).astype(np.int8)
        b = rng.integers(-1000, 1000, g.K).astype(np.int32)
        ref = torch.nn.functional.conv2d(
            torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2),
            torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2),
            torch.from_numpy(b.astype(np.float64)), stride=(g.stride_h, g.stride_w),
            padding=(g.pad_h, g.pad_w), dilation=(g.dil_h, g.dil_w)).permute(0, 2, 3, 1).numpy()
        assert np.array_equal(orc.conv_u8(g, x, w, b), ref.astype(np.int64))
    # the identity the GPU path relies on: codes = (codes - 128) + 128, so the signed
    # contraction of the shifted bytes plus 128 * (sum of the taps that read inside the
    # image) is the same accumulator
    g = orc.ConvGeom(N=1, H=5, W=5, C=3, K=2, R=3, S=3, pad_h=1, pad_w=1)
    x = rng.integers(0, 256, (1, 5, 5, 3)).astype(np.uint8)
    w = rng.integers(-128, 128, (2, 3, 3, 3)).astype(np.int8)
    shifted = orc.conv_i8(g, (x.astype(np.int16) - 128).astype(np.int8), w)
    ones = orc.conv_i8(g, np.ones((1, 5, 5, 3), np.int8), w)      # sum of the inside taps
    assert np.array_equal(orc.conv_u8(g, x, w), shifted + 128 * ones)


def test_requant_mixed_against_exact_rational():
    rng = np.random.default_rng(42)
    acc = rng.integers(-60000, 60000, (1, 512)).astype(np.int32)
    m, m_r = np.float32(0.00437), np.float32(0.613)
    for res_dtype in (np.uint8, np.int8):
        lo_r, hi_r = (0, 256) if res_dtype == np.uint8 else (-128, 128)
        res = rng.integers(lo_r, hi_r, (1, 512)).astype(res_dtype)
        for out_u in (True, False):
            got = orc.requant_mixed(acc, m, True, res, m_r, out_unsigned=out_u)
            lo, hi = (0, 255) if out_u else (-128, 127)
            want = []
            for a, r in zip(acc.ravel().tolist(), res.ravel().tolist()):
                t = fl32(fl32(F(a)) * F(float(m)))
                t = fl32(t + fl32(F(r) * F(float(m_r))))
                t = max(t, F(0))
                want.append(round_half_even(clamp(t, F(lo), F(hi))))
            assert got.ravel().tolist() == want, (res_dtype, out_u)
    # hand-worked: acc * 0.5 = 2.5 300 -4 255.5 -> ties to even, saturation at 255, ReLU
    assert orc.requant_mixed(np.array([[5, 600, -8, 511]], np.int32), 0.5, True,
                             out_unsigned=True).ravel().tolist() == [2, 255, 0, 255]


def test_dequantize_u8_hand_worked():
    """Eq. D on unsigned codes: the hand-worked values of tests/golden/eq_D_u8.txt (exact where
    the product is a binary fraction, else within one fp32 rounding of q * z), the identity
    Q(D(z)) = z on all 256 codes, and agreement with the signed form on the shared range."""
    for name, c in golden_io.load("eq_D_u8.txt").items():
        got = orc.D_u8(np.array(c["z"], np.uint8), c["q"])
        want = np.array(c["r"], np.float64)
        assert got.dtype == np.float32
        assert np.all(np.abs(got.astype(np.float64) - want) <= 2.0 ** -23 * np.abs(want)), name
        if name == "halves":
            assert got.tolist() == c["r"]
    z = np.arange(256, dtype=np.uint8)
    for q in (0.5, 0.02, 0.0371):
        r = orc.D_u8(z, q)
        assert np.all(np.diff(r) > 0) and r[0] == 0.0
        back = np.clip(np.rint(r.astype(np.float64) / np.float32(q)), 0, 255)
        assert np.array_equal(back.astype(np.uint8), z)
        assert np.array_equal(r[:128], orc.D(z[:128].astype(np.int8), q))


def test_unsigned_network_reading_on_a_small_resnet():
    """Unsigned codes halve the quantisation step of the ReLU outputs: the int8 network's
    dequantised output is closer to the fp32 network's with them than without."""
    from oracle import net as onet
    from paper_1805_08691_amd import workloads as wl
    net = wl.resnet50(image=64)
    params = {op.name: wl.conv_params(3, i, op) for i, op in enumerate(net.convs())}
    folded = onet.fold_all(net, params)
    cal = [wl.input_batch(3, net, 2, 100)]
    x = wl.input_batch(3, net, 1, 0)
    ref = onet.forward_f32(net, folded, x)[0][net.outputs[0]]
    err = {}
    for mode in (False, True):
        U = onet.unsigned_tensors(net) if mode else set()
        q = onet.calibrate(net, folded, cal, unsigned=U)
        qp = onet.quantize_params(net, folded, q)
        acts = onet.forward_i8(net, qp, q, orc.Q(x, q[net.input], 7), unsigned=U)
        o = net.outputs[0]
        assert acts[o].dtype == (np.uint8 if mode else np.int8)
        y = orc.D_u8(acts[o], q[o]) if mode else orc.D(acts[o], q[o])
        err[mode] = float(np.sqrt(np.mean((y - ref) ** 2)))
    assert err[True] < err[False]


def test_sum_factor_rule_and_its_variant_on_a_small_resnet():
    """Eq. + gives a fused sum the factor max(q1, q2), under which the sum can exceed the
    int8 range; calibrating the sum's own max-abs (the variant) never saturates on the
    calibration data itself."""
    from oracle import net as onet
    from paper_1805_08691_amd import workloads as wl
    net = wl.resnet50(image=64)
    params = {op.name: wl.conv_params(3, i, op) for i, op in enumerate(net.convs())}
    folded = onet.fold_all(net, params)
    x = wl.input_batch(3, net, 2, 100)
    sums = [op for op in net.convs() if op.res]
    ref = onet.forward_f32(net, folded, x)[0]
    q_rule = onet.calibrate(net, folded, [x])
    q_own = onet.calibrate(net, folded, [x], own_sum_factor=True)
    for op in sums:
        assert q_rule[op.dst] == max(q_rule[op.name + ":branch"], q_rule[op.res])
        assert q_own[op.dst] == orc.qfactor(orc.maxabs(ref[op.dst]), 7)
    assert {k: v for k, v in q_rule.items() if k not in {o.dst for o in sums}} == \
           {k: v for k, v in q_own.items() if k not in {o.dst for o in sums}}
    # the first fused sum reads tensors whose codes do not depend on the choice: compare there
    op = sums[0]
    sat = {}
    for tag, q in (("rule", q_rule), ("own", q_own)):
        qp = onet.quantize_params(net, folded, q)
        acts = onet.forward_i8(net, qp, q, orc.Q(x, q[net.input], 7))
        sat[tag] = int(np.sum(acts[op.dst] == 127))
        err = np.abs(orc.D(acts[op.dst], q[op.dst]) - ref[op.dst]).max()
        if tag == "own":       # no clipping: the error stays a few steps (it is inherited)
            assert err < 6 * q[op.dst]
    # under its own factor only the calibrated maximum (and near ties) reach the last code
    assert sat["own"] <= 4


# ----------------------------------------------------------------------------------------
# per-output-channel weight factors
# ----------------------------------------------------------------------------------------
def test_per_channel_weights_and_scales():
    rng = np.random.default_rng(51)
    W = (rng.standard_normal((6, 3, 3, 5)) * np.array([.01, .1, 1, 3, 0, 7])[:, None, None, None])
    W = W.astype(np.float32)
    z_w, q_w = orc.quantize_weights_pc(W)
    for k in range(6):
        mx = np.abs(W[k]).max()
        if mx == 0:
            assert q_w[k] == 1 and not z_w[k].any()           # all-zero filter: q = 1
            continue
        assert q_w[k] == np.float32(mx) / np.float32(127)
        assert np.abs(z_w[k].astype(int)).max() == 127        # the row's extreme hits the last code
        assert np.array_equal(z_w[k], orc.Q(W[k], q_w[k], 7))
    b = rng.standard_normal(6).astype(np.float32)
    q_x = np.float32(0.0173)
    z_b = orc.Q31_bias_pc(b, q_x, q_w)
    for k in range(6):
        q = fl64(F(float(q_x)) * F(float(q_w[k])))
        assert z_b[k] == clamp(round_half_even(fl64(F(float(b[k])) / q)), -2**31, 2**31 - 1)
    m = orc.requant_scales_pc(q_x, q_w, np.float32(0.31))
    for k in range(6):
        want = fl32(fl32(F(float(q_x)) * F(float(q_w[k]))) / F(float(np.float32(0.31))))
        assert F(float(m[k])) == want


def test_requant_per_channel_against_exact_rational():
    rng = np.random.default_rng(52)
    K = 9
    acc = rng.integers(-90000, 90000, (40, K)).astype(np.int32)
    m = (rng.uniform(0.0005, 0.004, K)).astype(np.float32)
    res = rng.integers(-128, 128, (40, K)).astype(np.int8)
    m_r = np.float32(0.37)
    got = orc.requant_pc(acc, m, True, res, m_r)
    for p in range(40):
        for k in range(K):
            t = fl32(fl32(F(int(acc[p, k]))) * F(float(m[k])))
            t = fl32(t + fl32(F(int(res[p, k])) * F(float(m_r))))
            t = max(t, F(0))
            assert got[p, k] == round_half_even(clamp(t, F(-128), F(127))), (p, k)
    # equal factors: the per-tensor tail
    same = np.full(K, np.float32(0.0021), np.float32)
    assert np.array_equal(orc.requant_pc(acc, same, False), orc.requant(acc, same[0], False))


# ----------------------------------------------------------------------------------------
# a layer whose output leaves the quantised domain: Eq. D on the accumulator, no Q
# ----------------------------------------------------------------------------------------
def test_real_output_against_exact_rational():
    rng = np.random.default_rng(61)
    K = 7
    acc = rng.integers(-3_000_000, 3_000_000, (30, K)).astype(np.int32)
    acc[0, :3] = [16777217, -16777219, 0]                 # int32 -> fp32 rounds first
    res = rng.integers(-128, 128, (30, K)).astype(np.int8)
    q_x, q_w, q_res = np.float32(0.0213), np.float32(0.00071), np.float32(0.0456)
    s = fl32(F(float(q_x)) * F(float(q_w)))
    for relu in (False, True):
        for with_res in (False, True):
            got = orc.real_output(acc, q_x, q_w, relu, res if with_res else None, q_res)
            assert got.dtype == np.float32
            for p in range(30):
                for k in range(K):
                    t = fl32(fl32(F(int(acc[p, k]))) * s)
                    if with_res:
                        t = fl32(t + fl32(F(int(res[p, k])) * F(float(q_res))))
                    if relu:
                        t = max(t, F(0))
                    assert F(float(got[p, k])) == t, (relu, with_res, p, k)


def test_real_output_is_the_value_the_int8_tail_quantises():
    # power-of-two factors: every fp32 step is exact, so Q(y', q_out) equals the int8 tail,
    # and y' equals the real-valued layer on the dequantised operands computed in float64
    rng = np.random.default_rng(62)
    g = orc.ConvGeom(N=2, H=6, W=5, C=8, K=6, R=3, S=3, pad_h=1, pad_w=1)
    z_x = rng.integers(-128, 128, (2, 6, 5, 8)).astype(np.int8)
    z_w = rng.integers(-127, 128, (6, 3, 3, 8)).astype(np.int8)
    z_b = rng.integers(-5000, 5000, 6).astype(np.int32)
    z_r = rng.integers(-128, 128, (2, 6, 5, 6)).astype(np.int8)
    q_x, q_w, q_res, q_out = (np.float32(2.0 ** e) for e in (-5, -9, -4, -3))
    acc = orc.conv_i8(g, z_x, z_w, z_b)
    y = orc.real_output(acc, q_x, q_w, True, z_r, q_res)
    xt = torch.from_numpy(z_x.astype(np.float64) * float(q_x)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(z_w.astype(np.float64) * float(q_w)).permute(0, 3, 1, 2)
    bt = torch.from_numpy(z_b.astype(np.float64) * float(q_x) * float(q_w))
    want = torch.nn.functional.conv2d(xt, wt, bt, padding=1).permute(0, 2, 3, 1).numpy()
    want = np.maximum(want + z_r.astype(np.float64) * float(q_res), 0.0)
    assert np.array_equal(y.astype(np.float64), want)
    m = orc.requant_scale(q_x, q_w, q_out)
    z_y = orc.requant(acc, m, True, z_r, orc.residual_scale(q_res, q_out))
    assert np.array_equal(orc.Q(y, q_out, 7), z_y)


def test_real_output_channel_slice():
    rng = np.random.default_rng(63)
    acc = rng.integers(-1000, 1000, (5, 3)).astype(np.int32)
    out = np.full((5, 8), np.float32(-7.0))
    orc.real_output(acc, 0.5, 0.25, False, out=out, out_c_stride=8, out_c_off=2)
    assert np.array_equal(out[:, 2:5], acc.astype(np.float32) * np.float32(0.125))
    assert np.all(out[:, :2] == -7.0) and np.all(out[:, 5:] == -7.0)
