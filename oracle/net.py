"""Oracle-side network evaluation (TEST INFRASTRUCTURE): chains the oracle's layer
functions over a layer list, with its own calibration.  Shares no code with the GPU
engine; it only reads the same graph description objects (duck-typed: ``ops`` with
``kind``, ``src``, ``dst``, ... and ``tensors``).

Calibration (text after Eq. +/x): every activation factor is max|tensor| / (2^p - 1) with
p = 7, the maximum taken over all calibration batches of an fp32 forward of the folded
network.  For a conv with a fused sum, the + rule sets q_out = max(q1, q_res) where q1 is
the factor of the branch's own pre-sum output.
"""
import numpy as np
import torch

from . import (ConvGeom, Q, Q31_bias, Q31_bias_pc, conv_f32, conv_i8, conv_u8, fold_bn, maxabs,
               pool_i8, qfactor, quantize_weights_pc, requant, requant_mixed, requant_pc,
               requant_scale, requant_scales_pc, residual_scale)

P_ACT = 7
P_W = 7


def geom(op, tensors, N):
    s = tensors[op.src]
    return ConvGeom(N=N, H=s.H, W=s.W, C=op.C, K=op.K, R=op.R, S=op.S, stride_h=op.stride,
                    stride_w=op.stride, pad_h=op.pad_h, pad_w=op.pad_w, dil_h=op.dil,
                    dil_w=op.dil)


def fold_all(net, params):
    """Eq. BN for every conv: name -> (W' KRSC fp32, b' fp32)."""
    out = {}
    for op in net.ops:
        if op.kind != "conv":
            continue
        p = params[op.name]
        out[op.name] = fold_bn(p["W"], p["b"], p["gamma"], p["beta"], p["mu"], p["var"], p["eps"])
    return out


def _conv_f32_lib(op, x, Wf, bf):
    """fp32 library convolution (a step of the calibration forward, not of the method)."""
    xt = torch.from_numpy(x).permute(0, 3, 1, 2)
    wt = torch.from_numpy(Wf).permute(0, 3, 1, 2)
    y = torch.nn.functional.conv2d(xt, wt, torch.from_numpy(bf), stride=op.stride,
                                   padding=(op.pad_h, op.pad_w), dilation=op.dil)
    return np.ascontiguousarray(y.permute(0, 2, 3, 1).numpy())


def forward_f32(net, folded, x, use_library=True):
    """fp32 forward of the folded network.  Returns (tensors, pre_sum) where pre_sum holds,
    per conv with a fused sum, the branch output before the sum."""
    t = {net.input: x}
    pre = {}
    for op in net.ops:
        if op.kind == "pool":
            d = net.tensors[op.dst]
            xt = torch.from_numpy(t[op.src]).permute(0, 3, 1, 2)
            ceil = d.H != (xt.shape[2] + 2 * op.pad - op.R) // op.stride + 1
            if op.mode == "max":
                y = torch.nn.functional.max_pool2d(xt, (op.R, op.S), op.stride, op.pad,
                                                   ceil_mode=ceil)
            else:
                y = torch.nn.functional.avg_pool2d(xt, (op.R, op.S), op.stride, op.pad,
                                                   count_include_pad=True)
            y = np.ascontiguousarray(y.permute(0, 2, 3, 1).numpy())
            assert y.shape[1:3] == (d.H, d.W), (op.name, y.shape, d)
            if d.C == y.shape[3]:
                t[op.dst] = y
            else:
                if op.dst not in t:
                    t[op.dst] = np.zeros(y.shape[:3] + (d.C,), np.float32)
                t[op.dst][..., op.dst_c_off:op.dst_c_off + y.shape[3]] = y
            continue
        Wf, bf = folded[op.name]
        xin = t[op.src]
        if use_library:
            y = _conv_f32_lib(op, xin, Wf, bf)
        else:
            y = conv_f32(geom(op, net.tensors, xin.shape[0]), xin, Wf, bf)
        if op.res is not None:
            pre[op.name] = y
            y = y + t[op.res]
        if op.relu:
            y = np.maximum(y, 0)
        d = net.tensors[op.dst]
        if d.C == op.K:
            t[op.dst] = y
        else:
            if op.dst not in t:
                t[op.dst] = np.zeros(y.shape[:3] + (d.C,), np.float32)
            t[op.dst][..., op.dst_c_off:op.dst_c_off + op.K] = y
    return t, pre


def unsigned_tensors(net):
    """Tensors that hold unsigned p = 8 codes when the calibration paragraph's rule for
    non-negative activations is applied: outputs of ReLU layers (a fused sum included) and
    max-poolings of such tensors.  Everything else (the image, outputs without ReLU) stays
    signed p = 7 (reading: instead of the paper's FP32 fallback)."""
    u = set()
    for op in net.ops:
        if op.kind == "conv":
            assert net.tensors[op.dst].C == op.K, "unsigned mode: no concatenations"
            if op.relu:
                u.add(op.dst)
        else:
            assert op.mode == "max" and net.tensors[op.dst].C == net.tensors[op.src].C
            if op.src in u:
                u.add(op.dst)
    return u


def calibrate(net, folded, batches, use_library=True, unsigned=None, own_sum_factor=False):
    """Running max-abs over ``batches`` (iterable of fp32 NHWC inputs) -> factor table
    {tensor name: q} plus {conv name + ':branch': q1} for fused sums.

    ``unsigned`` (a set of tensor names): those tensors get q = max / (2^8 - 1); and the
    output of a fused sum then keeps its OWN calibrated factor (the max(q1, q2) rule of
    Eq. + presumes equal precisions, which a signed branch and an unsigned output are not).
    ``own_sum_factor``: the same choice with signed codes -- a variant, not the paper's rule:
    max(q1, q2) lets the sum saturate where both branches are large, the sum's own max-abs
    does not."""
    mx = {}

    def upd(key, arr):
        m = maxabs(arr)
        if m > mx.get(key, np.float32(0)):
            mx[key] = m
        mx.setdefault(key, np.float32(0))

    for x in batches:
        t, pre = forward_f32(net, folded, x, use_library)
        for name, arr in t.items():
            upd(name, arr)
        for name, arr in pre.items():
            upd(name + ":branch", arr)
    unsigned = unsigned or set()
    q = {k: qfactor(v, 8 if k in unsigned else P_ACT) for k, v in mx.items()}
    # + rule: a fused sum is re-quantised at max(q1, q2)
    for op in net.ops:
        if op.kind == "conv" and op.res is not None and not unsigned and not own_sum_factor:
            q[op.dst] = max(q[op.name + ":branch"], q[op.res])
        if op.kind == "pool" and net.tensors[op.dst].C == net.tensors[op.src].C:
            q[op.dst] = q[op.src]          # a stand-alone pool keeps its input's factor
    return q


def quantize_params(net, folded, q, per_channel=False):
    """name -> dict(z_w int8 KRSC, q_w, z_b int32).  ``per_channel``: q_w is an fp32 vector
    with one factor per output channel."""
    out = {}
    for op in net.ops:
        if op.kind != "conv":
            continue
        Wf, bf = folded[op.name]
        if per_channel:
            z_w, q_w = quantize_weights_pc(Wf, P_W)
            out[op.name] = dict(z_w=z_w, q_w=q_w, z_b=Q31_bias_pc(bf, q[op.src], q_w))
            continue
        q_w = qfactor(maxabs(Wf), P_W)
        out[op.name] = dict(z_w=Q(Wf, q_w, P_W), q_w=q_w, z_b=Q31_bias(bf, q[op.src], q_w))
    return out


def _maxpool_u8(x, op, Ho, Wo):
    """max-pooling of unsigned codes with the library routine (exact on small integers)."""
    xt = torch.from_numpy(x.astype(np.float32)).permute(0, 3, 1, 2)
    ceil = Ho != (x.shape[1] + 2 * op.pad - op.R) // op.stride + 1
    y = torch.nn.functional.max_pool2d(xt, (op.R, op.S), op.stride, op.pad, ceil_mode=ceil)
    y = y.permute(0, 2, 3, 1).numpy()
    assert y.shape[1:3] == (Ho, Wo)
    return np.ascontiguousarray(y.astype(np.uint8))


def forward_i8(net, qparams, q, z_in, keep_acc=False, unsigned=None):
    """int8 forward (Eq. A' per conv).  Returns {tensor: int8 array} (and accumulators).
    Tensors named in ``unsigned`` are uint8 arrays of p = 8 codes."""
    unsigned = unsigned or set()
    t = {net.input: z_in}
    accs = {}
    N = z_in.shape[0]
    for op in net.ops:
        if op.kind == "pool" and op.src in unsigned:
            d = net.tensors[op.dst]
            t[op.dst] = _maxpool_u8(t[op.src], op, d.H, d.W)
            continue
        if op.kind == "conv" and unsigned:
            qp = qparams[op.name]
            g = geom(op, net.tensors, N)
            conv = conv_u8 if op.src in unsigned else conv_i8
            acc = conv(g, t[op.src], qp["z_w"], qp["z_b"])
            if keep_acc:
                accs[op.name] = acc
            res, m_r = None, 0.0
            if op.res is not None:
                res, m_r = t[op.res], residual_scale(q[op.res], q[op.dst])
            t[op.dst] = requant_mixed(acc, requant_scale(q[op.src], qp["q_w"], q[op.dst]),
                                      op.relu, res, m_r, out_unsigned=op.dst in unsigned)
            continue
        if op.kind == "pool":
            d = net.tensors[op.dst]
            if op.dst not in t:
                t[op.dst] = np.zeros((N, d.H, d.W, d.C), np.int8)
            m = residual_scale(q[op.src], q[op.dst])        # q_in / q_out in fp32 (1 if equal)
            pool_i8(t[op.src], op.mode, op.R, op.S, op.stride, op.pad, d.H, d.W, m,
                    out=t[op.dst], out_c_off=op.dst_c_off)
            continue
        qp = qparams[op.name]
        g = geom(op, net.tensors, N)
        acc = conv_i8(g, t[op.src], qp["z_w"], qp["z_b"])
        if keep_acc:
            accs[op.name] = acc
        q_out = q[op.dst]
        d = net.tensors[op.dst]
        if op.dst not in t:
            t[op.dst] = np.zeros((N, d.H, d.W, d.C), np.int8)
        res, m_r = None, 0.0
        if op.res is not None:
            res, m_r = t[op.res], residual_scale(q[op.res], q_out)
        if np.ndim(qp["q_w"]) == 1:                     # one weight factor per channel
            requant_pc(acc, requant_scales_pc(q[op.src], qp["q_w"], q_out), op.relu, res, m_r,
                       out=t[op.dst], out_c_stride=d.C, out_c_off=op.dst_c_off)
            continue
        m = requant_scale(q[op.src], qp["q_w"], q_out)
        requant(acc, m, op.relu, res, m_r, out=t[op.dst], out_c_stride=d.C,
                out_c_off=op.dst_c_off)
    return (t, accs) if keep_acc else t
