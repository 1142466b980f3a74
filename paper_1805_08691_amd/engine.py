"""Runs a layer list on the GPU through the C-ABI calls of ``binding``.

Host-side orchestration only: which call follows which, which buffer a layer reads and
writes, which factor goes with which tensor.  All arithmetic happens inside libq8conv.so.
Offline steps (in the paper's flow, Fig. "steps to generate the optimized model"):
  fold()               Eq. BN on every conv
  calibrate(batches)   fp32 forward of the folded net + running max-abs per tensor
  quantize_weights()   per-tensor q_w, int8 filters (packed), int32 bias at q_x * q_w
Online step:
  run_step(x, dequant) Q on the input image, one fused conv launch per layer (Eq. A'), D on the
                       outputs that leave the int8 domain; forward(x) is run_step without D.
"""
import numpy as np
import torch

from . import binding as B

P_ACT = 7
P_W = 7


def _pad_c(c):
    """Stored channel count of an activation tensor (3-channel images are stored as 4)."""
    return 4 if c < 4 else c


class Engine:
    """``n_streams`` = 2 (up to 4) runs every layer as that many concurrent part-batch pipelines
    (batch elements are independent once the factor table is frozen): one on the caller's
    stream, the others on side streams of the same (default) priority, forked behind the
    quantisation of the input and joined again before the outputs are dequantised.  A layer's launch latency and its
    tail then overlap the other half's work.  Results are the same bits as with one stream."""

    def __init__(self, net, batch, device="cuda", n_streams=1, unsigned_activations=False,
                 per_channel_weights=False, real_outputs=False, own_sum_factor=False,
                 fuse_pairs=False, chain=False, fuse_duals=False, fuse_head=False,
                 fuse_dequant=False):
        self.net = net
        # fuse_dequant: where run_step is asked for Eq. D of a tensor that one convolution writes
        # whole, that convolution writes the fp32 values beside its codes (same values; no
        # separate pass over the tensor)
        self.fuse_dequant = fuse_dequant
        self._deq = {}        # tensor name -> fp32 buffer of the running step (fused Eq. D)
        # fuse_head: Eq. Q on the input image, the first convolution and the max-pool behind it
        # run as one launch per pipeline where the library has a build for them (same
        # results; the image's codes and the convolution's own output are then not written
        # in a step that starts from the real-valued batch)
        self.fuse_head = fuse_head
        self.head = None      # (first conv, the pool fused into it or None)
        self._x = None        # the real-valued batch of the running step (fused head)
        # fuse_duals: two consecutive convolutions that read the same tensor and do not depend on
        # each other (a stage's projection branch and its first 1x1) run as one launch where
        # the library has a tile-shape pair for them
        self.fuse_duals = fuse_duals
        self.duals = {}       # first conv name -> second conv
        self.dualed = set()
        # chain: every run of consecutive convolutions the library can take as a list runs as
        # ONE persistent launch (q8_conv_chain_int8: the batch split over the XCDs, tiles
        # started by the completion of the tiles they read) instead of one launch per layer
        self.chain = chain
        self.chains = None    # [(first op index, one past the last, binding.ConvChain)]
        assert not (chain and (n_streams > 1 or unsigned_activations or per_channel_weights
                               or real_outputs or fuse_pairs))
        # fuse_pairs: a convolution whose output only one 1x1 layer reads runs together with
        # that layer in one launch where the library supports the pair (same results; the
        # intermediate tensor is then never written)
        self.fuse_pairs = fuse_pairs
        self.pairs = {}       # first conv name -> second conv (launched together)
        self.paired = set()   # names of the second convs
        # own_sum_factor: a fused sum's output is calibrated by its own max-abs instead of
        # the max(q1, q2) rule of Eq. + (a variant; implied by unsigned activations)
        self.own_sum_factor = own_sum_factor
        assert not (unsigned_activations and per_channel_weights)
        # real_outputs: a network output that a convolution writes whole and no layer reads
        # is produced as fp32 by that convolution (no int8 code, no separate Eq. D pass)
        self.real = set()
        if real_outputs:
            assert not (unsigned_activations or per_channel_weights)
            read = {o.src for o in net.ops} | {o.res for o in net.ops if o.kind == "conv" and o.res}
            for o in net.convs():
                if o.dst in net.outputs and o.dst not in read and net.tensors[o.dst].C == o.K:
                    self.real.add(o.dst)
        self.act_f32 = {}     # tensor name -> fp32 device buffer (real_outputs)
        self.per_channel = per_channel_weights
        self.m_vec = {}       # conv name -> per-channel scales (per_channel_weights)
        # Unsigned p = 8 codes for the outputs of ReLU layers (the calibration paragraph's
        # rule for non-negative tensors) and for max-poolings of such tensors; stored as
        # code - 128.  Everything else stays signed p = 7.
        self.unsigned = set()
        if unsigned_activations:
            for o in net.ops:
                if o.kind == "conv":
                    assert net.tensors[o.dst].C == o.K, "unsigned mode: no concatenations"
                    if o.relu:
                        self.unsigned.add(o.dst)
                else:
                    assert o.mode == "max" and net.tensors[o.dst].C == net.tensors[o.src].C
                    if o.src in self.unsigned:
                        self.unsigned.add(o.dst)
        self.taps = {}        # conv name -> table of accumulator start values (padded layers
                              # reading unsigned codes)
        self.N = batch
        self.dev = torch.device(device)
        assert 1 <= n_streams <= 4
        self.n_streams = min(n_streams, max(batch, 1))
        self.side = [torch.cuda.Stream(device=self.dev) for _ in range(self.n_streams - 1)]
        # the batch in n_streams nearly equal parts (the first ones one image larger)
        self.parts, lo = [], 0
        for i in range(self.n_streams):
            n = batch // self.n_streams + (1 if i < batch % self.n_streams else 0)
            self.parts.append((lo, n))
            lo += n
        # number of leading layers that run on the whole batch before it is split (none: the
        # pipelines start right behind the quantisation of the input)
        self.n_unsplit = 0 if self.n_streams > 1 else len(net.ops)
        self.part_desc = {}   # (conv name, images) -> ConvDesc
        # An image of fewer than 4 channels read by one convolution is stored inside a zero
        # frame that holds that layer's padding, and the layer runs without padding.
        self.in_frame = None
        t_in = net.tensors[net.input]
        readers = [o for o in net.convs() if o.src == net.input]
        if _pad_c(t_in.C) != t_in.C and len(readers) == 1 and readers[0].dil == 1:
            o = readers[0]
            self.in_frame = (o.pad_h, o.pad_w, t_in.H + 2 * o.pad_h, t_in.W + 2 * o.pad_w)
        self.params = {}      # conv name -> dict of fp32 device tensors
        self.folded = {}      # conv name -> (W', b')
        self.q = {}           # tensor name -> activation factor (host float)
        self.qw = {}          # conv name -> weight factor
        self.wq = {}          # conv name -> (packed int8 filters, int32 bias)
        self.act = {}         # tensor name -> int8 device buffer [N, H, W, C_stored]
        self.desc = {}        # conv name -> ConvDesc
        self.graph = None
        for op in net.ops:
            if op.kind == "conv":
                self.desc[op.name] = self._desc(op, batch)
        if fuse_pairs:
            assert not (unsigned_activations or per_channel_weights)
            self._find_pairs()
        if fuse_head:
            assert not (unsigned_activations or per_channel_weights or chain)
            self._find_head()
        if fuse_duals:
            assert not (unsigned_activations or per_channel_weights or real_outputs)
            self._find_duals()

    def _find_head(self):
        ops, t_in = self.net.ops, self.net.tensors[self.net.input]
        if not self.in_frame or not ops or ops[0].kind != "conv" or ops[0].src != self.net.input:
            return
        conv = ops[0]
        if conv.res or conv.dst_c_off or conv.name in self.pairs or conv.name in self.duals \
                or conv.dst in self.real:
            return
        top, left = self.in_frame[:2]
        pool = None
        if len(ops) > 1 and ops[1].kind == "pool" and ops[1].src == conv.dst:
            o = ops[1]
            others = [u for u in ops[2:] if u.src == conv.dst or (u.kind == "conv" and u.res == conv.dst)]
            s, d = self.net.tensors[o.src], self.net.tensors[o.dst]
            if (o.mode == "max" and (o.R, o.S, o.stride, o.pad) == (3, 3, 2, 1) and not others
                    and conv.dst not in self.net.outputs and d.C == s.C and o.dst_c_off == 0
                    and (d.H, d.W) == ((s.H - 1) // 2 + 1, (s.W - 1) // 2 + 1)):
                pool = o
        for cand in ((pool,) if pool is None else (pool, None)):
            if B.conv_image_f32_supported(self.desc[conv.name], t_in.H, t_in.W, t_in.C, top, left,
                                          1 if cand else 0):
                self.head = (conv, cand)
                return

    def _find_duals(self):
        ops = self.net.ops
        n_part = self.parts[0][1]
        for a, b in zip(ops, ops[1:]):
            if a.kind != "conv" or b.kind != "conv" or a.src != b.src:
                continue
            if a.name in self.dualed or a.name in self.pairs or b.name in self.pairs or \
                    a.name in self.paired or b.name in self.paired:
                continue
            if a.dst in (b.src, b.res) or b.dst in (a.src, a.res) or a.dst == b.dst:
                continue
            if B.conv_dual_supported(self.conv_desc(a, n_part), self.conv_desc(b, n_part)):
                self.duals[a.name] = b
                self.dualed.add(b.name)

    def _find_pairs(self):
        net = self.net
        ops = net.ops
        for i, a in enumerate(ops):
            if a.kind != "conv" or a.res or a.dst in net.outputs or a.dst in self.real:
                continue
            if net.tensors[a.dst].C != a.K or a.name in self.paired:
                continue
            readers = [o for o in ops if o.src == a.dst or (o.kind == "conv" and o.res == a.dst)]
            if len(readers) != 1 or readers[0].kind != "conv" or readers[0].src != a.dst:
                continue
            b = readers[0]
            if b.dst in self.real or ops.index(b) != i + 1:
                continue
            # both launches must lie on the same side of the half-batch split
            if (i < self.n_unsplit) != (i + 1 < self.n_unsplit):
                continue
            if B.conv_pair_supported(self.desc[a.name], self.desc[b.name]):
                self.pairs[a.name] = b
                self.paired.add(b.name)

    # ------------------------------------------------------------------ descriptors
    def _desc(self, op, N, framed=True):
        s, d = self.net.tensors[op.src], self.net.tensors[op.dst]
        res_cs = _pad_c(self.net.tensors[op.res].C) if op.res else 0
        H, W, pad_h, pad_w = s.H, s.W, op.pad_h, op.pad_w
        if framed and op.src == self.net.input and self.in_frame:
            _, _, H, W = self.in_frame
            pad_h = pad_w = 0
        desc = B.ConvDesc(N, H, W, op.C, op.K, op.R, op.S, op.stride, op.stride, pad_h, pad_w,
                          op.dil, op.dil, relu=op.relu, in_c_stride=_pad_c(s.C),
                          out_c_stride=_pad_c(d.C), out_c_off=op.dst_c_off, res_c_stride=res_cs)
        assert (desc.Ho, desc.Wo) == (d.H, d.W), (op.name, desc.Ho, desc.Wo, d)
        return desc

    # ------------------------------------------------------------------ offline steps
    def load_params(self, params):
        for name, p in params.items():
            self.params[name] = {k: (torch.from_numpy(v).to(self.dev) if isinstance(v, np.ndarray)
                                     else v) for k, v in p.items()}

    def fold(self):
        for op in self.net.convs():
            p = self.params[op.name]
            self.folded[op.name] = B.fold_bn(p["W"], p["b"], p["gamma"], p["beta"], p["mu"],
                                             p["var"], p["eps"])

    def forward_f32(self, x, observe=None):
        """fp32 forward of the folded network; ``observe(key, tensor)`` sees every activation."""
        t = {self.net.input: x}
        N = x.shape[0]
        for op in self.net.ops:
            d = self.net.tensors[op.dst]
            if op.kind == "pool":
                if d.C == self.net.tensors[op.src].C:
                    t[op.dst] = B.pool_f32(t[op.src], op.mode, op.R, op.S, op.stride, op.pad, d.H,
                                           d.W)
                else:
                    if op.dst not in t:
                        t[op.dst] = torch.zeros((N, d.H, d.W, d.C), dtype=torch.float32,
                                                device=self.dev)
                    B.pool_f32(t[op.src], op.mode, op.R, op.S, op.stride, op.pad, d.H, d.W,
                               out=t[op.dst], out_c_off=op.dst_c_off)
            else:
                Wf, bf = self.folded[op.name]
                desc = self._desc(op, N, framed=False)
                desc.in_c_stride = desc.out_c_stride = desc.res_c_stride = 0
                if op.res is not None and observe:
                    desc.relu = 0                  # the branch's own output, before the sum
                    observe(op.name + ":branch", B.conv_f32_ref(desc, t[op.src], Wf, bf))
                desc.relu = int(op.relu)
                y = B.conv_f32_ref(desc, t[op.src], Wf, bf, t[op.res] if op.res else None)
                if d.C == op.K:
                    t[op.dst] = y
                else:
                    if op.dst not in t:
                        t[op.dst] = torch.zeros((N, d.H, d.W, d.C), dtype=torch.float32,
                                                device=self.dev)
                    t[op.dst][..., op.dst_c_off:op.dst_c_off + op.K] = y
            width = op.K if op.kind == "conv" else self.net.tensors[op.src].C
            if observe and d.C == width:
                observe(op.dst, t[op.dst])
        if observe:
            seen = set()
            for op in self.net.ops:             # concat targets: observe once complete
                d = self.net.tensors[op.dst]
                width = op.K if op.kind == "conv" else self.net.tensors[op.src].C
                if d.C != width and op.dst not in seen:
                    seen.add(op.dst)
                    observe(op.dst, t[op.dst])
        return t

    def calibrate(self, batches):
        """Running max-abs over fp32 forwards of ``batches`` (device fp32 NHWC tensors)."""
        slots = {}

        def observe(key, tensor):
            if key not in slots:
                slots[key] = torch.zeros(1, dtype=torch.float32, device=self.dev)
            B.calibrate_maxabs(tensor.contiguous(), slots[key])

        for x in batches:
            observe(self.net.input, x)
            self.forward_f32(x, observe)
        keys = list(slots)
        vals = torch.cat([slots[k] for k in keys]).cpu().numpy()
        q = {k: B.qfactor(float(v), 8 if k in self.unsigned else P_ACT)
             for k, v in zip(keys, vals)}
        for op in self.net.ops:
            if (op.kind == "conv" and op.res is not None and not self.unsigned
                    and not self.own_sum_factor):
                q[op.dst] = B.sum_factor(q[op.name + ":branch"], q[op.res])   # Eq. +
            if op.kind == "pool" and self.net.tensors[op.dst].C == self.net.tensors[op.src].C:
                q[op.dst] = q[op.src]       # a stand-alone pool keeps its input's factor
        self.q = q
        return q

    def set_factors(self, q):
        self.q = {k: float(v) for k, v in q.items()}

    def quantize_weights_per_channel(self):
        for op in self.net.convs():
            Wf, bf = self.folded[op.name]
            q_w, z_w = B.quantize_weights_per_channel(Wf, P_W)
            self.zw_dense = getattr(self, "zw_dense", {})
            self.zw_dense[op.name] = z_w
            self.qw[op.name] = q_w
            self.wq[op.name] = (B.pack_weights(self.desc[op.name], z_w),
                                B.quantize_bias_per_channel(bf, self.q[op.src], q_w))
            self.m_vec[op.name] = B.requant_scales(self.q[op.src], q_w, self.q[op.dst])

    def quantize_weights(self):
        if self.per_channel:
            return self.quantize_weights_per_channel()
        slots = {}
        for op in self.net.convs():
            Wf, _ = self.folded[op.name]
            slots[op.name] = torch.zeros(1, dtype=torch.float32, device=self.dev)
            B.calibrate_maxabs(Wf, slots[op.name])
        names = list(slots)
        vals = torch.cat([slots[k] for k in names]).cpu().numpy()
        self.zw_dense = {}
        for name, v in zip(names, vals):
            op = next(o for o in self.net.convs() if o.name == name)
            Wf, bf = self.folded[name]
            q_w = B.qfactor(float(v), P_W)
            z_w = B.quantize(Wf, q_w, P_W)
            self.zw_dense[name] = z_w
            self.qw[name] = q_w
            bias = B.quantize_bias(bf, self.q[op.src], q_w)
            if op.src in self.unsigned:
                self.taps[name], bias = B.u8_prepare(self.desc[name], z_w, bias)
            self.wq[name] = (B.pack_weights(self.desc[name], z_w), bias)

    # ------------------------------------------------------------------ online step
    def allocate(self):
        for name, t in self.net.tensors.items():
            H, W = t.H, t.W
            if name == self.net.input and self.in_frame:
                H, W = self.in_frame[2:]
            self.act[name] = torch.zeros((self.N, H, W, _pad_c(t.C)), dtype=torch.int8,
                                         device=self.dev)
            if name in self.real:
                self.act_f32[name] = torch.zeros((self.N, H, W, _pad_c(t.C)),
                                                 dtype=torch.float32, device=self.dev)

    def input_codes(self):
        """The int8 codes of the network input without the frame: [N, H, W, C_stored]."""
        a = self.act[self.net.input]
        if not self.in_frame:
            return a
        t = self.net.tensors[self.net.input]
        top, left = self.in_frame[:2]
        return a[:, top:top + t.H, left:left + t.W]

    def quantize_input(self, x, lo=0, n=None):
        """Eq. Q on images [lo, lo + n) of the fp32 batch ``x`` into the input's codes."""
        n = self.N if n is None else n
        t = self.net.tensors[self.net.input]
        x = x[lo:lo + n]
        z = self.act[self.net.input][lo:lo + n]
        if self.in_frame:
            B.quantize_image(x, self.q[self.net.input], P_ACT, z, self.in_frame[0], self.in_frame[1])
        elif _pad_c(t.C) != t.C:
            B.quantize_pad_channels(x, _pad_c(t.C), self.q[self.net.input], P_ACT, out=z)
        else:
            B.quantize(x, self.q[self.net.input], P_ACT, out=z)

    def _dequant_writer(self, name):
        """The convolution that can write Eq. D of tensor ``name`` beside its codes, or None."""
        if not self.fuse_dequant or self.unsigned or self.per_channel or name in self.real:
            return None
        writers = [o for o in self.net.ops if o.dst == name]
        if len(writers) != 1 or writers[0].kind != "conv":
            return None
        o = writers[0]
        if o.dst_c_off or self.net.tensors[name].C != o.K or _pad_c(o.K) != o.K:
            return None
        if o.name in self.paired or o.name in self.dualed or o.name in self.pairs or o.name in self.duals:
            return None
        if self.head and o is self.head[0]:
            return None
        return o

    def set_input(self, x):
        """The real-valued batch of the next layers: with a fused head it is only remembered
        (the head's launches apply Eq. Q), otherwise Eq. Q runs on it now."""
        if self.head:
            self._x = x
        else:
            self.quantize_input(x)

    def run_head(self, lo, n):
        conv, pool = self.head
        packed, bias = self.wq[conv.name]
        dst = pool.dst if pool else conv.dst
        B.conv_image_f32(self.conv_desc(conv, n), self._x[lo:lo + n], self.in_frame[0],
                         self.in_frame[1], self.q[self.net.input], P_ACT, packed, bias,
                         self.qw[conv.name], self.q[conv.dst], pool=1 if pool else 0,
                         out=self.act[dst][lo:lo + n])

    def run_pool(self, op, lo=0, n=None):
        n = self.N if n is None else n
        s, d = self.net.tensors[op.src], self.net.tensors[op.dst]
        q_in, q_out = self.q[op.src], self.q[op.dst]
        src, dst = self.act[op.src][lo:lo + n], self.act[op.dst][lo:lo + n]
        if op.mode == "max" and q_in == q_out and _pad_c(d.C) == _pad_c(s.C):
            # exact copy of the maximum: the vectorised kernel
            B._check(B.lib.q8_maxpool_i8(src.data_ptr(), n, s.H, s.W, _pad_c(s.C), op.R, op.S,
                                         op.stride, op.pad, d.H, d.W, dst.data_ptr(),
                                         B._stream()))
        else:
            B.pool_i8(src, op.mode, op.R, op.S, op.stride, op.pad, d.H, d.W, q_in, q_out,
                      out=dst, out_c_off=op.dst_c_off)

    def conv_desc(self, op, n):
        """Descriptor of ``op`` over ``n`` images (the whole batch or one part of it)."""
        if n == self.N:
            return self.desc[op.name]
        key = (op.name, n)
        if key not in self.part_desc:
            self.part_desc[key] = self._desc(op, n)
        return self.part_desc[key]

    def run_conv(self, op, lo=0, n=None, acc_dump=None, fuse=True):
        n = self.N if n is None else n
        packed, bias = self.wq[op.name]
        res = self.act[op.res][lo:lo + n] if op.res else None
        q_res = self.q[op.res] if op.res else 0.0
        U = self.unsigned
        if (op.name in self.paired or op.name in self.dualed) and fuse:
            return                       # ran with the layer in front of it
        if op.name in self.duals and fuse:
            b = self.duals[op.name]

            def args(o):
                w, bias = self.wq[o.name]
                return (self.conv_desc(o, n), self.act[o.src][lo:lo + n], w, bias, self.q[o.src],
                        self.qw[o.name], self.q[o.dst],
                        self.act[o.res][lo:lo + n] if o.res else None,
                        self.q[o.res] if o.res else 0.0, self.act[o.dst][lo:lo + n])
            B.conv_dual_int8(args(op), args(b))
            return
        if op.name in self.pairs and fuse:
            b = self.pairs[op.name]
            packed2, bias2 = self.wq[b.name]
            res2 = self.act[b.res][lo:lo + n] if b.res else None
            B.conv_pair_int8(self.conv_desc(op, n), self.act[op.src][lo:lo + n], packed, bias,
                             self.q[op.src], self.qw[op.name], self.q[op.dst],
                             self.conv_desc(b, n), packed2, bias2, self.qw[b.name], self.q[b.dst],
                             res2, self.q[b.res] if b.res else 0.0,
                             out=self.act[b.dst][lo:lo + n])
            return
        if op.dst in self.real and acc_dump is None:
            B.conv_int8_real_output(self.conv_desc(op, n), self.act[op.src][lo:lo + n], packed,
                                    bias, self.q[op.src], self.qw[op.name], res, q_res,
                                    out=self.act_f32[op.dst][lo:lo + n])
            return
        if self.per_channel:
            B.conv_int8_per_channel(self.conv_desc(op, n), self.act[op.src][lo:lo + n], packed,
                                    bias, self.m_vec[op.name], self.q[op.dst], res, q_res,
                                    out=self.act[op.dst][lo:lo + n], acc_dump=acc_dump)
            return
        if op.src in U or op.dst in U or op.res in U:
            B.conv_u8(self.conv_desc(op, n), op.src in U, op.dst in U, op.res in U,
                      self.act[op.src][lo:lo + n], packed, bias, self.taps.get(op.name),
                      self.q[op.src], self.qw[op.name], self.q[op.dst], res, q_res,
                      out=self.act[op.dst][lo:lo + n], acc_dump=acc_dump)
            return
        if op.dst in self._deq and acc_dump is None:
            B.conv_int8_dequantized(self.conv_desc(op, n), self.act[op.src][lo:lo + n], packed, bias,
                                    self.q[op.src], self.qw[op.name], self.q[op.dst], res, q_res,
                                    out=self.act[op.dst][lo:lo + n],
                                    out_f32=self._deq[op.dst][lo:lo + n])
            return
        B.conv_int8(self.conv_desc(op, n), self.act[op.src][lo:lo + n], packed, bias,
                    self.q[op.src], self.qw[op.name], self.q[op.dst], res, q_res,
                    out=self.act[op.dst][lo:lo + n], acc_dump=acc_dump)

    def run_ops(self, ops, lo, n):
        for op in ops:
            if self._x is not None and self.head:
                if op is self.head[0]:
                    self.run_head(lo, n)
                    continue
                if op is self.head[1]:
                    continue             # ran inside the head's launch
            if op.kind == "pool":
                self.run_pool(op, lo, n)
            else:
                self.run_conv(op, lo, n)

    # ------------------------------------------------------------------ layer lists
    def _chainable(self, op):
        if op.kind != "conv" or op.dst_c_off != 0:
            return False
        s, d = self.net.tensors[op.src], self.net.tensors[op.dst]
        if d.C != op.K or s.C != op.C or (op.res and self.net.tensors[op.res].C != op.K):
            return False
        return B.conv_chain_supported(self.desc[op.name])

    def build_chains(self, variants=None):
        """Plan one q8_conv_chain_int8 launch per run of two or more chainable convolutions.
        ``variants`` ({conv name: tile variant}) forces tile shapes (tests, tuning)."""
        ops = self.net.ops
        self.chains = []
        i = 0
        while i < len(ops):
            j = i
            while j < len(ops) and self._chainable(ops[j]):
                j += 1
            if j - i >= 2:
                writer = {}
                layers = []
                for k, op in enumerate(ops[i:j]):
                    packed, bias = self.wq[op.name]
                    layers.append(dict(
                        desc=self.desc[op.name], z_x=self.act[op.src], w=packed, bias=bias,
                        q_x=self.q[op.src], q_w=self.qw[op.name], q_out=self.q[op.dst],
                        residual=self.act[op.res] if op.res else None,
                        q_res=self.q[op.res] if op.res else 0.0, out=self.act[op.dst],
                        src_layer=writer.get(op.src, -1),
                        res_layer=writer.get(op.res, -1) if op.res else -1,
                        variant=(variants or {}).get(op.name, -1)))
                    writer[op.dst] = k
                self.chains.append((i, j, B.ConvChain(layers, self.dev)))
                i = j
            else:
                i = max(j, i + 1)
        return self.chains

    def run_chained(self):
        """Every op on the whole batch: planned runs as one launch each, the rest one by one."""
        if self.chains is None:
            self.build_chains()
        ops = self.net.ops
        starts = {a: (b, c) for a, b, c in self.chains}
        i = 0
        while i < len(ops):
            if i in starts:
                end, ch = starts[i]
                ch.run()
                i = end
            else:
                self.run_ops([ops[i]], 0, self.N)
                i += 1

    def run_step(self, x=None, dequant=None, serial=False):
        """One pass over the batch: Eq. Q on ``x`` (if given), every layer, Eq. D on the
        tensors named in ``dequant`` ({name: fp32 output buffer}).  With two streams the
        layers of each half batch form a pipeline of their own between the (whole-batch)
        quantise and dequantise launches -- splitting those two as well was slower;
        ``serial`` issues the same launches one pipeline after the other on the caller's
        stream."""
        self._x = None
        if x is not None:
            self.set_input(x)
        # Eq. D inside the launch that writes the tensor, where there is such a launch
        self._deq = {name: out for name, out in (dequant or {}).items()
                     if out is not None and not self.chain and self._dequant_writer(name)}
        if self.chain:
            self.run_chained()
        elif self.n_streams == 1 or serial:
            for lo, n in self.parts:
                self.run_ops(self.net.ops, lo, n)
        else:
            main = torch.cuda.current_stream()
            for side in self.side:
                side.wait_stream(main)
            # layer by layer, alternating between the pipelines: a captured graph hands its
            # nodes to the GPU in the order they were recorded, and a pipeline recorded whole
            # before the next one starts that much earlier and runs alone meanwhile
            for op in self.net.ops:
                for side, part in zip(self.side, self.parts[1:]):
                    with torch.cuda.stream(side):
                        self.run_ops([op], *part)
                self.run_ops([op], *self.parts[0])
            for side in self.side:
                main.wait_stream(side)
        self._x = None
        done, self._deq = self._deq, {}
        for name, out in (dequant or {}).items():
            if name not in done:
                self.dequantize(name, out=out)

    def run_layers(self, acc_dump=None, serial=False):
        """Every layer on the codes already in the input buffer.  ``acc_dump``
        ({conv name: int32 buffer}): whole-batch launches that also store the accumulators."""
        if acc_dump:
            # every layer on its own in this pass (no fused pairs): a dumped layer needs its
            # input tensor written, whether or not the layer in front of it is dumped too
            for op in self.net.ops:
                if op.kind == "pool":
                    self.run_pool(op)
                else:
                    self.run_conv(op, acc_dump=acc_dump.get(op.name), fuse=False)
            return
        self.run_step(serial=serial)

    def dequantize(self, name, out=None, lo=0, n=None):
        """Eq. D on images [lo, lo + n) of tensor ``name`` (signed or unsigned codes); a
        real-valued output is already there."""
        n = self.N if n is None else n
        if out is not None:
            out = out[lo:lo + n]
        if name in self.real:
            if out is not None:
                out.copy_(self.act_f32[name][lo:lo + n])
                return out
            return self.act_f32[name][lo:lo + n]
        fn = B.dequantize_u8 if name in self.unsigned else B.dequantize
        return fn(self.act[name][lo:lo + n], self.q[name], out=out)

    def forward(self, x):
        """x: fp32 NHWC device tensor of the network input.  Returns the int8 outputs."""
        if not self.act:
            self.allocate()
        self.run_step(x)
        return [self.act[o] for o in self.net.outputs]

    def capture(self, x):
        """Record forward(x) into a HIP graph (x's storage is read at every replay)."""
        if not self.act:
            self.allocate()
        self.forward(x)                     # warm-up outside capture
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.forward(x)
        self.graph = g
        return g
