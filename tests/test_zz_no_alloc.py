"""The entry point that allocates nothing: q8_conv_chain_int8_static runs a layer list on the
workspace that lives inside the library's device image.  Its output must equal that of
q8_conv_chain_int8 (caller-provided workspace) bit for bit, on two calls in a row, the second
on a smaller input (the shared array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_1805_08691_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _engine(batch):
    from paper_1805_08691_amd.engine import Engine
    net = wl.CONFIGS[2]["make"]()                     # bottleneck block: three layers + fused sum
    params = {op.name: wl.conv_params(2, i, op) for i, op in enumerate(net.convs())}
    eng = Engine(net, batch, chain=True)
    eng.load_params(params)
    eng.fold()
    eng.calibrate([torch.from_numpy(wl.input_batch(2, net, 4, 100, relu=True)).cuda()])
    eng.quantize_weights()
    eng.allocate()
    chains = eng.build_chains()
    assert len(chains) == 1
    x = torch.from_numpy(wl.input_batch(2, net, batch, 0, relu=True)).cuda()
    eng.quantize_input(x)
    return eng, net, chains[0][2]


def test_static_workspace_entry_equals_the_workspace_entry():
    from paper_1805_08691_amd import binding as B
    limit = B.lib.q8_conv_chain_static_workspace_limit()
    for batch in (21, 5):                             # the second call is the smaller one
        eng, net, chain = _engine(batch)
        assert chain.ws.numel() * 4 <= limit
        chain.run()
        torch.cuda.synchronize()
        assert chain.status() == 0
        want = {n: t.clone() for n, t in eng.act.items()}
        for n, t in eng.act.items():
            if n != net.input:
                t.fill_(-7)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        chain.run_static()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert B.ConvChain.static_status() == 0
        for n, t in eng.act.items():
            assert torch.equal(t, want[n]), (batch, n)
        assert len(torch.unique(eng.act[net.outputs[0]])) > 32    # not degenerate


def test_static_workspace_entry_refuses_a_plan_beyond_its_limit():
    from paper_1805_08691_amd import binding as B
    # a single-layer-pair list at a batch whose completion counters exceed 1 MiB
    import ctypes as C
    n_img = 4096
    base = 0x7F0000000000
    arr = (B.ChainLayer * 2)()
    for i in range(2):
        a = arr[i]
        a.d = B.ConvDesc(n_img, 56, 56, 64, 64, 1, 1, relu=1)
        a.z_x, a.z_y = base + i * (1 << 36), base + (i + 1) * (1 << 36)
        a.z_w_packed, a.bias_i32 = 0x100000 + i * 0x100000, 0x10000
        a.q_x = a.q_w = a.q_out = 0.5
        a.residual, a.src_layer, a.res_layer, a.variant = None, i - 1, -1, 3
    n = B.lib.q8_conv_chain_plan_bytes(arr, 2)
    assert n > 0
    buf = C.create_string_buffer(n)
    assert B.lib.q8_conv_chain_plan(arr, 2, buf, n) == 0
    assert B.lib.q8_conv_chain_workspace_bytes(buf) > B.lib.q8_conv_chain_static_workspace_limit()
    # refused on the host: nothing is launched, no device memory is touched
    assert B.lib.q8_conv_chain_int8_static(buf, C.c_void_p(0x7F2000000000), None) == -5
