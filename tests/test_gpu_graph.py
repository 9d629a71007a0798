"""The entry points only enqueue work on the caller's stream (no allocation, no synchronisation),
so a chain of them can be captured into a HIP graph: capture one fused stack step, replay it several
times with eager work and synchronisations in between, and compare every replay with the eager result."""
import numpy as np
import pytest
import torch

import qnn_workloads as wl

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402


def _plan(c, bits):
    x = torch.from_numpy(c["x"]).cuda()
    layers = c["layers"]
    B, H, W, C = c["x"].shape
    first = torch.empty((bits, B * H * W, C // 32), dtype=torch.int32, device="cuda")
    cur, h, steps = first, H, []
    for li, L in enumerate(layers):
        wp = qnn.qnn_encode_pack(torch.from_numpy(L["w"]).cuda(), 1.0, bits).view(bits, L["cout"], 3, 3, -1)
        ho = (h + 2 - 3) // L["stride"] + 1
        last = li + 1 == len(layers)
        nxt = None if last else torch.empty((bits, B * ho * ho, L["cout"] // 32), dtype=torch.int32, device="cuda")
        out = torch.empty((B, ho, ho, L["cout"]), dtype=torch.float32, device="cuda") if last else None
        steps.append((cur, wp, (B, h, h), L, torch.from_numpy(L["scale"]).cuda(), out, nxt,
                      None if last else layers[li + 1]))
        cur, h = nxt, ho

    def step():
        qnn.qnn_encode_pack(x, layers[0]["clip"], bits, planes=first)
        for planes, wp, shape, L, sc, out, nxt, Ln in steps:
            qnn.qnn_conv2d(planes, wp, shape, L["cin"], L["stride"], L["pad"], scale=sc, want_acc=False,
                           want_out=out is not None, out=out, next_clip=None if Ln is None else Ln["clip"],
                           next_bits=0 if Ln is None else bits, next_planes=nxt)
    return step, steps[-1][5], x


def test_fused_stack_step_in_a_hip_graph():
    c = wl.resnet18_stack(batch=2)
    step, out, x = _plan(c, 3)
    step()
    torch.cuda.synchronize()
    ref = out.clone()
    side = torch.cuda.Stream()                 # warm up on a side stream, as graph capture asks for
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        out.fill_(float(rep))                  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), rep
    # new input through the same graph: the captured pointers are read at replay time
    x.mul_(-1.0)
    graph.replay()
    step_out = out.clone()
    step()
    torch.cuda.synchronize()
    assert torch.equal(out, step_out) and not torch.equal(out, ref)


def test_block_deconv_and_gradient_calls_in_a_hip_graph():
    # the later entry points under capture: a residual block (shift + shortcut planes), a transposed
    # convolution on its output planes (one launch over its four phases), and the two training-side gradients
    gen = np.random.default_rng(3)
    B, H, C, bits = 2, 10, 64, 2
    x = torch.from_numpy(gen.normal(0, 1, size=(B * H * H, C)).astype(np.float32)).cuda()
    top = (1 << bits) - 1
    lv = lambda shape: torch.from_numpy((2 * gen.integers(0, top + 1, size=shape) - top).astype(np.int8)).cuda()
    w1 = qnn.qnn_encode_pack(lv((C, 3, 3, C)), 1.0, bits).view(bits, C, 3, 3, -1)
    ph = qnn.qnn_deconv_pack_weights(qnn.qnn_encode_pack(lv((32, 4, 4, C)), 1.0, bits).view(bits, 32, 4, 4, -1), C, 2)
    sc1 = torch.full((C,), 0.02, device="cuda")
    sc2 = torch.full((32,), 0.03, device="cuda")
    bias = torch.from_numpy(gen.uniform(-0.2, 0.2, size=C).astype(np.float32)).cuda()
    planes = torch.empty((bits, B * H * H, C // 32), dtype=torch.int32, device="cuda")
    mid = torch.empty_like(planes)
    out = torch.empty((B, 2 * H, 2 * H, 32), dtype=torch.float32, device="cuda")
    g = torch.from_numpy(gen.normal(size=(bits, B * H * H * C)).astype(np.float32)).cuda()
    gx, gq = torch.empty(B * H * H * C, device="cuda"), torch.empty(B * H * H * C, device="cuda")

    def step():
        qnn.qnn_encode_pack(x, 3.0, bits, planes=planes)
        qnn.qnn_conv2d_block(planes, w1, (B, H, H), C, 1, 1, sc1, bias=bias, res_planes=planes, res_scale=0.5,
                             want_acc=False, next_clip=3.0, next_bits=bits, next_planes=mid)
        qnn.qnn_deconv2d(mid, ph, (B, H, H), C, 32, 4, 4, 2, 1, bits, scale=sc2, want_acc=False, want_out=True, out=out)
        qnn.qnn_encoder_backward(x.view(-1), g, 3.0, grad_x=gx)
        qnn.qnn_quantize_ste_backward(x.view(-1), g[0], 3.0, grad_x=gq)

    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (out, gx, gq)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in (out, gx, gq, mid):
            t.fill_(rep)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip((out, gx, gq), ref)), rep


def test_network_ends_and_one_launch_layer_in_a_hip_graph():
    # fp32 first convolution with planes out -> pooling of the planes; average pooling -> fp32 classifier;
    # and the one-launch quantized layer: captured together, replayed with eager work in between
    gen = np.random.default_rng(5)
    B, bits = 2, 2
    img = torch.from_numpy(gen.normal(size=(B, 32, 32, 3)).astype(np.float32)).cuda()
    w0 = torch.from_numpy((gen.normal(size=(64, 7, 7, 3)) / 12).astype(np.float32)).cuda()
    sc, sh = torch.full((64,), 1.1, device="cuda"), torch.full((64,), -0.1, device="cuda")
    planes = torch.empty((bits, B * 16 * 16, 2), dtype=torch.int32, device="cuda")
    pooled = torch.empty((bits, B * 8 * 8, 2), dtype=torch.int32, device="cuda")
    feat_in = torch.from_numpy(gen.normal(size=(B, 7, 7, 96)).astype(np.float32)).cuda()
    feat, logits = torch.empty((B, 96), device="cuda"), torch.empty((B, 10), device="cuda")
    fc_w = torch.from_numpy(gen.normal(size=(10, 96)).astype(np.float32)).cuda()
    fc_b = torch.from_numpy(gen.normal(size=10).astype(np.float32)).cuda()
    top = (1 << bits) - 1
    a = torch.from_numpy((2 * gen.integers(0, top + 1, size=(6, 200)) - top).astype(np.int8)).cuda()
    wq = qnn.qnn_encode_pack(torch.from_numpy((2 * gen.integers(0, top + 1, size=(33, 200)) - top).astype(np.int8)).cuda(), 1.0, bits)
    acc = torch.empty((6, 33), dtype=torch.int32, device="cuda")

    def step():
        qnn.qnn_dense_conv2d_f32(img, w0, 2, 3, scale=sc, shift=sh, relu=True, want_out=False, next_clip=3.0,
                                 next_bits=bits, next_planes=planes)
        qnn.qnn_maxpool_planes(planes, (B, 16, 16), 64, 3, 2, 1, out=pooled)
        qnn.qnn_global_avgpool_f32(feat_in, out=feat)
        qnn.qnn_dense_fc_f32(feat, fc_w, fc_b, out=logits)
        qnn.qnn_fc_fused(a, 1.0, bits, wq, acc=acc)

    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (pooled, logits, acc)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in (planes, pooled, feat, logits, acc):
            t.fill_(rep)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(x, y) for x, y in zip((pooled, logits, acc), ref)), rep
