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
