"""A whole quantized network assembled from the entry points -- convolutions with the fused
next-layer epilogue, max-pooling on the codes, fully connected layers as binary GEMMs -- against the
same chain of oracle primitives.  Shape: the CIFAR-10 network of the paper's Table 3 from its second
layer on, at 1 and 2 bits (the widths that table reports), on both machine routes."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, pack_levels, planes_to_numpy

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402


def _oracle_network(x, ops):
    """quantize -> op -> scale per weighted layer; pooling acts on the quantized levels.
    Returns the list of level tensors entering every op and the final fp32 output."""
    cur, lv, trace = np.ascontiguousarray(x), None, []
    for i, op in enumerate(ops):
        if op["kind"] == "pool":
            if lv is None:
                raise ValueError("pooling needs quantized input")
            trace.append(lv)
            lv = oracle.maxpool(lv, op["k"], op["stride"])
            continue
        if lv is None:
            lv, _ = oracle.quantize(cur, op["clip"], op["a_bits"])
        trace.append(lv)
        if op["kind"] == "conv":
            acc = oracle.conv2d(lv.astype(np.int8), op["w"], op["stride"], op["pad"])
        else:
            acc = oracle.gemm(lv.reshape(lv.shape[0], -1).astype(np.int8), op["w"])
        cur, lv = oracle.scale(acc, op["scale"]), None
        nxt = ops[i + 1:]
        nxt_w = next((o for o in nxt if o["kind"] != "pool"), None)
        if nxt and nxt[0]["kind"] == "pool":
            # the quantizer of the next weighted layer is applied before the pooling (on codes)
            lv, _ = oracle.quantize(cur, nxt_w["clip"], nxt_w["a_bits"])
    return trace, cur


def _next_weighted(ops, i):
    return next((o for o in ops[i + 1:] if o["kind"] != "pool"), None)


@pytest.mark.parametrize("bits", [1, 2])
def test_cifar_network_binary_route(bits):
    net = wl.cifar_vgg_network(batch=4, bits=bits)
    ops = net["ops"]
    B, H, W, C = net["x"].shape
    planes = qnn.qnn_encode_pack(dev(net["x"]), ops[0]["clip"], bits)      # [bits][B*H*W][cw]
    got, out = [], None
    for i, op in enumerate(ops):
        got.append((planes, C))
        nw_op = _next_weighted(ops, i)
        if op["kind"] == "pool":
            planes = qnn.qnn_maxpool_planes(planes, (B, H, W), C, op["k"], op["stride"])
            H, W = H // 2, W // 2
        elif op["kind"] == "conv":
            wp = pack_levels(op["w"], bits).view(bits, op["cout"], 3, 3, -1)
            _, _, planes = qnn.qnn_conv2d(planes, wp, (B, H, W), C, 1, 1, scale=dev(op["scale"]), want_acc=False,
                                          next_clip=nw_op["clip"], next_bits=bits)
            C = op["cout"]
        else:
            n = op["n"]
            a = planes.view(bits, B, n // 32)            # NHWC flatten = the plane layout itself
            _, out = qnn.qnn_binary_gemm(a, pack_levels(op["w"], bits), n, want_acc=False, scale=dev(op["scale"]))
            if nw_op is not None:
                planes = qnn.qnn_encode_pack(out, nw_op["clip"], bits)
            H = W = 1
            C = op["cout"]
    torch.cuda.synchronize()
    want, want_out = _oracle_network(net["x"], ops)
    assert len(want) == len(got)
    for i, ((p, c), lv) in enumerate(zip(got, want)):
        assert np.array_equal(planes_to_numpy(p).reshape(bits, -1, (c + 31) // 32),
                              oracle.pack_planes(lv.reshape(-1, c), bits)), i
    np.testing.assert_allclose(out.cpu().numpy(), want_out, rtol=1e-5, atol=0)
    assert want_out.shape == (4, 10)


@pytest.mark.parametrize("bits", [1, 2])
def test_cifar_network_matrix_core_route(bits):
    net = wl.cifar_vgg_network(batch=4, bits=bits)
    ops = net["ops"]
    lv = qnn.qnn_encode_levels_i8(dev(net["x"]), ops[0]["clip"], bits)
    got, out = [], None
    for i, op in enumerate(ops):
        got.append(lv)
        nw_op = _next_weighted(ops, i)
        if op["kind"] == "pool":
            lv = qnn.qnn_maxpool_levels_i8(lv, op["k"], op["stride"])
        elif op["kind"] == "conv":
            _, _, lv = qnn.qnn_level_conv2d_i8(lv, dev(op["w"]), 1, 1, bits, bits, scale=dev(op["scale"]),
                                               want_acc=False, next_clip=nw_op["clip"], next_bits=bits)
        else:
            n = op["n"]
            assert n == qnn.qnn_level_row_bytes(n)       # rows need no padding here
            _, out = qnn.qnn_level_gemm_i8(lv.view(lv.shape[0], n), dev(op["w"]), n, want_acc=False,
                                           scale=dev(op["scale"]))
            if nw_op is not None:
                lv = qnn.qnn_encode_levels_i8(out, nw_op["clip"], bits)
    torch.cuda.synchronize()
    want, want_out = _oracle_network(net["x"], ops)
    for i, (g, o) in enumerate(zip(got, want)):
        assert np.array_equal(g.cpu().numpy().reshape(o.shape), o.astype(np.int8)), i
    np.testing.assert_allclose(out.cpu().numpy(), want_out, rtol=1e-5, atol=0)
