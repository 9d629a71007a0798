"""GPU parity of the detection network run as ONE chain (wl.vgg_ssd_chained: the VGG16 backbone's twelve convolutions
joined by max-pooling on the codes, the SSD-style extra layers down to 1x1, localisation / class heads on six maps)
against oracle.layer_graph, on both machine routes:

  planes: qnn_encode_pack -> qnn_conv2d / qnn_conv2d_dilated (fused next-layer planes) / qnn_maxpool_planes; heads write fp32
  levels: qnn_encode_levels_i8 -> qnn_level_conv2d_i8 / qnn_level_conv2d_dilated_i8 / qnn_maxpool_levels_i8

batch 1: every accumulator, every plane / level tensor, every fp32 head output; batch 32 (the benchmark's): every
plane / level tensor between layers and every head output, in the fused configuration the benchmark times."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, pack_levels, planes_to_numpy

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

RTOL = 1e-5


def run_graph_planes(net, keep_acc):
    """The graph on the xor + bitcount route.  Returns {name: (planes or None, acc or None, out or None, C)}."""
    bits, x = net["bits"], net["x"]
    B, H, W, C = x.shape
    vals = {"input": (qnn.qnn_encode_pack(dev(x), net["clip0"], bits), None, None, (H, W, C))}
    for nd in net["nodes"]:
        planes, _, _, (H, W, C) = vals[nd["src"]]
        if nd["kind"] == "pool":
            out = qnn.qnn_maxpool_planes(planes, (B, H, W), C, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"])
            ho = qnn.qnn_pool_out_size(H, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"])
            vals[nd["name"]] = (out, None, None, (ho, ho, C))
            continue
        k = nd["k"]
        wp = pack_levels(nd["w"], bits).view(bits, nd["cout"], k, k, -1)
        dil = nd.get("dilation", 1)
        ho = (H + 2 * nd["pad"] - dil * (k - 1) - 1) // nd["stride"] + 1
        head = nd["head"]
        # above 4 bits the plane-chunk launches keep their running sum in acc
        kw = dict(scale=dev(nd["scale"]), want_acc=keep_acc or bits > 4, want_out=head,
                  next_clip=None if head else nd["clip"], next_bits=0 if head else bits)
        if dil == 1:
            acc, out, nxt = qnn.qnn_conv2d(planes, wp, (B, H, W), C, nd["stride"], nd["pad"], **kw)
        else:
            acc, out, nxt = qnn.qnn_conv2d_dilated(planes, wp, (B, H, W), C, nd["stride"], nd["pad"], dil, **kw)
        vals[nd["name"]] = (nxt, acc if keep_acc else None, out, (ho, ho, nd["cout"]))
    torch.cuda.synchronize()
    return vals


def run_graph_levels(net, keep_acc):
    """The same graph on the matrix-core route: int8 levels between layers."""
    bits, x = net["bits"], net["x"]
    vals = {"input": (qnn.qnn_encode_levels_i8(dev(x), net["clip0"], bits), None, None)}
    for nd in net["nodes"]:
        lv = vals[nd["src"]][0]
        if nd["kind"] == "pool":
            vals[nd["name"]] = (qnn.qnn_maxpool_levels_i8(lv, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"]), None, None)
            continue
        head = nd["head"]
        kw = dict(scale=dev(nd["scale"]), want_acc=keep_acc, want_out=head, next_clip=None if head else nd["clip"],
                  next_bits=0 if head else bits)
        if nd.get("dilation", 1) == 1:
            acc, out, nxt = qnn.qnn_level_conv2d_i8(lv, dev(nd["w"]), nd["stride"], nd["pad"], bits, bits, **kw)
        else:
            acc, out, nxt = qnn.qnn_level_conv2d_dilated_i8(lv, dev(nd["w"]), nd["stride"], nd["pad"], nd["dilation"], bits,
                                                            bits, **kw)
        vals[nd["name"]] = (nxt, acc, out)
    torch.cuda.synchronize()
    return vals


def _check(net, got, want, route, accs):
    bits = net["bits"]
    for nd in [{"name": "input", "kind": "input", "head": False}] + net["nodes"]:
        name = nd["name"]
        g, o = got[name], want[name]
        if o["levels"] is not None:
            if route == "planes":
                C = o["levels"].shape[-1]
                assert np.array_equal(planes_to_numpy(g[0]), oracle.pack_planes(o["levels"].reshape(-1, C), bits)), name
            else:
                assert np.array_equal(g[0].cpu().numpy(), o["levels"].astype(np.int8)), name
        if accs and o["acc"] is not None:
            assert np.array_equal(g[1].cpu().numpy(), o["acc"]), name
        if nd["head"]:
            np.testing.assert_allclose(g[2].cpu().numpy(), o["out"], rtol=RTOL, atol=0, err_msg=name)


@pytest.mark.parametrize("bits", [4, 5])
@pytest.mark.parametrize("route", ["planes", "levels"])
def test_batch_1_every_accumulator(route, bits):
    print("detection graph, batch 1, %d bit, %s" % (bits, route), flush=True)
    net = wl.vgg_ssd_chained(batch=1, bits=bits)
    want = oracle.layer_graph(net["x"], net["clip0"], bits, net["nodes"])
    got = (run_graph_planes if route == "planes" else run_graph_levels)(net, keep_acc=True)
    _check(net, got, want, route, accs=True)
    # the heads see real scores: unit-variance-ish, not collapsed
    assert 0.2 < float(np.std(want["conf_conv4_3"]["out"])) < 5.0


@pytest.fixture(scope="module")
def full_batch():
    net = wl.vgg_ssd_chained(batch=32, bits=4)
    print("oracle: detection graph at batch 32", flush=True)
    want = oracle.layer_graph(net["x"], net["clip0"], 4, net["nodes"])
    for v in want.values():
        v["acc"] = None                      # keep the levels and the head outputs only
    return net, want


@pytest.mark.parametrize("route", ["planes", "levels"])
def test_batch_32_every_tensor_between_layers(full_batch, route):
    net, want = full_batch
    print("detection graph, batch 32, 4 bit, %s" % route, flush=True)
    got = (run_graph_planes if route == "planes" else run_graph_levels)(net, keep_acc=False)
    _check(net, got, want, route, accs=False)
    del got
    torch.cuda.empty_cache()
