"""Pins of oracle.layer_graph (the detection network as one chain of quantized layers) against routines that
share nothing with it: the library's float64 convolution and max-pooling on the real values the levels stand for,
node by node, on a small instance of the graph; plus structural checks of the workload (shapes down to 1x1, every
level busy, heads read the right maps)."""
import numpy as np
import torch
import torch.nn.functional as F

import oracle
import qnn_workloads as wl


def _nchw(a):
    return torch.from_numpy(np.ascontiguousarray(a.transpose(0, 3, 1, 2)).astype(np.float64))


def _nhwc(t):
    return t.permute(0, 2, 3, 1).contiguous().numpy()


def test_small_detection_graph_against_library_float64_routines():
    bits = 3
    net = wl.vgg_ssd_chained(batch=1, bits=bits, image=75)
    # at 75 pixels the backbone ends at 5x5 and the last extra layers would shrink below 1x1: keep the nodes that
    # still have an output (all pooling variants, 1x1 / 3x3, stride 1 / 2, pad 0 / 1 and heads remain)
    nodes = []
    size = {"input": 75}
    for nd in net["nodes"]:
        s_in = size.get(nd["src"])
        if s_in is None:
            continue
        if nd["kind"] == "pool":
            s_out = oracle.pool_out_size(s_in, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"])
        else:
            s_out = (s_in + 2 * nd["pad"] - nd.get("dilation", 1) * (nd["k"] - 1) - 1) // nd["stride"] + 1
        if s_out < 1:
            continue
        size[nd["name"]] = s_out
        nodes.append(nd)
    assert len(nodes) >= 30 and any(n["head"] for n in nodes)
    got = oracle.layer_graph(net["x"], net["clip0"], bits, nodes)
    top = (1 << bits) - 1
    # independent evaluation: levels as float64 integers, library conv2d / max_pool2d
    lv0, _ = oracle.quantize(net["x"], net["clip0"], bits)
    ref = {"input": _nchw(lv0)}
    for nd in nodes:
        src = ref[nd["src"]]
        if nd["kind"] == "pool":
            if nd["ceil_mode"] or nd["pad"]:
                r = F.max_pool2d(src, nd["k"], nd["stride"], nd["pad"], ceil_mode=nd["ceil_mode"])
            else:
                r = F.max_pool2d(src, nd["k"], nd["stride"])
            ref[nd["name"]] = r
            assert np.array_equal(_nhwc(r), got[nd["name"]]["levels"].astype(np.float64)), nd["name"]
            continue
        w = torch.from_numpy(nd["w"].transpose(0, 3, 1, 2).astype(np.float64))
        acc = F.conv2d(src, w, stride=nd["stride"], padding=nd["pad"], dilation=nd.get("dilation", 1))
        assert np.array_equal(_nhwc(acc), got[nd["name"]]["acc"].astype(np.float64)), nd["name"]
        # the scale is one fp32 multiply of the exact integer; the next quantizer acts on that fp32 value
        out32 = (_nhwc(acc).astype(np.float32) * nd["scale"].astype(np.float32)[None, None, None, :]).astype(np.float32)
        assert np.array_equal(out32, got[nd["name"]]["out"]), nd["name"]
        if nd["head"]:
            assert got[nd["name"]]["levels"] is None
            continue
        # Eq. 15 in float64 on the fp32 value, away from thresholds; on them the fp32 sequence decides
        t = np.clip(out32.astype(np.float64) / nd["clip"], -1.0, 1.0)
        u = np.floor((t + 1.0) * top / 2.0 + 0.5)
        frac = (t + 1.0) * top / 2.0 + 0.5
        safe = np.abs(frac - np.round(frac)) > 1e-4
        lv = got[nd["name"]]["levels"].astype(np.float64)
        assert np.array_equal((2 * u - top)[safe], lv[safe]), nd["name"]
        ref[nd["name"]] = _nchw(lv)


def test_full_size_graph_shapes_and_busy_levels():
    bits = 4
    net = wl.vgg_ssd_chained(batch=1, bits=bits)
    names = [n["name"] for n in net["nodes"]]
    assert names[:4] == ["conv1_2", "pool1", "conv2_1", "conv2_2"] and "conv11_2" in names
    assert sum(n["kind"] == "conv" and not n["head"] for n in net["nodes"]) == 12 + 10
    assert sum(n["head"] for n in net["nodes"]) == 12
    size, chans = {"input": 300}, {"input": 64}
    for nd in net["nodes"]:
        s_in = size[nd["src"]]
        if nd["kind"] == "pool":
            size[nd["name"]] = oracle.pool_out_size(s_in, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"])
            chans[nd["name"]] = chans[nd["src"]]
        else:
            assert nd["cin"] == chans[nd["src"]], nd["name"]
            size[nd["name"]] = (s_in + 2 * nd["pad"] - nd.get("dilation", 1) * (nd["k"] - 1) - 1) // nd["stride"] + 1
            chans[nd["name"]] = nd["cout"]
    assert [size[k] for k in ("pool1", "pool2", "pool3", "pool4", "pool5", "conv8_2", "conv9_2", "conv10_2", "conv11_2")] \
        == [150, 75, 38, 19, 19, 10, 5, 3, 1]
    assert size["loc_conv4_3"] == 38 and chans["loc_conv4_3"] == 16 and chans["conf_conv7"] == 126
    # the backbone's first half on a crop keeps every level busy and saturates only a little
    crop = wl.vgg_ssd_chained(batch=1, bits=bits, image=64, heads=False)
    vals = oracle.layer_graph(crop["x"], crop["clip0"], bits, crop["nodes"][:9])
    for name in ("conv1_2", "conv2_2", "conv3_3"):
        lv = vals[name]["levels"]
        assert set(np.unique(lv).tolist()) == set(range(-15, 16, 2)), name
        assert (np.abs(lv) == 15).mean() < 0.1, name
