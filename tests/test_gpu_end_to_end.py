"""GPU parity of the whole image -> logits graph that `bench.py --workload trunk` times as its "network" step
(the ResNet-18 of the experiments section with its first convolution and classifier unquantized):

    image -> fp32 first convolution with scale, shift, ReLU and the first quantizer fused (planes or levels out)
          -> 3x3 stride-2 max-pooling of the codes -> residual trunk (8 blocks) -> global average pooling -> classifier

on both machine routes, at batch 4, in one chain on one input.

The first convolution's fp32 sums are in the kernel's own order, so its value is bounded against the float64
oracle (worst case of recursive summation) and the first quantizer's decision is taken on the kernel's fp32 value:
the oracle chain is seeded with the oracle quantizer applied to that value.  Every code where this differs from
the code of the float64 oracle's value is counted and must be explained by the bound (the float64 value lies
within the bound of a threshold of the ladder).  From there on everything is exact: every plane / level tensor
between layers must equal the oracle chain bit for bit, the trunk's fp32 output to 1e-5 relative, and the logits
must lie within the summation bound of the pooling and the classifier."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import codes_explained_by_bound, dev, pack_levels, planes_to_numpy

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

U = 2.0 ** -24
RTOL = 1e-5
BITS = 3
BATCH = 4


def _oracle_tail(pooled_levels, net, ends, clip0):
    """The oracle's chain from the pooled codes on: trunk (seeded with the real values of the codes), average
    pooling and classifier in float64."""
    top = (1 << BITS) - 1
    x = (pooled_levels.astype(np.float32) * np.float32(clip0)) / np.float32(top)   # the real value of a level
    relv, _ = oracle.quantize(x, clip0, BITS)
    assert np.array_equal(relv, pooled_levels)            # the trunk's first quantizer returns the same codes
    trace = oracle.residual_trunk(x, net["blocks"])
    y = trace[-1]["y"]
    feat = oracle.global_avgpool(y)
    logits, mag = oracle.dense_fc(feat, ends["fc_w"], ends["fc_b"])
    hw = y.shape[1] * y.shape[2]
    feat_bound = (hw + 2) * U * np.abs(y.astype(np.float64)).sum(axis=(1, 2)) / hw \
        + RTOL * np.abs(y.astype(np.float64)).mean(axis=(1, 2))            # the trunk's output itself is held to RTOL
    bound = (ends["fc_w"].shape[1] + 4) * U * mag + feat_bound @ np.abs(ends["fc_w"].astype(np.float64)).T + 1e-30
    return trace, feat, logits, bound


def _trunk_planes(a, net, B, H, W, C):
    blocks, out = net["blocks"], []
    for bi, blk in enumerate(blocks):
        c1, c2, dn = blk["conv1"], blk["conv2"], blk["down"]
        last = bi + 1 == len(blocks)
        cout, st = c1["cout"], c1["stride"]
        Ho, Wo = (H + 2 - 3) // st + 1, (W + 2 - 3) // st + 1
        wp = lambda L, k: pack_levels(L["w"], BITS).view(BITS, L["cout"], k, k, -1)
        _, _, hq = qnn.qnn_conv2d_block(a, wp(c1, 3), (B, H, W), C, st, 1, dev(c1["scale"]), bias=dev(c1["bias"]),
                                        want_acc=False, next_clip=c2["clip"], next_bits=BITS)
        if dn is not None:
            _, short, _ = qnn.qnn_conv2d_block(a, wp(dn, 1), (B, H, W), C, st, 0, dev(dn["scale"]), bias=dev(dn["bias"]),
                                               want_acc=False, want_out=True)
            kw = {"res_f32": short}
        else:
            kw = {"res_planes": a, "res_scale": blk["res_scale"]}
        _, y, nxt = qnn.qnn_conv2d_block(hq, wp(c2, 3), (B, Ho, Wo), cout, 1, 1, dev(c2["scale"]), bias=dev(c2["bias"]),
                                         want_acc=False, want_out=last, next_clip=None if last else blocks[bi + 1]["conv1"]["clip"],
                                         next_bits=0 if last else BITS, **kw)
        out.append({"a": a, "hq": hq, "y": y, "C": C, "cout": cout})
        a, H, W, C = nxt, Ho, Wo, cout
    return out


def _trunk_levels(a, net):
    blocks, out = net["blocks"], []
    for bi, blk in enumerate(blocks):
        c1, c2, dn = blk["conv1"], blk["conv2"], blk["down"]
        last = bi + 1 == len(blocks)
        st = c1["stride"]
        _, _, hq = qnn.qnn_level_conv2d_block_i8(a, dev(c1["w"]), st, 1, BITS, BITS, dev(c1["scale"]), bias=dev(c1["bias"]),
                                                 want_acc=False, next_clip=c2["clip"], next_bits=BITS)
        if dn is not None:
            _, short, _ = qnn.qnn_level_conv2d_block_i8(a, dev(dn["w"]), st, 0, BITS, BITS, dev(dn["scale"]),
                                                        bias=dev(dn["bias"]), want_acc=False, want_out=True)
            kw = {"res_f32": short}
        else:
            kw = {"res_levels": a, "res_bits": BITS, "res_scale": blk["res_scale"]}
        _, y, nxt = qnn.qnn_level_conv2d_block_i8(hq, dev(c2["w"]), 1, 1, BITS, BITS, dev(c2["scale"]), bias=dev(c2["bias"]),
                                                  want_acc=False, want_out=last,
                                                  next_clip=None if last else blocks[bi + 1]["conv1"]["clip"],
                                                  next_bits=0 if last else BITS, **kw)
        out.append({"a": a, "hq": hq, "y": y})
        a = nxt
    return out


@pytest.fixture(scope="module")
def graph():
    net = wl.resnet18_trunk(batch=BATCH, bits=BITS)
    ends = wl.resnet18_ends(batch=BATCH)
    clip0 = net["blocks"][0]["conv1"]["clip"]
    stem64, mag = oracle.dense_layer(ends["image"], ends["stem_w"], 2, 3, ends["stem_scale"], ends["stem_shift"], True)
    return net, ends, clip0, stem64, (147 + 4) * U * mag + 1e-30


@pytest.mark.parametrize("route", ["planes", "levels"])
def test_image_to_logits(graph, route):
    net, ends, clip0, stem64, stem_bound = graph
    img, w0, s0, b0 = (dev(ends[k]) for k in ("image", "stem_w", "stem_scale", "stem_shift"))
    print("route %s: first convolution" % route, flush=True)
    if route == "planes":
        stem32, stem_q = qnn.qnn_dense_conv2d_f32(img, w0, 2, 3, scale=s0, shift=b0, relu=True, want_out=True,
                                                  next_clip=clip0, next_bits=BITS)
    else:
        stem32, stem_q = qnn.qnn_dense_conv2d_f32_levels(img, w0, 2, 3, clip0, BITS, scale=s0, shift=b0, relu=True,
                                                         want_out=True)
    torch.cuda.synchronize()
    got32 = stem32.cpu().numpy()
    side = got32.shape[1]
    assert (np.abs(got32.astype(np.float64) - stem64) <= stem_bound).all()
    seed_levels, _ = oracle.quantize(got32, clip0, BITS)       # the decision is taken on the kernel's fp32 value
    flipped = codes_explained_by_bound(got32, stem64, stem_bound, clip0, BITS)
    print("route %s: %d of %d first-layer codes differ from the float64 oracle's, all within the bound of a threshold"
          % (route, flipped, seed_levels.size), flush=True)
    assert flipped <= seed_levels.size // 1000
    if route == "planes":
        assert np.array_equal(planes_to_numpy(stem_q), oracle.pack_planes(seed_levels.reshape(-1, 64), BITS))
        pooled = qnn.qnn_maxpool_planes(stem_q, (BATCH, side, side), 64, 3, 2, 1)
    else:
        assert np.array_equal(stem_q.cpu().numpy(), seed_levels.astype(np.int8))
        pooled = qnn.qnn_maxpool_levels_i8(stem_q, 3, 2, 1)
    want_pool = oracle.maxpool(seed_levels, 3, 2, 1)
    H = want_pool.shape[1]
    assert H == net["x"].shape[1]
    print("route %s: trunk" % route, flush=True)
    got = _trunk_planes(pooled, net, BATCH, H, H, 64) if route == "planes" else _trunk_levels(pooled, net)
    feat = qnn.qnn_global_avgpool_f32(got[-1]["y"])
    logits = qnn.qnn_dense_fc_f32(feat, dev(ends["fc_w"]), dev(ends["fc_b"]))
    torch.cuda.synchronize()
    trace, want_feat, want_logits, bound = _oracle_tail(want_pool, net, ends, clip0)
    for bi, (g, o) in enumerate(zip(got, trace)):
        if route == "planes":
            assert np.array_equal(planes_to_numpy(g["a"]), oracle.pack_planes(o["a"].reshape(-1, g["C"]), BITS)), bi
            assert np.array_equal(planes_to_numpy(g["hq"]), oracle.pack_planes(o["hq"].reshape(-1, g["cout"]), BITS)), bi
        else:
            assert np.array_equal(g["a"].cpu().numpy(), o["a"].astype(np.int8)), bi
            assert np.array_equal(g["hq"].cpu().numpy(), o["hq"].astype(np.int8)), bi
    np.testing.assert_allclose(got[-1]["y"].cpu().numpy(), trace[-1]["y"], rtol=RTOL, atol=0)
    err = np.abs(logits.cpu().numpy().astype(np.float64) - want_logits)
    assert logits.shape == (BATCH, 1000) and (err <= bound).all(), float((err / bound).max())
    # the logits are not degenerate: every image has its own, spread over the classes
    assert np.std(want_logits) > 0.05 and len({int(i) for i in want_logits.argmax(axis=1)}) >= 2
