"""GPU parity of the residual-block epilogue (qnn_conv2d_block, qnn_level_conv2d_block_i8): a per-channel
shift and a shortcut term -- quantized or fp32 -- between the scale factor and the next quantizer,
against the CPU oracle; then a ResNet-18-shaped trunk of such blocks on both machine routes."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, pack_levels, planes_to_numpy, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

RTOL = 1e-5

GEOMS = [
    # B, H, W, Cin, Cout, k, stride, pad
    (2, 7, 9, 16, 4, 3, 1, 1),
    (1, 8, 8, 32, 6, 3, 2, 1),       # Cout not a multiple of 4: scalar stores and loads
    (2, 6, 5, 48, 37, 1, 1, 0),      # 1x1, ragged word of shortcut planes
    (1, 9, 7, 48, 70, 5, 1, 2),      # three words of shortcut planes, the last ragged
    (2, 14, 14, 128, 132, 3, 1, 1),  # several column tiles
    (5, 13, 13, 64, 64, 3, 1, 1),    # several row tiles, ragged tail
]
TERMS = ["bias", "res_q", "res_f32", "bias+res_q", "bias+res_f32", "all"]


def _terms(gen, which, shape, res_bits):
    cout = shape[-1]
    bias = gen.uniform(-1, 1, size=cout).astype(np.float32) if "bias" in which or which == "all" else None
    res_lv = levels(gen, shape, res_bits) if "res_q" in which or which == "all" else None
    res_f = gen.normal(0, 1, size=shape).astype(np.float32) if "res_f32" in which or which == "all" else None
    return bias, res_lv, np.float32(0.37), res_f


def _opt(a):
    return None if a is None else dev(a)


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("which", TERMS)
@pytest.mark.parametrize("bits", [(2, 2, 2), (3, 3, 4), (4, 4, 1), (1, 2, 8)])
def test_block_terms_binary_route(geom, which, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits, res_bits = bits
    gen = np.random.default_rng(sum(geom) * 7 + sum(bits) + len(which))
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    var = (4.0 ** w_bits - 1) / 3 * (4.0 ** a_bits - 1) / 3
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(k * k * Cin * var)).astype(np.float32)
    want_acc = oracle.conv2d(a, w, stride, pad)
    if res_bits == 8:
        top = 255
        res_shape = want_acc.shape
        bias, _, rs, res_f = _terms(gen, which, res_shape, 7)
        res_lv = (2 * gen.integers(0, 256, size=res_shape) - top).astype(np.int16) if "res_q" in which or which == "all" else None
    else:
        bias, res_lv, rs, res_f = _terms(gen, which, want_acc.shape, res_bits)
    res_planes = None
    if res_lv is not None:
        # 8-bit codes do not fit int8 levels: pack them on the host
        res_planes = dev(oracle.pack_planes(res_lv.reshape(-1, Cout), res_bits).view(np.int32))
    wp = pack_levels(w, w_bits).view(w_bits, Cout, k, k, -1)
    acc, out, nxt = qnn.qnn_conv2d_block(pack_levels(a, a_bits), wp, (B, H, W), Cin, stride, pad, dev(s),
                                         bias=_opt(bias), res_planes=res_planes, res_scale=float(rs), res_f32=_opt(res_f),
                                         want_out=True, next_clip=2.5, next_bits=3)
    torch.cuda.synchronize()
    want = oracle.block_epilogue(want_acc, s, bias, res_lv, rs, res_f)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
    lv, _ = oracle.quantize(want, 2.5, 3)
    assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, Cout), 3))


@pytest.mark.parametrize("geom", [g for g in GEOMS if g[3] % 16 == 0])
@pytest.mark.parametrize("which", TERMS)
@pytest.mark.parametrize("bits", [(2, 2, 2), (3, 3, 4), (4, 4, 1), (7, 5, 7)])
def test_block_terms_matrix_core_route(geom, which, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits, res_bits = bits
    gen = np.random.default_rng(sum(geom) * 7 + sum(bits) + len(which))
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    var = (4.0 ** w_bits - 1) / 3 * (4.0 ** a_bits - 1) / 3
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(k * k * Cin * var)).astype(np.float32)
    want_acc = oracle.conv2d(a, w, stride, pad)
    bias, res_lv, rs, res_f = _terms(gen, which, want_acc.shape, res_bits)
    acc, out, nxt = qnn.qnn_level_conv2d_block_i8(dev(a), dev(w), stride, pad, a_bits, w_bits, dev(s), bias=_opt(bias),
                                                  res_levels=_opt(res_lv), res_bits=res_bits, res_scale=float(rs),
                                                  res_f32=_opt(res_f), want_out=True, next_clip=2.5, next_bits=3)
    torch.cuda.synchronize()
    want = oracle.block_epilogue(want_acc, s, bias, res_lv, rs, res_f)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
    lv, _ = oracle.quantize(want, 2.5, 3)
    assert np.array_equal(nxt.cpu().numpy(), lv.astype(np.int8))
    # levels only: neither acc nor out leaves the chip
    _, _, nxt2 = qnn.qnn_level_conv2d_block_i8(dev(a), dev(w), stride, pad, a_bits, w_bits, dev(s), bias=_opt(bias),
                                               res_levels=_opt(res_lv), res_bits=res_bits, res_scale=float(rs),
                                               res_f32=_opt(res_f), want_acc=False, next_clip=2.5, next_bits=3)
    torch.cuda.synchronize()
    assert np.array_equal(nxt2.cpu().numpy(), lv.astype(np.int8))


def test_block_terms_wide_bits_and_plain_kernel():
    gen = np.random.default_rng(9)
    # 6 x 5 bits: chunk launches, the terms belong to the last one only
    a = (2 * gen.integers(0, 32, size=(2, 9, 9, 64)) - 31).astype(np.int8)
    w = (2 * gen.integers(0, 64, size=(40, 3, 3, 64)) - 63).astype(np.int8)
    s = (gen.uniform(0.5, 1.5, size=40) / 20000).astype(np.float32)
    want_acc = oracle.conv2d(a, w, 1, 1)
    bias, res_lv, rs, res_f = _terms(gen, "all", want_acc.shape, 3)
    wp = pack_levels(w, 6).view(6, 40, 3, 3, -1)
    for want_acc_buf in (True, False):          # running sum in acc, or in out's memory
        acc, out, nxt = qnn.qnn_conv2d_block(pack_levels(a, 5), wp, (2, 9, 9), 64, 1, 1, dev(s), bias=dev(bias),
                                             res_planes=pack_levels(res_lv.reshape(-1, 40), 3), res_scale=float(rs),
                                             res_f32=dev(res_f), want_acc=want_acc_buf, want_out=True, next_clip=2.5,
                                             next_bits=2)
        torch.cuda.synchronize()
        want = oracle.block_epilogue(want_acc, s, bias, res_lv, rs, res_f)
        if want_acc_buf:
            assert np.array_equal(acc.cpu().numpy(), want_acc)
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
        lv, _ = oracle.quantize(want, 2.5, 2)
        assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, 40), 2))
    # 7x7 taps over 160 channels: more reduction words than the tiled kernel's tap table -> plain kernel
    a, w = levels(gen, (1, 9, 9, 800), 2), levels(gen, (5, 7, 7, 800), 2)
    s = gen.uniform(1e-3, 2e-3, size=5).astype(np.float32)
    want_acc = oracle.conv2d(a, w, 1, 3)
    bias, res_lv, rs, res_f = _terms(gen, "all", want_acc.shape, 2)
    wp = pack_levels(w, 2).view(2, 5, 7, 7, -1)
    acc, out, _ = qnn.qnn_conv2d_block(pack_levels(a, 2), wp, (1, 9, 9), 800, 1, 3, dev(s), bias=dev(bias),
                                       res_planes=pack_levels(res_lv.reshape(-1, 5), 2), res_scale=float(rs),
                                       res_f32=dev(res_f), want_out=True)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.block_epilogue(want_acc, s, bias, res_lv, rs, res_f),
                               rtol=RTOL, atol=0)


def test_null_epilogue_is_the_plain_convolution():
    gen = np.random.default_rng(10)
    a, w = levels(gen, (2, 8, 8, 32), 2), levels(gen, (16, 3, 3, 32), 2)
    s = gen.uniform(0.01, 0.1, size=16).astype(np.float32)
    wp = pack_levels(w, 2).view(2, 16, 3, 3, -1)
    a0, o0, n0 = qnn.qnn_conv2d(pack_levels(a, 2), wp, (2, 8, 8), 32, 1, 1, scale=dev(s), want_out=True,
                                next_clip=1.0, next_bits=2)
    a1, o1, n1 = qnn.qnn_conv2d_block(pack_levels(a, 2), wp, (2, 8, 8), 32, 1, 1, dev(s), want_out=True,
                                      next_clip=1.0, next_bits=2)
    torch.cuda.synchronize()
    assert torch.equal(a0, a1) and torch.equal(o0, o1) and torch.equal(n0, n1)


# ---------------------------------------------------------------------------------- residual trunk
def run_trunk_planes(net, bits, keep=True):
    """The trunk on the xor + bitcount route: planes between layers, the identity shortcut read back from
    the block's own input planes, the 1x1 shortcut handed over in fp32."""
    x, blocks = net["x"], net["blocks"]
    B, H, W, C = x.shape
    a = qnn.qnn_encode_pack(dev(x), blocks[0]["conv1"]["clip"], bits)
    trace = []
    for bi, blk in enumerate(blocks):
        c1, c2, dn = blk["conv1"], blk["conv2"], blk["down"]
        nxt_clip = blocks[bi + 1]["conv1"]["clip"] if bi + 1 < len(blocks) else None
        cout, st = c1["cout"], c1["stride"]
        Ho, Wo = (H + 2 - 3) // st + 1, (W + 2 - 3) // st + 1
        wp = lambda L, k: pack_levels(L["w"], bits).view(bits, L["cout"], k, k, -1)
        acc1, _, hq = qnn.qnn_conv2d_block(a, wp(c1, 3), (B, H, W), C, st, 1, dev(c1["scale"]), bias=dev(c1["bias"]),
                                           want_acc=keep, next_clip=c2["clip"], next_bits=bits)
        accd = short = None
        if dn is not None:
            accd, short, _ = qnn.qnn_conv2d_block(a, wp(dn, 1), (B, H, W), C, st, 0, dev(dn["scale"]),
                                                  bias=dev(dn["bias"]), want_acc=keep, want_out=True)
            kw = {"res_f32": short}
        else:
            kw = {"res_planes": a, "res_scale": blk["res_scale"]}
        acc2, y, nxt = qnn.qnn_conv2d_block(hq, wp(c2, 3), (B, Ho, Wo), cout, 1, 1, dev(c2["scale"]), bias=dev(c2["bias"]),
                                            want_acc=keep, want_out=keep or nxt_clip is None, next_clip=nxt_clip,
                                            next_bits=bits if nxt_clip is not None else 0, **kw)
        trace.append({"a": a, "acc1": acc1, "hq": hq, "acc2": acc2, "accd": accd, "shortcut": short, "y": y, "C": C,
                      "cout": cout})
        a, H, W, C = nxt, Ho, Wo, cout
    torch.cuda.synchronize()
    return trace


def run_trunk_levels(net, bits, keep=True):
    """The same trunk on the matrix-core route: int8 levels between layers."""
    x, blocks = net["x"], net["blocks"]
    a = qnn.qnn_encode_levels_i8(dev(x), blocks[0]["conv1"]["clip"], bits)
    trace = []
    for bi, blk in enumerate(blocks):
        c1, c2, dn = blk["conv1"], blk["conv2"], blk["down"]
        nxt_clip = blocks[bi + 1]["conv1"]["clip"] if bi + 1 < len(blocks) else None
        st = c1["stride"]
        acc1, _, hq = qnn.qnn_level_conv2d_block_i8(a, dev(c1["w"]), st, 1, bits, bits, dev(c1["scale"]), bias=dev(c1["bias"]),
                                                    want_acc=keep, next_clip=c2["clip"], next_bits=bits)
        accd = short = None
        if dn is not None:
            accd, short, _ = qnn.qnn_level_conv2d_block_i8(a, dev(dn["w"]), st, 0, bits, bits, dev(dn["scale"]),
                                                           bias=dev(dn["bias"]), want_acc=keep, want_out=True)
            kw = {"res_f32": short}
        else:
            kw = {"res_levels": a, "res_bits": bits, "res_scale": blk["res_scale"]}
        acc2, y, nxt = qnn.qnn_level_conv2d_block_i8(hq, dev(c2["w"]), 1, 1, bits, bits, dev(c2["scale"]), bias=dev(c2["bias"]),
                                                     want_acc=keep, want_out=keep or nxt_clip is None, next_clip=nxt_clip,
                                                     next_bits=bits if nxt_clip is not None else 0, **kw)
        trace.append({"a": a, "acc1": acc1, "hq": hq, "acc2": acc2, "accd": accd, "shortcut": short, "y": y})
        a = nxt
    torch.cuda.synchronize()
    return trace


def _np(t):
    return None if t is None else t.cpu().numpy()


@pytest.mark.parametrize("bits", [2, 3])
def test_resnet18_trunk_binary_route_small_batch(bits):
    net = wl.resnet18_trunk(batch=2, bits=bits)
    got = run_trunk_planes(net, bits)
    want = oracle.residual_trunk(net["x"], net["blocks"])
    assert len(got) == len(want) == 8
    for bi, (g, o) in enumerate(zip(got, want)):
        assert np.array_equal(planes_to_numpy(g["a"]), oracle.pack_planes(o["a"].reshape(-1, g["C"]), bits)), bi
        assert np.array_equal(planes_to_numpy(g["hq"]), oracle.pack_planes(o["hq"].reshape(-1, g["cout"]), bits)), bi
        assert np.array_equal(_np(g["acc1"]), o["acc1"]) and np.array_equal(_np(g["acc2"]), o["acc2"]), bi
        assert (g["accd"] is None) == (o["accd"] is None), bi
        if o["accd"] is not None:
            assert np.array_equal(_np(g["accd"]), o["accd"]), bi
            np.testing.assert_allclose(_np(g["shortcut"]), o["shortcut"], rtol=RTOL, atol=0)
        np.testing.assert_allclose(_np(g["y"]), o["y"], rtol=RTOL, atol=0)
    # fused only: nothing but planes (and the 1x1 shortcuts) between layers
    lean = run_trunk_planes(net, bits, keep=False)
    for bi, (g, o) in enumerate(zip(lean, want)):
        assert np.array_equal(planes_to_numpy(g["hq"]), oracle.pack_planes(o["hq"].reshape(-1, g["cout"]), bits)), bi
        assert g["acc1"] is None and g["acc2"] is None
    np.testing.assert_allclose(_np(lean[-1]["y"]), want[-1]["y"], rtol=RTOL, atol=0)


@pytest.mark.parametrize("bits", [2, 3])
def test_resnet18_trunk_matrix_core_route_small_batch(bits):
    net = wl.resnet18_trunk(batch=2, bits=bits)
    got = run_trunk_levels(net, bits)
    want = oracle.residual_trunk(net["x"], net["blocks"])
    for bi, (g, o) in enumerate(zip(got, want)):
        assert np.array_equal(_np(g["a"]), o["a"].astype(np.int8)), bi
        assert np.array_equal(_np(g["hq"]), o["hq"].astype(np.int8)), bi
        assert np.array_equal(_np(g["acc1"]), o["acc1"]) and np.array_equal(_np(g["acc2"]), o["acc2"]), bi
        if o["accd"] is not None:
            assert np.array_equal(_np(g["accd"]), o["accd"]), bi
        np.testing.assert_allclose(_np(g["y"]), o["y"], rtol=RTOL, atol=0)
    lean = run_trunk_levels(net, bits, keep=False)
    for bi, (g, o) in enumerate(zip(lean, want)):
        assert np.array_equal(_np(g["hq"]), o["hq"].astype(np.int8)), bi
    np.testing.assert_allclose(_np(lean[-1]["y"]), want[-1]["y"], rtol=RTOL, atol=0)


def test_resnet18_trunk_full_batch_every_image():
    # batch 256 as bench.py times it, against the oracle's trunk over the whole batch: the levels between
    # the two convolutions of every block and the trunk's output, on both routes
    bits = 3
    net = wl.resnet18_trunk(bits=bits)
    want = [(t["hq"].astype(np.int8), t["y"] if bi == 7 else None)
            for bi, t in enumerate(oracle.residual_trunk(net["x"], net["blocks"]))]
    for route, run in (("planes", run_trunk_planes), ("levels", run_trunk_levels)):
        got = run(net, bits, keep=False)
        for bi, (g, (hq, _)) in enumerate(zip(got, want)):
            if route == "planes":
                assert np.array_equal(planes_to_numpy(g["hq"]), oracle.pack_planes(hq.reshape(-1, hq.shape[-1]), bits)), bi
            else:
                assert np.array_equal(_np(g["hq"]), hq), (route, bi)
        np.testing.assert_allclose(_np(got[-1]["y"]), want[-1][1], rtol=RTOL, atol=0)
        del got
        torch.cuda.empty_cache()


@pytest.mark.parametrize("geom", [GEOMS[0], GEOMS[3], GEOMS[5]])
@pytest.mark.parametrize("which", ["relu", "bias+relu", "all+relu"])
def test_relu_term_all_routes(geom, which):
    # max(y, 0) after the other terms (HReLU's lower limit), then the fused quantizer: planes / levels of the
    # upper half only.  xor + bitcount route, int8 matrix-core route, and the plain one-lane kernel's shape.
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits = a_bits = res_bits = 2
    gen = np.random.default_rng(sum(geom) + len(which))
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(k * k * Cin * 25.0)).astype(np.float32)
    want_acc = oracle.conv2d(a, w, stride, pad)
    base = "all" if which.startswith("all") else which.replace("+relu", "").replace("relu", "")
    bias, res_lv, rs, res_f = _terms(gen, base, want_acc.shape, res_bits) if base else (None, None, np.float32(0.37), None)
    want = oracle.block_epilogue(want_acc, s, bias, res_lv, rs, res_f, relu=True)
    assert (want >= 0).all() and (want == 0).any()
    lv, _ = oracle.quantize(want, 2.5, 3)
    assert lv.min() >= 1

    wp = pack_levels(w, w_bits).view(w_bits, Cout, k, k, -1)
    res_planes = None if res_lv is None else pack_levels(res_lv.reshape(-1, Cout), res_bits)
    acc, out, nxt = qnn.qnn_conv2d_block(pack_levels(a, a_bits), wp, (B, H, W), Cin, stride, pad, dev(s), bias=_opt(bias),
                                         res_planes=res_planes, res_scale=float(rs), res_f32=_opt(res_f), relu=True,
                                         want_out=True, next_clip=2.5, next_bits=3)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
    assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, Cout), 3))

    if Cin % 16 == 0:
        acc, out, nl = qnn.qnn_level_conv2d_block_i8(dev(a), dev(w), stride, pad, a_bits, w_bits, dev(s), bias=_opt(bias),
                                                     res_levels=_opt(res_lv), res_bits=res_bits, res_scale=float(rs),
                                                     res_f32=_opt(res_f), relu=True, want_out=True, next_clip=2.5, next_bits=3)
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), want_acc)
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
        assert np.array_equal(nl.cpu().numpy(), lv.astype(np.int8))
