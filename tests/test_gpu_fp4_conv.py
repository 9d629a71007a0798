"""GPU parity of the fp4 matrix-core route for 1- and 2-bit convolutions (qnn_encode_levels_fp4,
qnn_levels_to_fp4, qnn_level_conv2d_fp4) against the CPU oracle: the same int32 accumulators and the
same levels after every layer, held as fp4 nibbles."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

RTOL = 1e-5


def nibbles(lv):
    """The documented layout: channel 2i in the low nibble of byte i; nibble = sign << 3 | E2M1 magnitude code."""
    lv = np.asarray(lv).astype(np.int64)
    assert lv.shape[-1] % 2 == 0 and set(np.unique(np.abs(lv))) <= {1, 3}
    code = np.where(lv < 0, 8, 0) | np.where(np.abs(lv) == 3, 5, 2)
    return (code[..., 0::2] | (code[..., 1::2] << 4)).astype(np.uint8)


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("count", [2, 14, 16, 18, 1000, 4096 * 3 + 6])
def test_encode_levels_fp4(bits, count):
    gen = np.random.default_rng(bits * 1000 + count)
    x = gen.normal(0, 1, size=count).astype(np.float32)
    x[:2] = [0.0, -5.0]
    got = qnn.qnn_encode_levels_fp4(dev(x), 1.5, bits)
    torch.cuda.synchronize()
    want, _ = oracle.quantize(x, 1.5, bits)
    assert np.array_equal(got.cpu().numpy(), nibbles(want))
    xb = torch.from_numpy(x).to(torch.bfloat16)
    gotb = qnn.qnn_encode_levels_fp4(xb.cuda(), 1.5, bits)
    torch.cuda.synchronize()
    wantb, _ = oracle.quantize(xb.to(torch.float32).numpy(), 1.5, bits)
    assert np.array_equal(gotb.cpu().numpy(), nibbles(wantb))


@pytest.mark.parametrize("count", [2, 16, 30, 32, 5000])
def test_levels_to_fp4(count):
    gen = np.random.default_rng(count)
    lv = levels(gen, (count,), 2)
    got = qnn.qnn_levels_to_fp4(dev(lv))
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), nibbles(lv))


GEOMS = [
    # B, H, W, Cin, Cout, k, stride, pad
    (2, 7, 9, 32, 4, 3, 1, 1),
    (1, 8, 8, 64, 6, 3, 2, 1),
    (2, 6, 5, 96, 38, 1, 1, 0),       # 1x1: reduction shorter than a stage
    (1, 9, 7, 64, 70, 5, 1, 2),       # ragged columns in the 256 x 128 block
    (2, 14, 14, 128, 130, 3, 1, 1),   # 256 x 256 block
    (5, 13, 13, 64, 64, 3, 1, 1),     # several row tiles, ragged tail
    (2, 24, 24, 32, 300, 3, 1, 1),    # two column tiles
    (1, 7, 7, 512, 512, 3, 1, 1),     # long reduction
]


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("bits", [(2, 2), (1, 1), (2, 1), (1, 2)])
def test_fp4_conv_acc_out_and_next_levels(geom, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits = bits
    gen = np.random.default_rng(sum(geom) * 10 + w_bits + a_bits)
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    var = (4.0 ** w_bits - 1) / 3 * (4.0 ** a_bits - 1) / 3
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(k * k * Cin * var)).astype(np.float32)
    a4, w4 = qnn.qnn_levels_to_fp4(dev(a)), qnn.qnn_levels_to_fp4(dev(w))
    acc, out, nxt = qnn.qnn_level_conv2d_fp4(a4, w4, stride, pad, a_bits, w_bits, scale=dev(s), want_out=True,
                                             next_clip=2.0, next_bits=2)
    torch.cuda.synchronize()
    want = oracle.conv2d(a, w, stride, pad)
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=RTOL, atol=0)
    lv, _ = oracle.quantize(oracle.scale(want, s), 2.0, 2)
    assert np.array_equal(nxt.cpu().numpy(), nibbles(lv))
    # levels only
    _, _, nxt2 = qnn.qnn_level_conv2d_fp4(a4, w4, stride, pad, a_bits, w_bits, scale=dev(s), want_acc=False,
                                          next_clip=2.0, next_bits=2)
    torch.cuda.synchronize()
    assert np.array_equal(nxt2.cpu().numpy(), nibbles(lv))


def test_fp4_conv_extreme_levels_hit_the_accumulator_bound():
    # all +3 against all +-3 over the longest test reduction: |acc| = 9 n, exact in fp32
    Cin, Cout = 1024, 8
    a = np.full((1, 5, 5, Cin), 3, np.int8)
    w = np.concatenate([np.full((4, 3, 3, Cin), 3, np.int8), np.full((4, 3, 3, Cin), -3, np.int8)])
    acc, _, _ = qnn.qnn_level_conv2d_fp4(qnn.qnn_levels_to_fp4(dev(a)), qnn.qnn_levels_to_fp4(dev(w)), 1, 1, 2, 2)
    torch.cuda.synchronize()
    want = oracle.conv2d(a, w, 1, 1)
    assert np.abs(want).max() == 9 * 9 * Cin
    assert np.array_equal(acc.cpu().numpy(), want)


def test_config3_conv_fp4_route_full_size():
    c = wl.resnet_conv_2x2()
    x4 = qnn.qnn_encode_levels_fp4(dev(c["x"]), c["clip"], 2)
    w4 = qnn.qnn_levels_to_fp4(dev(c["w"]))
    acc, out, _ = qnn.qnn_level_conv2d_fp4(x4, w4, 1, 1, 2, 2, scale=dev(c["scale"]), want_out=True)
    torch.cuda.synchronize()
    lv, _ = oracle.quantize(c["x"], c["clip"], 2)
    want = oracle.conv2d(lv.astype(np.int8), c["w"], 1, 1)
    assert np.array_equal(x4.cpu().numpy(), nibbles(lv))
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, c["scale"]), rtol=RTOL, atol=0)


def test_fp4_chain_matches_oracle_stack():
    # three fused layers, nothing but fp4 levels between them
    plan = ((64, 64, 1), (64, 128, 2), (128, 128, 1))
    c = wl.resnet18_stack(batch=2, hw=20, bits=2, plan=plan)
    want = oracle.conv_stack(c["x"], c["layers"])
    lv = qnn.qnn_encode_levels_fp4(dev(c["x"]), c["layers"][0]["clip"], 2)
    for li, L in enumerate(c["layers"]):
        last = li + 1 == len(c["layers"])
        assert np.array_equal(lv.cpu().numpy(), nibbles(want[li]["levels"])), li
        _, out, lv = qnn.qnn_level_conv2d_fp4(lv, qnn.qnn_levels_to_fp4(dev(L["w"])), L["stride"], L["pad"], 2, 2,
                                              scale=dev(L["scale"]), want_acc=False, want_out=last,
                                              next_clip=None if last else c["layers"][li + 1]["clip"],
                                              next_bits=0 if last else 2)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), want[-1]["out"], rtol=RTOL, atol=0)


@pytest.mark.parametrize("case", [(2, 8, 8, 32, 2, 2, 0, False), (1, 9, 7, 64, 3, 2, 1, False), (2, 5, 5, 6, 2, 2, 0, True),
                                  (1, 7, 7, 34, 3, 1, 1, False), (3, 10, 10, 96, 2, 2, 0, False)])
@pytest.mark.parametrize("bits", [1, 2])
def test_maxpool_levels_fp4(case, bits):
    B, H, W, C, k, stride, pad, ceil_mode = case
    gen = np.random.default_rng(sum(case[:7]) + bits)
    lv = levels(gen, (B, H, W, C), bits)
    got = qnn.qnn_maxpool_levels_fp4(qnn.qnn_levels_to_fp4(dev(lv)), k, stride, pad, ceil_mode)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), nibbles(oracle.maxpool(lv, k, stride, pad, ceil_mode)))


@pytest.mark.parametrize("bits", [1, 2])
def test_cifar_network_fp4_route(bits):
    # the CIFAR-10 network of the paper's Table 3 (from its second layer on) at the widths that table
    # reports, entirely on fp4 levels: convolutions, pooling on the codes, FC layers as fp4 GEMMs
    from test_gpu_network import _oracle_network, _next_weighted
    net = wl.cifar_vgg_network(batch=4, bits=bits)
    ops = net["ops"]
    lv = qnn.qnn_encode_levels_fp4(dev(net["x"]), ops[0]["clip"], bits)
    got, out = [], None
    for i, op in enumerate(ops):
        got.append(lv)
        nw_op = _next_weighted(ops, i)
        if op["kind"] == "pool":
            lv = qnn.qnn_maxpool_levels_fp4(lv, op["k"], op["stride"])
        elif op["kind"] == "conv":
            _, _, lv = qnn.qnn_level_conv2d_fp4(lv, qnn.qnn_levels_to_fp4(dev(op["w"])), 1, 1, bits, bits,
                                                scale=dev(op["scale"]), want_acc=False, next_clip=nw_op["clip"],
                                                next_bits=bits)
        else:
            n = op["n"]
            assert n // 2 == qnn.qnn_fp4_row_bytes(n)          # rows need no padding here
            _, out = qnn.qnn_level_gemm_fp4(lv.view(lv.shape[0], n // 2), qnn.qnn_levels_to_fp4(dev(op["w"])), n,
                                            want_acc=False, scale=dev(op["scale"]))
            if nw_op is not None:
                lv = qnn.qnn_encode_levels_fp4(out, nw_op["clip"], bits)
    torch.cuda.synchronize()
    want, want_out = _oracle_network(net["x"], ops)
    for i, (g, o) in enumerate(zip(got, want)):
        assert np.array_equal(g.cpu().numpy().reshape(o.shape[:-1] + (o.shape[-1] // 2,)), nibbles(o)), i
    np.testing.assert_allclose(out.cpu().numpy(), want_out, rtol=RTOL, atol=0)


@pytest.mark.parametrize("geom", [(2, 7, 9, 32, 4, 3, 1, 1), (2, 6, 5, 96, 38, 1, 1, 0), (2, 14, 14, 128, 130, 3, 1, 1),
                                  (5, 13, 13, 64, 64, 3, 1, 1)])
@pytest.mark.parametrize("which", ["bias", "res_q", "res_f32", "all"])
@pytest.mark.parametrize("res_bits", [1, 2])
def test_fp4_block_terms(geom, which, res_bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    gen = np.random.default_rng(sum(geom) + len(which) + res_bits)
    a, w = levels(gen, (B, H, W, Cin), 2), levels(gen, (Cout, k, k, Cin), 2)
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(k * k * Cin * 25.0)).astype(np.float32)
    want_acc = oracle.conv2d(a, w, stride, pad)
    bias = gen.uniform(-1, 1, size=Cout).astype(np.float32) if which in ("bias", "all") else None
    res_lv = levels(gen, want_acc.shape, res_bits) if which in ("res_q", "all") else None
    res_f = gen.normal(0, 1, size=want_acc.shape).astype(np.float32) if which in ("res_f32", "all") else None
    rs = np.float32(0.41)
    opt = lambda t: None if t is None else dev(t)
    acc, out, nxt = qnn.qnn_level_conv2d_block_fp4(
        qnn.qnn_levels_to_fp4(dev(a)), qnn.qnn_levels_to_fp4(dev(w)), stride, pad, 2, 2, dev(s), bias=opt(bias),
        res_levels=None if res_lv is None else qnn.qnn_levels_to_fp4(dev(res_lv)), res_bits=res_bits, res_scale=float(rs),
        res_f32=opt(res_f), want_out=True, next_clip=2.0, next_bits=2)
    torch.cuda.synchronize()
    want = oracle.block_epilogue(want_acc, s, bias, res_lv, rs, res_f)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
    lv, _ = oracle.quantize(want, 2.0, 2)
    assert np.array_equal(nxt.cpu().numpy(), nibbles(lv))


def test_resnet18_trunk_fp4_route():
    # the residual trunk at 2 bits entirely on fp4 levels: shifts, identity shortcuts read back as nibbles,
    # 1x1 shortcut convolutions handed over in fp32
    bits = 2
    net = wl.resnet18_trunk(batch=2, bits=bits)
    x, blocks = net["x"], net["blocks"]
    f4 = lambda t: qnn.qnn_levels_to_fp4(dev(t))
    a = qnn.qnn_encode_levels_fp4(dev(x), blocks[0]["conv1"]["clip"], bits)
    got = []
    for bi, blk in enumerate(blocks):
        c1, c2, dn = blk["conv1"], blk["conv2"], blk["down"]
        nxt_clip = blocks[bi + 1]["conv1"]["clip"] if bi + 1 < len(blocks) else None
        st = c1["stride"]
        _, _, hq = qnn.qnn_level_conv2d_block_fp4(a, f4(c1["w"]), st, 1, bits, bits, dev(c1["scale"]), bias=dev(c1["bias"]),
                                                  want_acc=False, next_clip=c2["clip"], next_bits=bits)
        if dn is not None:
            _, short, _ = qnn.qnn_level_conv2d_block_fp4(a, f4(dn["w"]), st, 0, bits, bits, dev(dn["scale"]),
                                                         bias=dev(dn["bias"]), want_acc=False, want_out=True)
            kw = {"res_f32": short}
        else:
            kw = {"res_levels": a, "res_bits": bits, "res_scale": blk["res_scale"]}
        _, y, nxt = qnn.qnn_level_conv2d_block_fp4(hq, f4(c2["w"]), 1, 1, bits, bits, dev(c2["scale"]), bias=dev(c2["bias"]),
                                                   want_acc=False, want_out=True, next_clip=nxt_clip,
                                                   next_bits=bits if nxt_clip is not None else 0, **kw)
        got.append((a, hq, y))
        a = nxt
    torch.cuda.synchronize()
    want = oracle.residual_trunk(x, blocks)
    for bi, ((ga, ghq, gy), o) in enumerate(zip(got, want)):
        assert np.array_equal(ga.cpu().numpy(), nibbles(o["a"])), bi
        assert np.array_equal(ghq.cpu().numpy(), nibbles(o["hq"])), bi
        np.testing.assert_allclose(gy.cpu().numpy(), o["y"], rtol=RTOL, atol=0)
