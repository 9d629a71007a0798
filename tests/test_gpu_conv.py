"""GPU parity: qnn_conv2d (implicit im2col, zero padding, fused next-layer epilogue) against the
CPU oracle's plain convolution on decoded levels."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, pack_levels, planes_to_numpy, levels, oracle_full_batch

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

RTOL = 1e-5


def _conv(a, w, a_bits, w_bits, stride, pad, scale=None, want_out=False, next_clip=None, next_bits=0):
    B, H, W, Cin = a.shape
    ap = pack_levels(a, a_bits)
    wp = pack_levels(w, w_bits)      # [w_bits][Cout*kh*kw][cw]
    wp = wp.view(w_bits, w.shape[0], w.shape[1], w.shape[2], -1)
    acc, out, nxt = qnn.qnn_conv2d(ap, wp, (B, H, W), Cin, stride, pad,
                                   scale=None if scale is None else dev(scale), want_out=want_out,
                                   next_clip=next_clip, next_bits=next_bits)
    torch.cuda.synchronize()
    return (acc.cpu().numpy(), None if out is None else out.cpu().numpy(),
            None if nxt is None else planes_to_numpy(nxt))


GEOMS = [
    # B, H, W, Cin, Cout, k, stride, pad
    (2, 7, 9, 5, 4, 3, 1, 1),        # cw = 1, ragged channels
    (1, 8, 8, 32, 6, 3, 2, 1),
    (2, 6, 5, 3, 3, 1, 1, 0),        # 1x1
    (1, 9, 7, 40, 70, 5, 1, 2),      # cw = 2 ragged, 5x5
    (1, 9, 10, 64, 64, 3, 2, 0),
    (3, 4, 4, 7, 5, 3, 1, 2),        # pad 2 with a 3x3 kernel: windows mostly in the padding
    (2, 14, 14, 128, 130, 3, 1, 1),  # cw = 4, two column tiles
    (1, 12, 12, 160, 32, 3, 1, 1),   # cw = 5
    (5, 13, 13, 64, 64, 3, 1, 1),    # several row tiles, ragged tail
    (1, 7, 7, 96, 100, 7, 1, 3),     # 7x7
]


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("bits", [(2, 2), (3, 3), (4, 4), (1, 1), (4, 1), (2, 3)])
def test_conv_acc_and_out(geom, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits = bits
    gen = np.random.default_rng(sum(geom) * 10 + w_bits + a_bits)
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    s = gen.uniform(0.01, 0.1, size=Cout).astype(np.float32)
    acc, out, _ = _conv(a, w, a_bits, w_bits, stride, pad, scale=s, want_out=True)
    want = oracle.conv2d(a, w, stride, pad)
    assert np.array_equal(acc, want)
    np.testing.assert_allclose(out, oracle.scale(want, s), rtol=RTOL, atol=0)


def _wide(gen, shape, bits):
    top = (1 << bits) - 1
    return (2 * gen.integers(0, top + 1, size=shape) - top).astype(np.int16)


def _zero_padded_im2col_gemm(a, w, k, stride, pad):
    # oracle GEMM on an explicit zero-padded im2col: the pad = 0 / 1x1 identities pinned for the
    # oracle's convolution, usable for 8-bit levels that do not fit its int8 input
    B, H, W, Cin = a.shape
    Cout = w.shape[0]
    ap = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), np.int16)
    ap[:, pad:pad + H, pad:pad + W] = a
    ho, wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    cols = np.stack([ap[b, y * stride:y * stride + k, x * stride:x * stride + k].reshape(-1)
                     for b in range(B) for y in range(ho) for x in range(wo)])
    return oracle.gemm(cols, w.reshape(Cout, -1)).reshape(B, ho, wo, Cout)


@pytest.mark.parametrize("bits", [(5, 5), (8, 8), (6, 2), (3, 7), (4, 5)])
@pytest.mark.parametrize("geom", [(1, 6, 6, 40, 9, 3, 1, 1), (2, 9, 10, 64, 70, 3, 2, 1), (1, 7, 7, 32, 33, 5, 1, 2)])
def test_conv_wide_bits(bits, geom):
    # widths above 4 run as chunk pairs of at most 4 x 4 planes with a shifted running sum, including
    # the zero-padding correction of every chunk pair
    w_bits, a_bits = bits
    B, H, W, Cin, Cout, k, stride, pad = geom
    gen = np.random.default_rng(w_bits + a_bits + sum(geom))
    a, w = _wide(gen, (B, H, W, Cin), a_bits), _wide(gen, (Cout, k, k, Cin), w_bits)
    s = gen.uniform(0.01, 0.1, size=Cout).astype(np.float32)
    ap = dev(oracle.pack_planes(a.reshape(-1, Cin), a_bits).view(np.int32))
    wp = dev(oracle.pack_planes(w.reshape(-1, Cin), w_bits).view(np.int32)).view(w_bits, Cout, k, k, -1)
    acc, out, _ = qnn.qnn_conv2d(ap, wp, (B, H, W), Cin, stride, pad, scale=dev(s), want_out=True)
    _, out_only, _ = qnn.qnn_conv2d(ap, wp, (B, H, W), Cin, stride, pad, scale=dev(s), want_acc=False, want_out=True)
    torch.cuda.synchronize()
    want = _zero_padded_im2col_gemm(a, w, k, stride, pad)
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=RTOL, atol=0)
    assert torch.equal(out, out_only)


def test_conv_wide_bits_fused_next_planes():
    # 6-bit layer feeding a 5-bit one: the last chunk pair's epilogue quantizes the complete sum
    gen = np.random.default_rng(65)
    B, H, W, Cin, Cout = 2, 8, 8, 64, 64
    a, w = _wide(gen, (B, H, W, Cin), 6), _wide(gen, (Cout, 3, 3, Cin), 6)
    var = (4.0 ** 6 - 1) / 3
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(9 * Cin * var * var)).astype(np.float32)
    ap = dev(oracle.pack_planes(a.reshape(-1, Cin), 6).view(np.int32))
    wp = dev(oracle.pack_planes(w.reshape(-1, Cin), 6).view(np.int32)).view(6, Cout, 3, 3, -1)
    acc, _, nxt = qnn.qnn_conv2d(ap, wp, (B, H, W), Cin, 1, 1, scale=dev(s), next_clip=2.5, next_bits=5)
    torch.cuda.synchronize()
    want = _zero_padded_im2col_gemm(a, w, 3, 1, 1)
    lv, _ = oracle.quantize(oracle.scale(want, s), 2.5, 5)
    assert np.array_equal(acc.cpu().numpy(), want)
    assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, Cout), 5))
    assert len(np.unique(lv)) == 32
    with pytest.raises(qnn.QnnError) as e:       # planes only: nowhere to keep the running sum
        qnn.qnn_conv2d(ap, wp, (B, H, W), Cin, 1, 1, scale=dev(s), want_acc=False, next_clip=2.5, next_bits=5)
    assert e.value.code == -2


@pytest.mark.parametrize("geom", [(2, 9, 9, 64, 64, 3, 1, 1), (1, 10, 10, 32, 100, 3, 2, 1),
                                  (2, 8, 8, 128, 128, 3, 1, 1)])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_conv_fused_next_planes(geom, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    gen = np.random.default_rng(sum(geom) + bits)
    a, w = levels(gen, (B, H, W, Cin), bits), levels(gen, (Cout, k, k, Cin), bits)
    var = (4.0 ** bits - 1) / 3
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(k * k * Cin * var * var)).astype(np.float32)
    acc, out, nxt = _conv(a, w, bits, bits, stride, pad, scale=s, want_out=True, next_clip=2.5, next_bits=bits)
    want_acc = oracle.conv2d(a, w, stride, pad)
    want_out = oracle.scale(want_acc, s)
    lv, _ = oracle.quantize(want_out, 2.5, bits)
    assert np.array_equal(acc, want_acc)
    assert np.array_equal(nxt, oracle.pack_planes(lv.reshape(-1, Cout), bits))
    assert len(np.unique(lv)) == (1 << bits)
    # planes only (no acc / out leaves the chip)
    ap, wp = pack_levels(a, bits), pack_levels(w, bits).view(bits, Cout, k, k, -1)
    _, _, nxt2 = qnn.qnn_conv2d(ap, wp, (B, H, W), Cin, stride, pad, scale=dev(s), want_acc=False,
                                next_clip=2.5, next_bits=bits)
    assert np.array_equal(planes_to_numpy(nxt2), nxt)


def test_config3_resnet_conv_full():
    # batch 64, 56x56, 64 -> 64, 2x2 bit, fp32 input encoded on device with clip = 3 sigma
    c = wl.resnet_conv_2x2()
    x = c["x"]
    B, H, W, Cin = x.shape
    ap = qnn.qnn_encode_pack(dev(x), c["clip"], 2)
    wp = pack_levels(c["w"], 2).view(2, 64, 3, 3, -1)
    acc, out, _ = qnn.qnn_conv2d(ap, wp, (B, H, W), Cin, 1, 1, scale=dev(c["scale"]), want_out=True)
    torch.cuda.synchronize()
    lv, _ = oracle.quantize(x, c["clip"], 2)
    assert np.array_equal(planes_to_numpy(ap), oracle.pack_planes(lv.reshape(-1, Cin), 2))
    want = oracle.conv2d(lv.astype(np.int8), c["w"], 1, 1)
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, c["scale"]), rtol=RTOL, atol=0)
    sat = np.mean(np.abs(x) >= c["clip"])
    assert 0.001 < sat < 0.006     # about 0.27 % of a Gaussian lies beyond 3 sigma


def _run_stack_gpu(x, layers, keep_acc):
    """encode -> [conv + scale + encode fused]* ; returns per-layer (planes_in, acc or None)."""
    B, H, W, C = x.shape
    planes = qnn.qnn_encode_pack(dev(x), layers[0]["clip"], layers[0]["a_bits"])
    trace = []
    for li, L in enumerate(layers):
        wp = pack_levels(L["w"], L["w_bits"]).view(L["w_bits"], L["cout"], 3, 3, -1)
        last = li + 1 == len(layers)
        nxt_clip = None if last else layers[li + 1]["clip"]
        nxt_bits = 0 if last else layers[li + 1]["a_bits"]
        acc, out, nxt = qnn.qnn_conv2d(planes, wp, (B, H, W), L["cin"], L["stride"], L["pad"],
                                       scale=dev(L["scale"]), want_acc=keep_acc, want_out=last,
                                       next_clip=nxt_clip, next_bits=nxt_bits)
        trace.append({"planes": planes, "acc": acc, "out": out})
        H = (H + 2 * L["pad"] - 3) // L["stride"] + 1
        W = (W + 2 * L["pad"] - 3) // L["stride"] + 1
        planes = nxt
    torch.cuda.synchronize()
    return trace


def test_config4_resnet18_stack_small_batch():
    # the full 16-layer 3x3-bit chain at batch 2: every layer's input planes and accumulators
    # must equal the oracle chain bit for bit
    c = wl.resnet18_stack(batch=2)
    trace = _run_stack_gpu(c["x"], c["layers"], keep_acc=True)
    want = oracle.conv_stack(c["x"], c["layers"])
    for li, (g, o) in enumerate(zip(trace, want)):
        cin = c["layers"][li]["cin"]
        assert np.array_equal(planes_to_numpy(g["planes"]),
                              oracle.pack_planes(o["levels"].reshape(-1, cin), 3)), li
        assert np.array_equal(g["acc"].cpu().numpy(), o["acc"]), li
        assert len(np.unique(o["levels"])) == 8, li       # the chain keeps exercising every level
    np.testing.assert_allclose(trace[-1]["out"].cpu().numpy(), want[-1]["out"], rtol=RTOL, atol=0)


def test_config5_vgg_ssd_stack_small_batch():
    groups = wl.vgg_ssd_stack(batch=1)
    for g in groups:
        trace = _run_stack_gpu(g["x"], g["layers"], keep_acc=True)
        want = oracle.conv_stack(g["x"], g["layers"])
        for li, (t, o) in enumerate(zip(trace, want)):
            cin = g["layers"][li]["cin"]
            assert np.array_equal(planes_to_numpy(t["planes"]),
                                  oracle.pack_planes(o["levels"].reshape(-1, cin), 4)), li
            assert np.array_equal(t["acc"].cpu().numpy(), o["acc"]), li


def test_config4_full_batch_every_image():
    # batch 256 as bench.py times it (fused epilogues only, no accumulator leaves the chip), against the
    # oracle's chain over the whole batch: the planes entering every layer and the final output
    c = wl.resnet18_stack()
    trace = _run_stack_gpu(c["x"], c["layers"], keep_acc=False)
    (want_levels, want_out), = oracle_full_batch("stack4")
    for li, (g, lv) in enumerate(zip(trace, want_levels)):
        assert np.array_equal(planes_to_numpy(g["planes"]), oracle.pack_planes(lv.reshape(-1, lv.shape[-1]), 3)), li
    np.testing.assert_allclose(trace[-1]["out"].cpu().numpy(), want_out, rtol=RTOL, atol=0)


def test_config5_full_batch_every_image():
    groups = wl.vgg_ssd_stack()     # batch 32
    for g, (want_levels, want_out) in zip(groups, oracle_full_batch("stack5")):
        trace = _run_stack_gpu(g["x"], g["layers"], keep_acc=False)
        for li, (t, lv) in enumerate(zip(trace, want_levels)):
            assert np.array_equal(planes_to_numpy(t["planes"]), oracle.pack_planes(lv.reshape(-1, lv.shape[-1]), 4)), li
        np.testing.assert_allclose(trace[-1]["out"].cpu().numpy(), want_out, rtol=RTOL, atol=0)
        del trace
        torch.cuda.empty_cache()
