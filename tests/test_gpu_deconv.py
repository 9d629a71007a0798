"""GPU parity of the transposed convolution on bit-planes (qnn_deconv_pack_weights + qnn_deconv2d)
against the CPU oracle's definition: accumulators bit-exact, fp32 out within 1e-5, next planes bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, pack_levels, planes_to_numpy, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

RTOL = 1e-5

GEOMS = [
    # B, H, W, Cin, Cout, k, stride, pad
    (2, 5, 6, 32, 8, 4, 2, 1),        # the usual 2x upsampling layer
    (1, 4, 4, 5, 6, 3, 2, 1),         # odd kernel: phases with 2x2, 2x1, 1x2, 1x1 taps; ragged channels
    (1, 3, 5, 40, 3, 2, 2, 0),        # kernel = stride: every output has one tap
    (2, 4, 3, 64, 70, 3, 1, 1),       # stride 1: one phase, a flipped convolution
    (1, 3, 3, 16, 5, 5, 3, 2),        # stride 3
    (1, 6, 5, 128, 33, 3, 2, 0),      # pad 0: the output grows by kh - stride
    (3, 9, 9, 64, 64, 4, 2, 1),       # several row tiles per phase
    (1, 7, 7, 96, 130, 6, 2, 2),      # 3x3 sub-kernels, several column tiles
    (1, 5, 5, 32, 16, 4, 4, 0),       # stride 4, 16 phases of one tap
    (1, 2, 2, 32, 4, 4, 2, 2),        # pad so large that every phase keeps a single output
]


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("bits", [(2, 2), (3, 3), (4, 4), (1, 1), (4, 1), (2, 3)])
def test_deconv_acc_out_and_next_planes(geom, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits = bits
    Ho, Wo = (H - 1) * stride - 2 * pad + k, (W - 1) * stride - 2 * pad + k
    if Ho < 1 or Wo < 1:
        pytest.skip("no output")
    gen = np.random.default_rng(sum(geom) * 10 + w_bits + a_bits)
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    var = (4.0 ** w_bits - 1) / 3 * (4.0 ** a_bits - 1) / 3
    taps = (-(-k // stride)) ** 2
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(taps * Cin * var)).astype(np.float32)
    bias = gen.uniform(-0.5, 0.5, size=Cout).astype(np.float32)
    wp = pack_levels(w, w_bits).view(w_bits, Cout, k, k, -1)
    ph = qnn.qnn_deconv_pack_weights(wp, Cin, stride)
    acc, out, nxt = qnn.qnn_deconv2d(pack_levels(a, a_bits), ph, (B, H, W), Cin, Cout, k, k, stride, pad, w_bits,
                                     scale=dev(s), bias=dev(bias), want_out=True, next_clip=2.5, next_bits=3)
    torch.cuda.synchronize()
    want_acc = oracle.deconv2d(a, w, stride, pad)
    assert acc.shape == want_acc.shape
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    want = oracle.block_epilogue(want_acc, s, bias)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
    lv, _ = oracle.quantize(want, 2.5, 3)
    assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, Cout), 3))


def _wide(gen, shape, bits):
    top = (1 << bits) - 1
    return (2 * gen.integers(0, top + 1, size=shape) - top).astype(np.int16)


@pytest.mark.parametrize("bits", [(5, 5), (8, 8), (6, 2), (3, 7), (4, 5)])
@pytest.mark.parametrize("geom", [GEOMS[0], GEOMS[1], GEOMS[5], GEOMS[7], GEOMS[4]])
def test_deconv_wide_bits(geom, bits):
    # widths above 4 run as chunk pairs of at most 4 x 4 planes over all phases, the running sum kept per output
    # pixel by the phase that owns it (one-launch phases and per-phase launches, masked border taps included)
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits = bits
    gen = np.random.default_rng(sum(geom) * 7 + 10 * w_bits + a_bits)
    a, w = _wide(gen, (B, H, W, Cin), a_bits), _wide(gen, (Cout, k, k, Cin), w_bits)
    var = (4.0 ** w_bits - 1) / 3 * (4.0 ** a_bits - 1) / 3
    taps = (-(-k // stride)) ** 2
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(taps * Cin * var)).astype(np.float32)
    bias = gen.uniform(-0.5, 0.5, size=Cout).astype(np.float32)
    ap = dev(oracle.pack_planes(a.reshape(-1, Cin), a_bits).view(np.int32))
    wp = dev(oracle.pack_planes(w.reshape(-1, Cin), w_bits).view(np.int32)).view(w_bits, Cout, k, k, -1)
    ph = qnn.qnn_deconv_pack_weights(wp, Cin, stride)
    acc, out, nxt = qnn.qnn_deconv2d(ap, ph, (B, H, W), Cin, Cout, k, k, stride, pad, w_bits, scale=dev(s), bias=dev(bias),
                                     want_out=True, next_clip=2.5, next_bits=5)
    _, out_only, nxt2 = qnn.qnn_deconv2d(ap, ph, (B, H, W), Cin, Cout, k, k, stride, pad, w_bits, scale=dev(s), bias=dev(bias),
                                         want_acc=False, want_out=True, next_clip=2.5, next_bits=5)
    torch.cuda.synchronize()
    want_acc = oracle.deconv2d(a, w, stride, pad)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    want = oracle.block_epilogue(want_acc, s, bias)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
    lv, _ = oracle.quantize(want, 2.5, 5)
    assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, Cout), 5))
    assert torch.equal(out, out_only) and torch.equal(nxt, nxt2)   # the running sum kept in the memory of out


def test_deconv_wide_bits_need_a_buffer_for_the_running_sum():
    ap = torch.zeros((5, 16, 1), dtype=torch.int32, device="cuda")
    ph = torch.zeros((5 * 8 * 16 * 1,), dtype=torch.int32, device="cuda")
    with pytest.raises(qnn.QnnError) as e:
        qnn.qnn_deconv2d(ap, ph, (1, 4, 4), 32, 8, 4, 4, 2, 1, 5, scale=torch.ones(8, device="cuda"), want_acc=False,
                         next_clip=1.0, next_bits=2)
    assert e.value.code == qnn.QNN_ERR_UNSUPPORTED


def test_deconv_acc_only_without_scale():
    gen = np.random.default_rng(4)
    a, w = levels(gen, (2, 6, 6, 64), 2), levels(gen, (32, 4, 4, 64), 2)
    ph = qnn.qnn_deconv_pack_weights(pack_levels(w, 2).view(2, 32, 4, 4, -1), 64, 2)
    acc, out, nxt = qnn.qnn_deconv2d(pack_levels(a, 2), ph, (2, 6, 6), 64, 32, 4, 4, 2, 1, 2)
    torch.cuda.synchronize()
    assert out is None and nxt is None
    assert np.array_equal(acc.cpu().numpy(), oracle.deconv2d(a, w, 2, 1))


def test_deconv_then_conv_chain():
    # a 2x upsampling layer feeding a 3x3 convolution through the fused planes, as in a decoder
    gen = np.random.default_rng(5)
    x = gen.normal(0, 1, size=(2, 7, 7, 64)).astype(np.float32)
    w1, w2 = levels(gen, (32, 4, 4, 64), 2), levels(gen, (16, 3, 3, 32), 2)
    s1 = (gen.uniform(0.5, 1.5, size=32) / np.sqrt(4 * 64 * 25)).astype(np.float32)
    s2 = gen.uniform(0.01, 0.1, size=16).astype(np.float32)
    xp = qnn.qnn_encode_pack(dev(x.reshape(-1, 64)), 3.0, 2)
    ph = qnn.qnn_deconv_pack_weights(pack_levels(w1, 2).view(2, 32, 4, 4, -1), 64, 2)
    _, _, mid = qnn.qnn_deconv2d(xp, ph, (2, 7, 7), 64, 32, 4, 4, 2, 1, 2, scale=dev(s1), want_acc=False,
                                 next_clip=3.0, next_bits=2)
    acc, out, _ = qnn.qnn_conv2d(mid, pack_levels(w2, 2).view(2, 16, 3, 3, -1), (2, 14, 14), 32, 1, 1, scale=dev(s2),
                                 want_out=True)
    torch.cuda.synchronize()
    lv, _ = oracle.quantize(x, 3.0, 2)
    up = oracle.scale(oracle.deconv2d(lv.astype(np.int8), w1, 2, 1), s1)
    lv2, _ = oracle.quantize(up, 3.0, 2)
    want = oracle.conv2d(lv2.astype(np.int8), w2, 1, 1)
    assert np.array_equal(planes_to_numpy(mid), oracle.pack_planes(lv2.reshape(-1, 32), 2))
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s2), rtol=RTOL, atol=0)


def _random_geoms(seed, count):
    gen = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        stride = int(gen.integers(1, 5))
        kh, kw = int(gen.integers(stride, 8)), int(gen.integers(stride, 8))
        pad = int(gen.integers(0, 4))
        H, W = int(gen.integers(1, 9)), int(gen.integers(1, 9))
        if (H - 1) * stride - 2 * pad + kh < 1 or (W - 1) * stride - 2 * pad + kw < 1:
            continue
        if -(-kh // stride) * -(-kw // stride) > 32:
            continue
        out.append((int(gen.integers(1, 4)), H, W, int(gen.choice([1, 31, 32, 33, 64, 100, 128])),
                    int(gen.choice([1, 3, 32, 33, 65, 130])), kh, kw, stride, pad, int(gen.integers(1, 5)),
                    int(gen.integers(1, 5))))
    return out


@pytest.mark.parametrize("geom", _random_geoms(19051, 40))
def test_deconv_random_geometry(geom):
    # rectangular kernels, strides up to 4, pads that crop whole phases, single-pixel images
    B, H, W, Cin, Cout, kh, kw, stride, pad, w_bits, a_bits = geom
    gen = np.random.default_rng(sum(x * (i + 1) for i, x in enumerate(geom)))
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, kh, kw, Cin), w_bits)
    s = gen.uniform(0.001, 0.01, size=Cout).astype(np.float32)
    ph = qnn.qnn_deconv_pack_weights(pack_levels(w, w_bits).view(w_bits, Cout, kh, kw, -1), Cin, stride)
    acc, out, nxt = qnn.qnn_deconv2d(pack_levels(a, a_bits), ph, (B, H, W), Cin, Cout, kh, kw, stride, pad, w_bits,
                                     scale=dev(s), want_out=True, next_clip=1.0, next_bits=2)
    torch.cuda.synchronize()
    want = oracle.deconv2d(a, w, stride, pad)
    assert np.array_equal(acc.cpu().numpy(), want), geom
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=RTOL, atol=0)
    lv, _ = oracle.quantize(oracle.scale(want, s), 1.0, 2)
    assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, Cout), 2)), geom


def test_deconv_benchmark_configuration_sampled_images():
    # the layer bench.py --workload deconv times (batch 64, 28x28x128 -> 56x56x64, 4x4 stride 2, 2x2 bit, one launch
    # over the four phases, fused next-layer planes); images are independent, so the oracle on three of them is exact
    import qnn_workloads as wl
    B, H, cin, cout, k, s, pad, bits = 64, 28, 128, 64, 4, 2, 1, 2
    x = wl.rng(7, 0).standard_normal((B * H * H, cin), dtype="float32")
    w = wl.odd_levels(wl.rng(7, 1), (cout, k, k, cin), bits)
    sc = wl.channel_scales(wl.rng(7, 2), cout)
    ph = qnn.qnn_deconv_pack_weights(pack_levels(w, bits).view(bits, cout, k, k, -1), cin, s)
    planes = qnn.qnn_encode_pack(dev(x), 3.0, bits)
    acc, out, nxt = qnn.qnn_deconv2d(planes, ph, (B, H, H), cin, cout, k, k, s, pad, bits, scale=dev(sc), want_out=True,
                                     next_clip=3.0, next_bits=bits)
    torch.cuda.synchronize()
    images = [0, 37, 63]
    lv, _ = oracle.quantize(x.reshape(B, H, H, cin)[images], 3.0, bits)
    want = oracle.deconv2d(lv.astype(np.int8), w, s, pad)
    assert np.array_equal(acc.cpu().numpy()[images], want)
    wout = oracle.scale(want, sc)
    np.testing.assert_allclose(out.cpu().numpy()[images], wout, rtol=RTOL, atol=0)
    nlv, _ = oracle.quantize(wout, 3.0, bits)
    got = planes_to_numpy(nxt).reshape(bits, B, 56 * 56, -1)[:, images].reshape(bits, -1, cout // 32)
    assert np.array_equal(got, oracle.pack_planes(nlv.reshape(-1, cout), bits))
