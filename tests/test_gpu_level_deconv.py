"""GPU parity of the transposed convolution on decoded levels (qnn_level_deconv_flip_weights + qnn_level_deconv2d_i8 /
qnn_level_deconv2d_fp4: zero insertion, flipped taps, the matrix-core convolution) against the CPU oracle's
definition of the transposed convolution: accumulators bit-exact, fp32 out within 1e-5, next levels bit-exact; and
against the bit-plane route (qnn_deconv2d) on the same tensors."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, levels, pack_levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

RTOL = 1e-5

GEOMS = [
    # B, H, W, Cin, Cout, k, stride, pad
    (2, 5, 6, 32, 8, 4, 2, 1),        # the usual 2x upsampling layer
    (1, 4, 4, 16, 6, 3, 2, 1),        # odd kernel
    (1, 3, 5, 48, 3, 2, 2, 0),        # kernel = stride: every output has one tap
    (2, 4, 3, 64, 70, 3, 1, 1),       # stride 1: a flipped convolution, nothing inserted
    (1, 3, 3, 16, 5, 5, 3, 2),        # stride 3
    (1, 6, 5, 128, 33, 3, 2, 0),      # pad 0: the output grows by k - stride
    (3, 9, 9, 64, 64, 4, 2, 1),       # several row tiles
    (1, 7, 7, 96, 130, 5, 2, 2),      # two column tiles of the 256 x 128 block; 25 of the at most 31 taps
    (1, 5, 5, 32, 16, 4, 4, 0),       # stride 4
    (1, 3, 3, 32, 4, 4, 2, 3),        # pad = k - 1: the widened tensor is not padded at all
    (2, 14, 14, 128, 256, 4, 2, 1),   # the 256 x 256 block
]


def _case(geom, w_bits, a_bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    gen = np.random.default_rng(sum(geom) * 10 + w_bits + a_bits)
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    var = (4.0 ** w_bits - 1) / 3 * (4.0 ** a_bits - 1) / 3
    taps = (-(-k // stride)) ** 2
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(taps * Cin * var)).astype(np.float32)
    bias = gen.uniform(-0.5, 0.5, size=Cout).astype(np.float32)
    return a, w, s, bias


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("bits", [(2, 2), (3, 3), (4, 4), (1, 1), (4, 1), (7, 7)])
def test_level_deconv_i8(geom, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits = bits
    a, w, s, bias = _case(geom, w_bits, a_bits)
    fw = qnn.qnn_level_deconv_flip_weights(dev(w))
    assert np.array_equal(fw.cpu().numpy(), w[:, ::-1, ::-1, :])
    acc, out, nxt = qnn.qnn_level_deconv2d_i8(dev(a), fw, stride, pad, a_bits, w_bits, scale=dev(s), bias=dev(bias),
                                              want_out=True, next_clip=2.5, next_bits=3)
    torch.cuda.synchronize()
    want_acc = oracle.deconv2d(a, w, stride, pad)
    assert acc.shape == want_acc.shape
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    want = oracle.block_epilogue(want_acc, s, bias)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
    lv, _ = oracle.quantize(want, 2.5, 3)
    assert np.array_equal(nxt.cpu().numpy(), lv.astype(np.int8))


def _nibbles(lv):
    lv = np.asarray(lv).astype(np.int64)
    code = np.where(lv < 0, 8, 0) | np.where(np.abs(lv) == 3, 5, 2)
    return (code[..., 0::2] | (code[..., 1::2] << 4)).astype(np.uint8)


@pytest.mark.parametrize("geom", [g for g in GEOMS if g[3] % 32 == 0])
@pytest.mark.parametrize("bits", [(2, 2), (1, 1), (2, 1)])
def test_level_deconv_fp4(geom, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits = bits
    a, w, s, bias = _case(geom, w_bits, a_bits)
    a4, w4 = qnn.qnn_levels_to_fp4(dev(a)), qnn.qnn_levels_to_fp4(dev(w))
    fw = qnn.qnn_level_deconv_flip_weights(w4)
    even = Cout % 2 == 0
    acc, out, nxt = qnn.qnn_level_deconv2d_fp4(a4, fw, stride, pad, a_bits, w_bits, scale=dev(s), bias=dev(bias),
                                               want_out=True, next_clip=2.5 if even else None, next_bits=2 if even else 0)
    torch.cuda.synchronize()
    want_acc = oracle.deconv2d(a, w, stride, pad)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    want = oracle.block_epilogue(want_acc, s, bias)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=RTOL, atol=0)
    if even:
        lv, _ = oracle.quantize(want, 2.5, 2)
        assert np.array_equal(nxt.cpu().numpy(), _nibbles(lv))


def test_level_deconv_equals_plane_route_and_reuses_workspace():
    # the benchmark's layer at a small batch: both routes give the same integers; one workspace serves two calls,
    # the second on a smaller input (whatever the first left behind the smaller tensor is not read)
    B, H, W, Cin, Cout, k, stride, pad = 4, 28, 28, 128, 64, 4, 2, 1
    gen = np.random.default_rng(77)
    a, w = levels(gen, (B, H, W, Cin), 2), levels(gen, (Cout, k, k, Cin), 2)
    fw = qnn.qnn_level_deconv_flip_weights(dev(w))
    ws = torch.empty((B * (2 * H - 1) * (2 * W - 1) * Cin,), dtype=torch.uint8, device="cuda")
    acc, _, _ = qnn.qnn_level_deconv2d_i8(dev(a), fw, stride, pad, 2, 2, workspace=ws)
    wp = pack_levels(w, 2).view(2, Cout, k, k, -1)
    ph = qnn.qnn_deconv_pack_weights(wp, Cin, stride)
    acc_planes, _, _ = qnn.qnn_deconv2d(pack_levels(a, 2), ph, (B, H, W), Cin, Cout, k, k, stride, pad, 2)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc_planes)
    assert np.array_equal(acc.cpu().numpy(), oracle.deconv2d(a, w, stride, pad))
    small = a[:1, :9, :11]
    acc2, _, _ = qnn.qnn_level_deconv2d_i8(dev(np.ascontiguousarray(small)), fw, stride, pad, 2, 2, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(acc2.cpu().numpy(), oracle.deconv2d(np.ascontiguousarray(small), w, stride, pad))
