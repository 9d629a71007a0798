"""GPU parity of the unquantized ends of a network (qnn_dense_conv2d_f32, qnn_global_avgpool_f32,
qnn_dense_fc_f32) against the float64 oracle.  fp32 sums in the kernel's own order: the bound is the
worst case of recursive summation, (terms + 4) 2^-24 sum |x| |w| per output (products, partial sums, the
scale and the shift each round once).  The fused next-layer planes are a decision taken in fp32 on the
kernel's own fp32 value (the fp32 sum has no unique value: it depends on the summation order, and the quantizer
acts on whichever value the kernel holds), so they are compared, bit for bit, with the oracle's quantizer applied
to the GPU's own fp32 output -- never with an oracle-only chain.  What that leaves open is closed separately:
the fp32 value is bounded against the float64 oracle, and every code that differs from the code of the float64
value is counted and must lie within that bound of a threshold of the ladder (codes_explained_by_bound)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import codes_explained_by_bound, dev, planes_to_numpy

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

U = 2.0 ** -24

GEOMS = [
    # B, H, W, Cin, Cout, kh, kw, stride, pad
    (2, 32, 32, 3, 64, 7, 7, 2, 3),      # the ResNet stem's shape: 147 reduction values (odd), one chunk
    (1, 9, 11, 3, 37, 3, 3, 1, 1),       # ragged channels
    (2, 12, 10, 40, 70, 3, 3, 1, 1),     # 360 reduction values: three chunks; two column tiles
    (1, 17, 13, 5, 32, 5, 3, 3, 2),      # rectangular kernel, stride 3
    (3, 8, 8, 16, 130, 1, 1, 1, 0),      # 1x1
    (1, 30, 30, 1, 8, 3, 3, 2, 0),       # one input channel, no padding
    (1, 1, 1, 7, 3, 1, 1, 1, 0),         # a single pixel
]


def _data(geom, seed=0):
    B, H, W, Cin, Cout, kh, kw, stride, pad = geom
    gen = np.random.default_rng(sum(geom) + seed)
    x = gen.normal(size=(B, H, W, Cin)).astype(np.float32)
    w = (gen.normal(size=(Cout, kh, kw, Cin)) / np.sqrt(kh * kw * Cin)).astype(np.float32)
    sc = gen.uniform(0.5, 1.5, size=Cout).astype(np.float32)
    sh = gen.normal(0, 0.3, size=Cout).astype(np.float32)
    return x, w, sc, sh


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("terms", ["plain", "scale", "scale+shift+relu", "shift"])
def test_dense_conv_against_oracle(geom, terms):
    B, H, W, Cin, Cout, kh, kw, stride, pad = geom
    x, w, sc, sh = _data(geom)
    use_sc, use_sh, relu = "scale" in terms, "shift" in terms, "relu" in terms
    out, planes = qnn.qnn_dense_conv2d_f32(dev(x), dev(w), stride, pad, scale=dev(sc) if use_sc else None,
                                           shift=dev(sh) if use_sh else None, relu=relu, next_clip=2.0, next_bits=3)
    torch.cuda.synchronize()
    want, mag = oracle.dense_layer(x, w, stride, pad, sc if use_sc else None, sh if use_sh else None, relu)
    got = out.cpu().numpy()
    assert got.shape == want.shape
    bound = (kh * kw * Cin + 4) * U * mag + 1e-30
    assert (np.abs(got.astype(np.float64) - want) <= bound).all(), float((np.abs(got - want) / bound).max())
    lv, _ = oracle.quantize(got, 2.0, 3)
    assert np.array_equal(planes_to_numpy(planes), oracle.pack_planes(lv.reshape(-1, Cout), 3))
    assert codes_explained_by_bound(got, want, bound, 2.0, 3) <= max(2, got.size // 500)
    # planes only: the fp32 tensor never leaves the chip
    none, planes2 = qnn.qnn_dense_conv2d_f32(dev(x), dev(w), stride, pad, scale=dev(sc) if use_sc else None,
                                             shift=dev(sh) if use_sh else None, relu=relu, want_out=False,
                                             next_clip=2.0, next_bits=3)
    assert none is None and torch.equal(planes2, planes)


def test_stem_at_the_workload_shape():
    geom = (4, 224, 224, 3, 64, 7, 7, 2, 3)
    x, w, sc, sh = _data(geom)
    out, planes = qnn.qnn_dense_conv2d_f32(dev(x), dev(w), 2, 3, scale=dev(sc), shift=dev(sh), relu=True,
                                           next_clip=3.0, next_bits=2)
    torch.cuda.synchronize()
    want, mag = oracle.dense_layer(x, w, 2, 3, sc, sh, True)
    got = out.cpu().numpy()
    assert (np.abs(got.astype(np.float64) - want) <= (147 + 4) * U * mag + 1e-30).all()
    assert codes_explained_by_bound(got, want, (147 + 4) * U * mag + 1e-30, 3.0, 2) <= got.size // 1000
    lv, _ = oracle.quantize(got, 3.0, 2)
    assert np.array_equal(planes_to_numpy(planes), oracle.pack_planes(lv.reshape(-1, 64), 2))
    # the pooled planes feed the first quantized layer: 3x3 stride-2 pooling of the codes
    pooled = qnn.qnn_maxpool_planes(planes, (4, 112, 112), 64, 3, 2, 1)
    want_pool = oracle.maxpool(lv, 3, 2, 1)
    assert np.array_equal(planes_to_numpy(pooled), oracle.pack_planes(want_pool.reshape(-1, 64), 2))


@pytest.mark.parametrize("geom", GEOMS[:4])
@pytest.mark.parametrize("bits", [1, 3, 7])
def test_dense_conv_levels_out(geom, bits):
    B, H, W, Cin, Cout, kh, kw, stride, pad = geom
    x, w, sc, sh = _data(geom, seed=1)
    out, lv = qnn.qnn_dense_conv2d_f32_levels(dev(x), dev(w), stride, pad, 2.0, bits, scale=dev(sc), shift=dev(sh), relu=True,
                                              want_out=True)
    _, planes = qnn.qnn_dense_conv2d_f32(dev(x), dev(w), stride, pad, scale=dev(sc), shift=dev(sh), relu=True,
                                         want_out=False, next_clip=2.0, next_bits=bits)
    torch.cuda.synchronize()
    want, mag = oracle.dense_layer(x, w, stride, pad, sc, sh, True)
    got = out.cpu().numpy()
    assert (np.abs(got.astype(np.float64) - want) <= (kh * kw * Cin + 4) * U * mag + 1e-30).all()
    want_lv, _ = oracle.quantize(got, 2.0, bits)
    assert np.array_equal(lv.cpu().numpy(), want_lv.astype(np.int8))
    assert np.array_equal(planes_to_numpy(planes), oracle.pack_planes(want_lv.reshape(-1, Cout), bits))
    only, _ = qnn.qnn_dense_conv2d_f32_levels(dev(x), dev(w), stride, pad, 2.0, bits, scale=dev(sc), shift=dev(sh), relu=True)
    assert only is None


@pytest.mark.parametrize("shape", [(3, 7, 7, 512), (2, 1, 1, 5), (5, 4, 9, 33), (1, 56, 56, 64)])
def test_global_avgpool(shape):
    gen = np.random.default_rng(sum(shape))
    x = gen.normal(size=shape).astype(np.float32)
    got = qnn.qnn_global_avgpool_f32(dev(x)).cpu().numpy()
    want = oracle.global_avgpool(x)
    hw = shape[1] * shape[2]
    bound = (hw + 2) * U * np.abs(x.astype(np.float64)).sum(axis=(1, 2)) / hw + 1e-30
    assert got.shape == want.shape and (np.abs(got - want) <= bound).all()


@pytest.mark.parametrize("shape", [(37, 1000, 512), (256, 1000, 512), (1, 10, 3), (65, 65, 153), (4, 64, 152)])
@pytest.mark.parametrize("with_bias", [False, True])
def test_dense_fc(shape, with_bias):
    rows, cols, n = shape
    gen = np.random.default_rng(sum(shape))
    x = gen.normal(size=(rows, n)).astype(np.float32)
    w = (gen.normal(size=(cols, n)) / np.sqrt(n)).astype(np.float32)
    b = gen.normal(size=cols).astype(np.float32) if with_bias else None
    got = qnn.qnn_dense_fc_f32(dev(x), dev(w), None if b is None else dev(b)).cpu().numpy()
    want, mag = oracle.dense_fc(x, w, b)
    assert (np.abs(got - want) <= (n + 4) * U * mag + 1e-30).all()


def test_empty_batch_is_a_no_op():
    out, planes = qnn.qnn_dense_conv2d_f32(torch.empty((0, 8, 8, 3), device="cuda"), torch.zeros((4, 3, 3, 3), device="cuda"),
                                           1, 1, next_clip=1.0, next_bits=1)
    assert out.shape == (0, 8, 8, 4) and planes.shape == (1, 0, 1)
    assert qnn.qnn_global_avgpool_f32(torch.empty((0, 2, 2, 3), device="cuda")).shape == (0, 3)
