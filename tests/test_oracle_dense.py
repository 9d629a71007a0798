"""Pins of the oracle's unquantized layers (dense_conv2d, dense_layer, global_avgpool, dense_fc) against
things other than themselves: brute-force loops on tiny shapes, the library's float64 convolution, closed
forms (one-hot kernels shift the image, all-ones tensors count taps), and the integer convolution of the
quantized path on integer-valued inputs."""
import numpy as np
import pytest
import torch

import oracle


def _brute(x, w, stride, pad):
    B, H, W, Cin = x.shape
    Cout, kh, kw, _ = w.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    out = np.zeros((B, Ho, Wo, Cout))
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(Cout):
                    acc = 0.0
                    for ky in range(kh):
                        for kx in range(kw):
                            y, xx = ho * stride + ky - pad, wo * stride + kx - pad
                            if 0 <= y < H and 0 <= xx < W:
                                for ci in range(Cin):
                                    acc += float(x[b, y, xx, ci]) * float(w[co, ky, kx, ci])
                    out[b, ho, wo, co] = acc
    return out


@pytest.mark.parametrize("geom", [(1, 5, 6, 3, 4, 3, 3, 1, 1), (2, 7, 5, 2, 3, 3, 2, 2, 1), (1, 9, 9, 3, 2, 7, 7, 2, 3),
                                  (1, 4, 4, 1, 1, 1, 1, 1, 0), (1, 6, 8, 2, 2, 5, 3, 3, 2)])
def test_dense_conv_against_brute_force(geom):
    B, H, W, Cin, Cout, kh, kw, stride, pad = geom
    gen = np.random.default_rng(sum(geom))
    x = gen.normal(size=(B, H, W, Cin)).astype(np.float32)
    w = gen.normal(size=(Cout, kh, kw, Cin)).astype(np.float32)
    np.testing.assert_allclose(oracle.dense_conv2d(x, w, stride, pad), _brute(x, w, stride, pad), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("geom", [(2, 20, 17, 3, 8, 7, 7, 2, 3), (1, 16, 16, 5, 6, 3, 3, 1, 1), (2, 11, 13, 4, 4, 5, 5, 3, 2)])
def test_dense_conv_against_library_float64(geom):
    B, H, W, Cin, Cout, kh, kw, stride, pad = geom
    gen = np.random.default_rng(sum(geom) + 1)
    x = gen.normal(size=(B, H, W, Cin)).astype(np.float32)
    w = gen.normal(size=(Cout, kh, kw, Cin)).astype(np.float32)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                     torch.from_numpy(w).double().permute(0, 3, 1, 2), stride=stride, padding=pad)
    np.testing.assert_allclose(oracle.dense_conv2d(x, w, stride, pad), ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)


def test_one_hot_kernel_shifts_the_image():
    gen = np.random.default_rng(5)
    x = gen.normal(size=(1, 8, 9, 3)).astype(np.float32)
    for ky, kx, ci in [(0, 0, 0), (2, 1, 2), (1, 2, 1)]:
        w = np.zeros((1, 3, 3, 3), np.float32)
        w[0, ky, kx, ci] = 1.0
        out = oracle.dense_conv2d(x, w, 1, 1)[0, :, :, 0]
        want = np.zeros((8, 9))
        for i in range(8):
            for j in range(9):
                y, xx = i + ky - 1, j + kx - 1
                if 0 <= y < 8 and 0 <= xx < 9:
                    want[i, j] = x[0, y, xx, ci]
        assert np.array_equal(out, want)


def test_all_ones_count_valid_taps():
    x, w = np.ones((1, 6, 6, 3), np.float32), np.ones((2, 3, 3, 3), np.float32)
    out = oracle.dense_conv2d(x, w, 1, 1)
    assert out[0, 0, 0, 0] == 4 * 3 and out[0, 0, 3, 1] == 6 * 3 and out[0, 2, 2, 0] == 9 * 3
    out2 = oracle.dense_conv2d(x, w, 2, 1)   # windows start at -1, 1, 3
    assert out2.shape == (1, 3, 3, 2) and out2[0, 0, 0, 0] == 12 and out2[0, 1, 1, 0] == 27


def test_integer_inputs_match_the_quantized_convolution():
    gen = np.random.default_rng(9)
    a = (2 * gen.integers(0, 4, size=(2, 9, 9, 8)) - 3).astype(np.int8)
    w = (2 * gen.integers(0, 4, size=(5, 3, 3, 8)) - 3).astype(np.int8)
    for stride, pad in [(1, 1), (2, 1), (1, 0)]:
        assert np.array_equal(oracle.dense_conv2d(a, w, stride, pad), oracle.conv2d(a, w, stride, pad).astype(np.float64))


def test_dense_layer_terms_and_magnitude():
    gen = np.random.default_rng(11)
    x = gen.normal(size=(1, 6, 6, 3)).astype(np.float32)
    w = gen.normal(size=(4, 3, 3, 3)).astype(np.float32)
    sc, sh = gen.uniform(0.5, 2, size=4).astype(np.float32), gen.normal(size=4).astype(np.float32)
    conv = _brute(x, w, 1, 1)
    y, mag = oracle.dense_layer(x, w, 1, 1, sc, sh, relu=True)
    np.testing.assert_allclose(y, np.maximum(conv * sc.astype(np.float64) + sh.astype(np.float64), 0), rtol=1e-12, atol=1e-12)
    assert (y >= 0).all() and (mag >= np.abs(conv * sc + sh) - 1e-9).all()
    y2, _ = oracle.dense_layer(x, w, 1, 1)
    np.testing.assert_allclose(y2, conv, rtol=1e-12, atol=1e-12)


def test_global_avgpool_and_fc():
    gen = np.random.default_rng(13)
    x = gen.normal(size=(3, 7, 7, 10)).astype(np.float32)
    np.testing.assert_allclose(oracle.global_avgpool(x), x.astype(np.float64).mean(axis=(1, 2)), rtol=1e-13, atol=1e-13)
    const = np.broadcast_to(np.arange(10, dtype=np.float32), (2, 4, 5, 10))
    assert np.array_equal(oracle.global_avgpool(const), np.broadcast_to(np.arange(10.0), (2, 10)))
    v, w, b = gen.normal(size=(3, 10)).astype(np.float32), gen.normal(size=(6, 10)).astype(np.float32), gen.normal(size=6).astype(np.float32)
    out, mag = oracle.dense_fc(v, w, b)
    want = np.array([[sum(float(v[r, i]) * float(w[o, i]) for i in range(10)) + float(b[o]) for o in range(6)] for r in range(3)])
    np.testing.assert_allclose(out, want, rtol=1e-13, atol=1e-13)
    assert (mag >= np.abs(out)).all()
    # a 1x1 convolution over a 1x1 image is the same layer
    np.testing.assert_allclose(oracle.dense_conv2d(v.reshape(3, 1, 1, 10), w.reshape(6, 1, 1, 10), 1, 0).reshape(3, 6) + b, out, rtol=1e-13, atol=1e-13)
