"""Pins of the oracle's max-pooling (CPU only): a library routine on the same integers, the
commutation with the quantizer that justifies pooling codes at all, and brute force."""
import numpy as np
import pytest
import torch

import oracle

GEOMS = [
    # H, W, k, stride, pad, ceil_mode
    (8, 8, 2, 2, 0, False),
    (7, 9, 2, 2, 0, False),     # floor mode drops the ragged border
    (7, 9, 2, 2, 0, True),      # ceil mode keeps it (75 -> 38 in the detection backbone)
    (75, 75, 2, 2, 0, True),
    (12, 10, 3, 2, 1, False),   # the residual network's stem pooling
    (9, 9, 3, 1, 1, False),     # 3x3 stride 1 pad 1 (keeps the size)
    (10, 7, 3, 3, 1, True),
    (5, 5, 5, 1, 2, False),
    (5, 5, 2, 2, 1, True),      # the window that would start in the right padding is dropped
]


@pytest.mark.parametrize("geom", GEOMS)
def test_maxpool_equals_library_routine(geom):
    H, W, k, s, p, ceil_mode = geom
    gen = np.random.default_rng(sum(geom[:5]))
    lv = (2 * gen.integers(0, 8, size=(2, H, W, 5)) - 7).astype(np.int8)
    got = oracle.maxpool(lv, k, s, p, ceil_mode)
    t = torch.from_numpy(lv.astype(np.float64)).permute(0, 3, 1, 2)
    want = torch.nn.functional.max_pool2d(t, k, s, p, ceil_mode=ceil_mode).permute(0, 2, 3, 1).numpy()
    assert got.shape == want.shape
    assert np.array_equal(got.astype(np.float64), want)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_pooling_commutes_with_the_quantizer(bits):
    # monotone quantizer: max of the quantized values = quantized max (on fp32 inputs with ties,
    # saturation and both signs)
    gen = np.random.default_rng(bits)
    x = gen.normal(0, 1.2, size=(3, 10, 11, 4)).astype(np.float32)
    x[0, :2] = 0.0
    clip = 2.0
    lv, _ = oracle.quantize(x, clip, bits)
    pooled_then_q, _ = oracle.quantize(
        torch.nn.functional.max_pool2d(torch.from_numpy(x).permute(0, 3, 1, 2), 2, 2).permute(0, 2, 3, 1)
        .contiguous().numpy(), clip, bits)
    assert np.array_equal(oracle.maxpool(lv, 2, 2), pooled_then_q)


def test_maxpool_brute_force_and_special_cases():
    gen = np.random.default_rng(3)
    lv = (2 * gen.integers(0, 4, size=(1, 5, 6, 2)) - 3).astype(np.int8)
    got = oracle.maxpool(lv, 2, 2)
    for oy in range(2):
        for ox in range(3):
            for c in range(2):
                assert got[0, oy, ox, c] == max(lv[0, 2 * oy + dy, 2 * ox + dx, c] for dy in (0, 1) for dx in (0, 1))
    assert np.array_equal(oracle.maxpool(lv, 1, 1), lv)                       # 1x1 window: identity
    assert np.array_equal(oracle.maxpool(lv, 5, 1, 0)[0, 0, 0], lv[0, :5, :5].reshape(-1, 2).max(0))
    assert np.array_equal(oracle.maxpool(-lv, 2, 2), -_minpool(lv))           # max(-x) = -min(x)
    with pytest.raises(ValueError):
        oracle.maxpool(lv, 7, 1)
    assert oracle.pool_out_size(75, 2, 2, 0, True) == 38 and oracle.pool_out_size(75, 2, 2, 0, False) == 37
    assert oracle.pool_out_size(112, 3, 2, 1, False) == 56


def _minpool(lv):
    B, H, W, C = lv.shape
    return lv[:, :H // 2 * 2, :W // 2 * 2].reshape(B, H // 2, 2, W // 2, 2, C).min(axis=(2, 4))
