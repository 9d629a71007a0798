"""GPU parity: qnn_maxpool_planes / qnn_maxpool_levels_i8 against the oracle's pooling of decoded levels."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, pack_levels, planes_to_numpy, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

GEOMS = [
    # B, H, W, C, k, stride, pad, ceil_mode
    (2, 8, 8, 32, 2, 2, 0, False),
    (1, 7, 9, 5, 2, 2, 0, False),       # ragged channels (pad bits stay 0), ragged border dropped
    (1, 7, 9, 40, 2, 2, 0, True),       # ceil mode keeps the border windows
    (2, 12, 10, 64, 3, 2, 1, False),    # stem pooling of a residual network
    (1, 9, 9, 100, 3, 1, 1, False),
    (3, 10, 7, 16, 3, 3, 1, True),
    (1, 5, 5, 33, 5, 1, 2, False),
    (2, 75, 75, 128, 2, 2, 0, True),    # 75 -> 38 of the detection backbone
]


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_maxpool_planes(geom, bits):
    B, H, W, C, k, s, p, ceil_mode = geom
    gen = np.random.default_rng(sum(geom[:7]) + bits)
    top = (1 << bits) - 1
    lv = (2 * gen.integers(0, top + 1, size=(B, H, W, C)) - top).astype(np.int16)
    planes = dev(oracle.pack_planes(lv.reshape(-1, C), bits).view(np.int32))
    got = qnn.qnn_maxpool_planes(planes, (B, H, W), C, k, s, p, ceil_mode)
    want = oracle.maxpool(lv, k, s, p, ceil_mode)
    assert qnn.qnn_pool_out_size(H, k, s, p, ceil_mode) == want.shape[1]
    assert qnn.qnn_pool_out_size(W, k, s, p, ceil_mode) == want.shape[2]
    assert np.array_equal(planes_to_numpy(got), oracle.pack_planes(want.reshape(-1, C), bits))


@pytest.mark.parametrize("geom", GEOMS)
def test_maxpool_levels(geom):
    B, H, W, C, k, s, p, ceil_mode = geom
    gen = np.random.default_rng(sum(geom[:7]))
    lv = levels(gen, (B, H, W, C), 7)
    got = qnn.qnn_maxpool_levels_i8(dev(lv), k, s, p, ceil_mode)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.maxpool(lv, k, s, p, ceil_mode))


def test_pooled_chain_matches_pooling_before_the_quantizer():
    # conv -> scale -> quantize -> pool (on planes) equals the oracle's quantize(pool(fp32 out)): the
    # commutation that lets the pooling run on codes
    gen = np.random.default_rng(9)
    a, w = levels(gen, (2, 12, 12, 64), 3), levels(gen, (64, 3, 3, 64), 3)
    s = (gen.uniform(0.5, 1.5, size=64) / np.sqrt(9 * 64 * 21 * 21)).astype(np.float32)
    _, _, nxt = qnn.qnn_conv2d(pack_levels(a, 3), pack_levels(w, 3).view(3, 64, 3, 3, -1), (2, 12, 12), 64, 1, 1,
                               scale=dev(s), want_acc=False, next_clip=2.5, next_bits=3)
    pooled = qnn.qnn_maxpool_planes(nxt, (2, 12, 12), 64, 2, 2)
    out = oracle.scale(oracle.conv2d(a, w, 1, 1), s)
    pooled_fp = out.reshape(2, 6, 2, 6, 2, 64).max(axis=(2, 4))
    lv, _ = oracle.quantize(np.ascontiguousarray(pooled_fp), 2.5, 3)
    assert np.array_equal(planes_to_numpy(pooled), oracle.pack_planes(lv.reshape(-1, 64), 3))


def test_pool_argument_errors():
    x = torch.zeros((1, 4, 4, 16), dtype=torch.int8, device="cuda")
    with pytest.raises(qnn.QnnError) as e:
        qnn.qnn_maxpool_levels_i8(x, 2, 2, pad=2)
    assert e.value.code == -1
    with pytest.raises(qnn.QnnError) as e:
        qnn.qnn_maxpool_levels_i8(x, 6, 1)
    assert e.value.code == -1
