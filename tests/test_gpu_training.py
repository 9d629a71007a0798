"""GPU parity of the training-side gradients (qnn_quantize_ste_backward, qnn_encoder_backward) against
the CPU oracle's float64 values."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402


def _x(gen, count):
    x = gen.normal(0, 1.2, size=count).astype(np.float32)
    edge = np.array([0.0, 1.0, -1.0, 2.0, -2.0, np.nextafter(np.float32(2), np.float32(3)), 1e-30, -5.0], np.float32)
    x[: min(count, edge.size)] = edge[: min(count, edge.size)]
    return x


@pytest.mark.parametrize("count", [1, 3, 4, 1023, 4096, 3 * 4096 + 5, 1 << 20])
@pytest.mark.parametrize("clip", [1.0, 2.0, 0.37])
def test_quantize_ste_backward(count, clip):
    gen = np.random.default_rng(count)
    x, g = _x(gen, count), gen.normal(size=count).astype(np.float32)
    got = qnn.qnn_quantize_ste_backward(dev(x), dev(g), clip)
    torch.cuda.synchronize()
    want = oracle.quantize_ste_backward(x, g, clip)
    # one fp32 multiply against the float64 product; the zero pattern is exact
    got = got.cpu().numpy()
    assert np.array_equal(got == 0, want == 0)
    np.testing.assert_allclose(got, want, rtol=1e-6, atol=0)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("count", [1, 5, 4096, 3 * 4096 + 7, 1 << 18])
@pytest.mark.parametrize("clip", [1.0, 2.0])
def test_encoder_backward(bits, count, clip):
    gen = np.random.default_rng(bits * 100 + count % 97)
    x, g = _x(gen, count), gen.normal(size=(bits, count)).astype(np.float32)
    got = qnn.qnn_encoder_backward(dev(x), dev(g), clip).cpu().numpy()
    torch.cuda.synchronize()
    want = oracle.encoder_backward(x, g, clip, bits)
    K = (1 << bits) - 1
    s = np.array([np.pi * K / (1 << m) for m in range(1, bits + 1)])
    # the bound the header states (argument rounding of the cosine plus a few roundings per term), doubled
    bound = 2 * (np.abs(g.astype(np.float64)) * (s * (s + 4))[:, None]).sum(0) * 2.0 ** -24 / clip
    assert np.all(np.abs(got - want) <= bound + 1e-30)
    outside = np.abs(x.astype(np.float64) * np.float64(np.float32(1) / np.float32(clip))) > 1
    assert np.all(got[outside] == 0)
    # at 2 bits and unit clip: Eq. 12-13 at x = 0
    if bits == 2 and clip == 1.0 and count >= 1:
        one = oracle.encoder_backward(np.zeros(1, np.float32), np.array([[0.0], [1.0]]), 1.0, 2)
        assert abs(one[0] - 0.75 * np.pi) < 1e-12


def test_binarize_forward_is_one_bit_encode_pack():
    x = np.array([-3, -1, -0.2, 0.0, 0.3, 1, 7, -0.0] * 8, np.float32)
    planes = qnn.qnn_encode_pack(dev(x.reshape(1, -1)), 1.0, 1)
    torch.cuda.synchronize()
    lv, _ = oracle.quantize(x, 1.0, 1)
    assert np.array_equal(planes.cpu().numpy().view(np.uint32), oracle.pack_planes(lv.reshape(1, -1), 1))
