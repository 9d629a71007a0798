"""GPU parity of the bit-plane-sum variant (qnn_plane_sum_i8 + qnn_level_gemm_i8) against the CPU
oracle and against the xor + bitcount path: identical int32 accumulators."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, pack_levels, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 7])
@pytest.mark.parametrize("shape", [(3, 1), (5, 31), (4, 64), (7, 100), (9, 1000), (130, 4096)])
def test_plane_sum_gives_levels(bits, shape):
    gen = np.random.default_rng(bits * 31 + shape[1])
    lv = levels(gen, shape, bits)
    got = qnn.qnn_plane_sum_i8(pack_levels(lv, bits), shape[1])
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    nk = qnn.qnn_level_row_bytes(shape[1])
    assert got.shape == (shape[0], nk) and nk % 64 == 0 and nk >= shape[1]
    # levels are the decode of the planes (oracle.unpack_planes of oracle.pack_planes is the identity)
    assert np.array_equal(oracle.unpack_planes(oracle.pack_planes(lv.astype(np.int16), bits), shape[1]), lv)
    assert np.array_equal(got[:, :shape[1]], lv)
    assert not got[:, shape[1]:].any()


@pytest.mark.parametrize("bits", [(2, 2), (1, 1), (4, 4), (3, 2), (7, 5)])
@pytest.mark.parametrize("shape", [(1, 1, 1), (130, 70, 100), (257, 300, 1000), (512, 256, 2080), (300, 64, 33)])
def test_level_gemm_matches_oracle_and_binary_path(bits, shape):
    w_bits, a_bits = bits
    rows, cols, n = shape
    gen = np.random.default_rng(w_bits * 100 + a_bits * 10 + rows)
    a, w = levels(gen, (rows, n), a_bits), levels(gen, (cols, n), w_bits)
    s = gen.uniform(0.01, 0.1, size=cols).astype(np.float32)
    ap, wp = pack_levels(a, a_bits), pack_levels(w, w_bits)
    a8, w8 = qnn.qnn_plane_sum_i8(ap, n), qnn.qnn_plane_sum_i8(wp, n)
    acc, out = qnn.qnn_level_gemm_i8(a8, w8, n, scale=dev(s))
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=1e-5, atol=0)
    if max(bits) <= 4:
        acc2, _ = qnn.qnn_binary_gemm(ap, wp, n)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc2)


def test_level_gemm_full_size_equals_binary_path():
    c = wl.gemm_square(2, 2, 4096)
    ap, wp = pack_levels(c["a"], 2), pack_levels(c["w"], 2)
    acc, _ = qnn.qnn_level_gemm_i8(qnn.qnn_plane_sum_i8(ap, 4096), qnn.qnn_plane_sum_i8(wp, 4096), 4096)
    acc2, _ = qnn.qnn_binary_gemm(ap, wp, 4096)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc2)
    rsel = [0, 1234, 4095]
    assert np.array_equal(acc.cpu().numpy()[rsel], oracle.gemm(c["a"][rsel], c["w"]))
