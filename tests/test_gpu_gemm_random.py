"""Seeded random GEMM shapes and bit widths 1..8 on the xor + bitcount path, and up to 7 / 2 bits on
the int8 / fp4 matrix-core routes, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402


def _cases(seed, count, max_bits):
    gen = np.random.default_rng(seed)
    return [(int(gen.integers(1, 400)), int(gen.integers(1, 400)), int(gen.integers(1, 3000)),
             int(gen.integers(1, max_bits + 1)), int(gen.integers(1, max_bits + 1))) for _ in range(count)]


def _operands(case):
    rows, cols, n, w_bits, a_bits = case
    gen = np.random.default_rng(abs(hash(case)) % (2 ** 32))
    ta, tw = (1 << a_bits) - 1, (1 << w_bits) - 1
    a = (2 * gen.integers(0, ta + 1, size=(rows, n)) - ta).astype(np.int16)
    w = (2 * gen.integers(0, tw + 1, size=(cols, n)) - tw).astype(np.int16)
    s = gen.uniform(0.01, 0.1, size=cols).astype(np.float32)
    ap = dev(oracle.pack_planes(a, a_bits).view(np.int32))
    wp = dev(oracle.pack_planes(w, w_bits).view(np.int32))
    return a, w, s, ap, wp


@pytest.mark.parametrize("case", _cases(7, 40, 8))
def test_binary_gemm_random(case):
    a, w, s, ap, wp = _operands(case)
    acc, out = qnn.qnn_binary_gemm(ap, wp, case[2], scale=dev(s))
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    assert np.array_equal(acc.cpu().numpy(), want), case
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=1e-5, atol=0)


@pytest.mark.parametrize("case", _cases(8, 25, 7))
def test_level_gemm_i8_random(case):
    a, w, s, ap, wp = _operands(case)
    n = case[2]
    acc, out = qnn.qnn_level_gemm_i8(qnn.qnn_plane_sum_i8(ap, n), qnn.qnn_plane_sum_i8(wp, n), n, scale=dev(s))
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    assert np.array_equal(acc.cpu().numpy(), want), case
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=1e-5, atol=0)


@pytest.mark.parametrize("case", _cases(9, 25, 2))
def test_level_gemm_fp4_random(case):
    a, w, s, ap, wp = _operands(case)
    n = case[2]
    acc, out = qnn.qnn_level_gemm_fp4(qnn.qnn_plane_sum_fp4(ap, n), qnn.qnn_plane_sum_fp4(wp, n), n, scale=dev(s))
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    assert np.array_equal(acc.cpu().numpy(), want), case
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=1e-5, atol=0)
