"""GPU parity: qnn_binary_gemm against the CPU oracle (integer matmul of decoded levels).
int32 accumulators must match bit for bit; fp32 scaled outputs within 1e-5 relative."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, pack_levels, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

RTOL = 1e-5


def _run(a, w, a_bits, w_bits, scale=None):
    ap, wp = pack_levels(a, a_bits), pack_levels(w, w_bits)
    acc, out = qnn.qnn_binary_gemm(ap, wp, a.shape[1], scale=None if scale is None else dev(scale))
    torch.cuda.synchronize()
    return acc.cpu().numpy(), None if out is None else out.cpu().numpy()


def test_config1_fc_2x2():
    c = wl.fc_2x2()
    acc, out = _run(c["a"], c["w"], 2, 2, c["scale"])
    want = oracle.gemm(c["a"], c["w"])
    assert np.array_equal(acc, want)
    np.testing.assert_allclose(out, oracle.scale(want, c["scale"]), rtol=RTOL, atol=0)


@pytest.mark.parametrize("w_bits", [1, 2, 3, 4])
@pytest.mark.parametrize("a_bits", [1, 2, 3, 4])
@pytest.mark.parametrize("shape", [(1, 1, 1), (130, 70, 100), (257, 129, 1000), (64, 300, 2080), (300, 64, 33)])
def test_tiled_kernels_ragged(w_bits, a_bits, shape):
    rows, cols, n = shape
    gen = np.random.default_rng(w_bits * 100 + a_bits * 10 + rows)
    a, w = levels(gen, (rows, n), a_bits), levels(gen, (cols, n), w_bits)
    s = gen.uniform(0.01, 0.1, size=cols).astype(np.float32)
    acc, out = _run(a, w, a_bits, w_bits, s)
    want = oracle.gemm(a, w)
    assert np.array_equal(acc, want)
    np.testing.assert_allclose(out, oracle.scale(want, s), rtol=RTOL, atol=0)


def _wide_levels(gen, shape, bits):
    top = (1 << bits) - 1
    return (2 * gen.integers(0, top + 1, size=shape) - top).astype(np.int16)


WIDE_BITS = [(5, 5), (8, 2), (3, 7), (1, 6), (8, 8), (6, 5), (7, 8), (4, 5), (5, 4)]


@pytest.mark.parametrize("bits", WIDE_BITS)
@pytest.mark.parametrize("shape", [(37, 19, 200), (130, 70, 1000), (257, 129, 33)])
def test_wide_bits_run_as_plane_chunks(bits, shape):
    # widths above 4 are split into chunks of at most 4 planes; the chunk pairs' results are summed
    # with their 2^shift weights in the int32 accumulator, also when only the scaled output is asked for
    w_bits, a_bits = bits
    rows, cols, n = shape
    gen = np.random.default_rng(w_bits * 10 + a_bits + rows)
    a, w = _wide_levels(gen, (rows, n), a_bits), _wide_levels(gen, (cols, n), w_bits)
    s = gen.uniform(0.01, 0.1, size=cols).astype(np.float32)
    ap = dev(oracle.pack_planes(a, a_bits).view(np.int32))   # 8-bit levels do not fit the int8 input path
    wp = dev(oracle.pack_planes(w, w_bits).view(np.int32))
    acc, out = qnn.qnn_binary_gemm(ap, wp, n, scale=dev(s))
    _, out_only = qnn.qnn_binary_gemm(ap, wp, n, want_acc=False, scale=dev(s))
    acc_only, _ = qnn.qnn_binary_gemm(ap, wp, n)
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    assert np.array_equal(acc.cpu().numpy(), want)
    assert np.array_equal(acc_only.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=RTOL, atol=0)
    assert torch.equal(out, out_only)


def test_wide_bits_extreme_levels():
    # 8 x 8 bit at the largest n the int32 accumulator allows: |acc| = n 255^2
    n = 33025
    a = np.full((3, n), 255, np.int16)
    w = np.stack([np.full(n, 255, np.int16), np.full(n, -255, np.int16)])
    a[2, ::2] = -255
    acc, _ = qnn.qnn_binary_gemm(dev(oracle.pack_planes(a, 8).view(np.int32)),
                                 dev(oracle.pack_planes(w, 8).view(np.int32)), n)
    torch.cuda.synchronize()
    want = a.astype(np.int64) @ w.astype(np.int64).T
    assert want[0, 0] == n * 255 * 255 < 2 ** 31
    assert np.array_equal(acc.cpu().numpy(), want)
    assert np.array_equal(oracle.gemm(a, w), want)


def test_extreme_levels_hit_the_bound():
    # all-max inputs reach |acc| = n (2^M-1)(2^K-1); sign flips with the weights
    n = 4096
    a = np.full((16, n), 15, np.int8)
    w = np.concatenate([np.full((8, n), 15, np.int8), np.full((8, n), -15, np.int8)])
    acc, _ = _run(a, w, 4, 4)
    assert np.all(acc[:, :8] == n * 225) and np.all(acc[:, 8:] == -n * 225)


def test_only_out_requested():
    gen = np.random.default_rng(3)
    a, w = levels(gen, (40, 96), 2), levels(gen, (24, 96), 2)
    s = gen.uniform(0.01, 0.1, size=24).astype(np.float32)
    _, out = qnn.qnn_binary_gemm(pack_levels(a, 2), pack_levels(w, 2), 96, want_acc=False, scale=dev(s))
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(oracle.gemm(a, w), s), rtol=RTOL, atol=0)


@pytest.mark.parametrize("w_bits", [1, 2, 3, 4])
@pytest.mark.parametrize("a_bits", [1, 2, 3, 4])
def test_config2_full_size_every_output(w_bits, a_bits):
    # 4096^3 in the launch configuration the benchmark times, against the oracle's whole product
    size = 4096
    c = wl.gemm_square(w_bits, a_bits, size)
    a, w = c["a"], c["w"]
    ap, wp = pack_levels(a, a_bits), pack_levels(w, w_bits)
    acc, out = qnn.qnn_binary_gemm(ap, wp, size, scale=dev(c["scale"]))
    torch.cuda.synchronize()
    acc = acc.cpu().numpy()
    out = out.cpu().numpy()
    want = oracle.gemm(a, w)
    assert np.array_equal(acc, want)
    # single outputs through the oracle's scalar routine, and invariants that hold for every output
    gen = np.random.default_rng(w_bits * 10 + a_bits)
    for r, col in zip(gen.integers(0, size, 64), gen.integers(0, size, 64)):
        assert acc[r, col] == oracle.gemm_one(a[r], w[col])
    top = ((1 << w_bits) - 1) * ((1 << a_bits) - 1)
    assert np.all((acc & 1) == 0)                      # n even -> sum of n odd products is even
    assert np.abs(acc).max() <= size * top
    np.testing.assert_allclose(out, oracle.scale(want, c["scale"]), rtol=RTOL, atol=0)


@pytest.mark.parametrize("bits", [(5, 5), (7, 6)])
def test_full_size_wide_bits_sampled(bits):
    # 4096^3 above 4 bits (four chunk-pair launches), checked like the sweep configurations
    w_bits, a_bits = bits
    size = 4096
    c = wl.gemm_square(w_bits, a_bits, size)
    a, w = c["a"], c["w"]
    acc, out = qnn.qnn_binary_gemm(pack_levels(a, a_bits), pack_levels(w, w_bits), size, scale=dev(c["scale"]))
    torch.cuda.synchronize()
    acc = acc.cpu().numpy()
    gen = np.random.default_rng(w_bits * 10 + a_bits)
    rsel = np.concatenate([[0, size - 1], gen.integers(0, size, 4)])
    csel = np.concatenate([[0, size - 1], gen.integers(0, size, 4)])
    assert np.array_equal(acc[rsel], oracle.gemm(a[rsel], w))
    assert np.array_equal(acc[:, csel], oracle.gemm(a, w[csel]))
    assert np.all((acc & 1) == 0)
    assert np.array_equal(out.cpu().numpy(), acc.astype(np.float32) * c["scale"][None, :])


@pytest.mark.parametrize("case", [(1, 1, (1 << 24) + 37), (2, 2, (1 << 22) + 5), (4, 4, 9544371)])
def test_longest_reductions(case):
    # reduction lengths near the int32 limit of each width (4 x 4 bit: n 225 < 2^31 -> n <= 9544371),
    # ragged against the 32-bit words; a few rows and columns only
    w_bits, a_bits, n = case
    gen = np.random.default_rng(n % 1000)
    a, w = levels(gen, (3, n), a_bits), levels(gen, (5, n), w_bits)
    a[0] = (1 << a_bits) - 1                      # a row at the positive extreme
    w[0] = (1 << w_bits) - 1
    w[1] = -((1 << w_bits) - 1)
    ap, wp = pack_levels(a, a_bits), pack_levels(w, w_bits)
    acc, _ = qnn.qnn_binary_gemm(ap, wp, n)
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    top = ((1 << a_bits) - 1) * ((1 << w_bits) - 1)
    assert want[0, 0] == n * top and want[0, 1] == -n * top
    assert np.array_equal(acc.cpu().numpy(), want)
    if w_bits == 4:
        assert (n + 1 + 31) // 32 == (n + 31) // 32       # same planes, one element more than int32 allows
        with pytest.raises(qnn.QnnError) as e:
            qnn.qnn_binary_gemm(ap, wp, n + 1)
        assert e.value.code == -4
