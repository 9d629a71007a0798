"""Pins of the oracle's transposed convolution: the library routine in float64, the adjoint identity
that defines a transposed convolution, brute force on a tiny case, and the stride-1 special case."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl

CASES = [
    # B, H, W, Cin, Cout, k, stride, pad
    (2, 5, 6, 7, 3, 4, 2, 1),
    (1, 4, 4, 5, 6, 3, 2, 1),
    (1, 3, 5, 4, 2, 2, 2, 0),
    (2, 4, 3, 3, 4, 3, 1, 1),
    (1, 3, 3, 2, 2, 5, 3, 2),
    (1, 6, 5, 8, 3, 3, 2, 0),
]


def _rand(case, seed):
    B, H, W, Cin, Cout, k, s, p = case
    gen = np.random.default_rng(seed)
    return wl.odd_levels(gen, (B, H, W, Cin), 3), wl.odd_levels(gen, (Cout, k, k, Cin), 2)


@pytest.mark.parametrize("case", CASES)
def test_matches_library_transposed_convolution(case):
    a, w = _rand(case, 1)
    s, p = case[6], case[7]
    x = torch.from_numpy(a.astype(np.float64)).permute(0, 3, 1, 2)
    k = torch.from_numpy(w.astype(np.float64)).permute(3, 0, 1, 2)      # [Cin][Cout][kh][kw]
    want = torch.nn.functional.conv_transpose2d(x, k, stride=s, padding=p).permute(0, 2, 3, 1).numpy()
    got = oracle.deconv2d(a, w, s, p)
    assert got.shape == want.shape and np.array_equal(got, want.astype(np.int64))


@pytest.mark.parametrize("case", CASES)
def test_is_the_adjoint_of_the_convolution(case):
    # <conv(x; w~), y> = <x, deconv(y; w)> with w~ = w with its channel axes exchanged
    B, H, W, Cin, Cout, k, s, p = case
    a, w = _rand(case, 2)
    y = oracle.deconv2d(a, w, s, p)                                 # [B][Ho][Wo][Cout]
    gen = np.random.default_rng(3)
    z = wl.odd_levels(gen, y.shape, 2)                              # a tensor of deconv's output shape
    wt = np.ascontiguousarray(np.transpose(w, (3, 1, 2, 0)))        # [Cin][kh][kw][Cout]
    back = oracle.conv2d(z, wt, s, p)                               # [B][H'][W'][Cin]
    assert back.shape[1] >= H and back.shape[2] >= W                # floor in the conv's size formula may add a row
    lhs = int((back[:, :H, :W, :].astype(np.int64) * a).sum())
    rhs = int((z.astype(np.int64) * y).sum())
    assert lhs == rhs


def test_brute_force_tiny():
    a, w = _rand((1, 2, 3, 2, 2, 3, 2, 1), 4)
    s, p = 2, 1
    B, H, W, Cin = a.shape
    Cout, kh, kw, _ = w.shape
    Ho, Wo = (H - 1) * s - 2 * p + kh, (W - 1) * s - 2 * p + kw
    want = np.zeros((B, Ho, Wo, Cout), np.int64)
    for y in range(Ho):
        for x in range(Wo):
            for i in range(H):
                for j in range(W):
                    ky, kx = y + p - i * s, x + p - j * s
                    if 0 <= ky < kh and 0 <= kx < kw:
                        for co in range(Cout):
                            want[0, y, x, co] += int(a[0, i, j].astype(np.int64) @ w[co, ky, kx].astype(np.int64))
    assert np.array_equal(oracle.deconv2d(a, w, s, p), want)


def test_stride_one_is_a_convolution_with_the_flipped_kernel():
    a, w = _rand((2, 5, 4, 6, 3, 3, 1, 1), 5)
    flipped = np.ascontiguousarray(w[:, ::-1, ::-1, :])
    assert np.array_equal(oracle.deconv2d(a, w, 1, 1), oracle.conv2d(a, flipped, 1, 3 - 1 - 1))


def test_random_rectangular_geometries_against_library():
    gen = np.random.default_rng(7)
    for _ in range(40):
        s = int(gen.integers(1, 5))
        kh, kw, p = int(gen.integers(s, 8)), int(gen.integers(s, 8)), int(gen.integers(0, 4))
        B, H, W, Cin, Cout = (int(gen.integers(1, 4)), int(gen.integers(1, 9)), int(gen.integers(1, 9)),
                              int(gen.integers(1, 9)), int(gen.integers(1, 6)))
        if (H - 1) * s - 2 * p + kh < 1 or (W - 1) * s - 2 * p + kw < 1:
            continue
        a, w = wl.odd_levels(gen, (B, H, W, Cin), 2), wl.odd_levels(gen, (Cout, kh, kw, Cin), 3)
        x = torch.from_numpy(a.astype(np.float64)).permute(0, 3, 1, 2)
        k = torch.from_numpy(w.astype(np.float64)).permute(3, 0, 1, 2)
        want = torch.nn.functional.conv_transpose2d(x, k, stride=s, padding=p).permute(0, 2, 3, 1).numpy()
        assert np.array_equal(oracle.deconv2d(a, w, s, p), want.astype(np.int64)), (B, H, W, Cin, Cout, kh, kw, s, p)
