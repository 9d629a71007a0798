"""Pins for the oracle's quantizer, plane split and bit-vector storage (CPU only).

Each test checks the oracle against something other than itself: values printed in the
paper (Table 2), the paper's closed-form 2-bit encoders (Eq. 11), Eq. 15 evaluated in
float64, and closed forms / invariants of the {-1,+1} code (Eq. 10).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _read_table2(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "table2_encoded_states.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            q, hi, lo = line.split()
            rows.append((Fraction(q), int(hi), int(lo)))
    return rows


def test_table2_states(golden_dir):
    # Table 2: the four 2-bit quantized reals and their {high, low} states.
    rows = _read_table2(golden_dir)
    assert len(rows) == 4
    x = np.array([float(q) for q, _, _ in rows], dtype=np.float32)
    level, code = oracle.quantize(x, 1.0, 2)
    planes = oracle.pack_planes(level.reshape(1, -1), 2)  # [2][1][1]
    for t, (q, hi, lo) in enumerate(rows):
        got_lo = 1 if (planes[0, 0, 0] >> t) & 1 else -1
        got_hi = 1 if (planes[1, 0, 0] >> t) & 1 else -1
        assert (got_hi, got_lo) == (hi, lo)
        # x = x1 + 2 x2 (Section "Model Decomposition") and alpha = 3
        assert level[t] == 2 * hi + lo
        assert Fraction(int(level[t]), 3) == q


def _grid(n=100001):
    return np.linspace(-1.0, 1.0, n, dtype=np.float64)


def _away_from_thresholds(x, bits, eps=1e-6):
    # thresholds of Eq. 15: (2^b-1)(x+1)/2 = k + 1/2
    top = (1 << bits) - 1
    z = top * (x + 1.0) / 2.0
    frac = z - np.floor(z)
    return np.abs(frac - 0.5) > eps * top


def test_eq11_two_bit_encoders_on_grid():
    # Eq. 11: phi_2^2 = sign(sin(3/4 pi x)) (high bit), phi_2^1 = sign(-sin(3/2 pi x)) (low bit)
    x = _grid()
    keep = _away_from_thresholds(x, 2) & (np.abs(np.sin(0.75 * np.pi * x)) > 1e-9) \
        & (np.abs(np.sin(1.5 * np.pi * x)) > 1e-9)
    x = x[keep]
    hi = np.sign(np.sin(0.75 * np.pi * x))
    lo = np.sign(-np.sin(1.5 * np.pi * x))
    level, code = oracle.quantize(x.astype(np.float32), 1.0, 2)
    code = code.astype(np.int64)
    assert np.array_equal(((code >> 1) & 1) * 2 - 1, hi.astype(np.int64))
    assert np.array_equal((code & 1) * 2 - 1, lo.astype(np.int64))
    assert np.array_equal(level, (2 * hi + lo).astype(np.int16))


@pytest.mark.parametrize("bits", range(1, 9))
def test_eq15_float64_on_grid(bits):
    # Eq. 15: q_k(x) = 2(<(2^k-1)(x+1)/2>/(2^k-1) - 1/2); level = (2^k-1) q_k(x)
    x = _grid(60001)
    x = x[_away_from_thresholds(x, bits)]
    top = (1 << bits) - 1
    rounded = np.floor(top * (x + 1.0) / 2.0 + 0.5)
    q = 2.0 * (rounded / top - 0.5)
    level, code = oracle.quantize(x.astype(np.float32), 1.0, bits)
    assert np.array_equal(level.astype(np.float64), np.rint(q * top))
    assert np.array_equal(code.astype(np.float64), rounded)


@pytest.mark.parametrize("bits", range(1, 9))
def test_general_trig_encoders(bits):
    # The 2-bit encoders of Eq. 11 generalise (same derivation, Fig. 2's periodic curves) to
    # top bit: sign(sin(pi (2^M-1) x / 2^M)); bit m < M: sign(-sin(pi (2^M-1) x / 2^m)).
    x = _grid(40001)
    x = x[_away_from_thresholds(x, bits, eps=1e-5)]
    top = (1 << bits) - 1
    _, code = oracle.quantize(x.astype(np.float32), 1.0, bits)
    for m in range(1, bits + 1):
        arg = np.pi * top * x / float(1 << m)
        s = np.sin(arg) if m == bits else -np.sin(arg)
        ok = np.abs(s) > 1e-6
        got = ((code[ok] >> (m - 1)) & 1).astype(np.int64) * 2 - 1
        assert np.array_equal(got, np.sign(s[ok]).astype(np.int64)), (bits, m)


@pytest.mark.parametrize("bits", range(1, 9))
def test_level_set_is_all_odd_integers(bits):
    # Eq. 10 and the remark after Eq. 20: 2^M states, odd, |v| <= 2^M - 1
    top = (1 << bits) - 1
    codes = np.arange(top + 1)
    planes = np.zeros((bits, 1, (top + 1 + 31) // 32), dtype=np.uint32)
    for t, u in enumerate(codes):
        for j in range(bits):
            if (u >> j) & 1:
                planes[j, 0, t // 32] |= np.uint32(1 << (t % 32))
    level = oracle.unpack_planes(planes, top + 1)[0]
    assert sorted(level.tolist()) == list(range(-top, top + 1, 2))
    assert np.array_equal(level, 2 * codes - top)


@pytest.mark.parametrize("bits", range(1, 9))
def test_quantizer_shape_properties(bits):
    top = (1 << bits) - 1
    x = np.linspace(-4.0, 4.0, 32001).astype(np.float32)
    for clip in (0.5, 1.0, 3.0):
        level, code = oracle.quantize(x, clip, bits)
        assert np.all(np.diff(code.astype(np.int64)) >= 0)          # monotone ladder
        assert set(np.unique(code).tolist()) == set(range(top + 1))  # every state reached
        assert np.all(level[x >= clip] == top) and np.all(level[x <= -clip] == -top)
        # quantization error of the ladder is at most half a step inside the range
        inside = np.abs(x) <= clip
        err = np.abs(level[inside].astype(np.float64) / top - x[inside].astype(np.float64) / clip)
        assert err.max() <= 1.0 / top + 1e-6
    # x = 0 sits on a threshold for every bit width; round-half-up gives the positive middle level
    level, _ = oracle.quantize(np.zeros(1, np.float32), 1.0, bits)
    assert level[0] == 1
    # infinities saturate
    level, _ = oracle.quantize(np.array([np.inf, -np.inf], np.float32), 2.0, bits)
    assert level.tolist() == [top, -top]


def test_bit_layout_lsb_first():
    # element 32 j + t lives in bit t of word j; bit 1 <=> +1; pad bits are 0
    n = 70
    level = -np.ones((2, n), dtype=np.int16)   # 1-bit: all -1 -> all bits 0
    level[0, 0] = 1
    level[0, 33] = 1
    level[1, 69] = 1
    planes = oracle.pack_planes(level, 1)
    assert planes.shape == (1, 2, 3)
    assert planes[0, 0].tolist() == [1, 2, 0]
    assert planes[0, 1].tolist() == [0, 0, 1 << 5]
    # 3-bit, levels 5, -7, 7, -1 = codes 6 (110), 0 (000), 7 (111), 3 (011); by hand:
    # low plane bits (t=0..3) 0,0,1,1 -> 0b1100; middle 1,0,1,1 -> 0b1101; high 1,0,1,0 -> 0b0101
    lv = np.array([[5, -7, 7, -1]], dtype=np.int16)
    p3 = oracle.pack_planes(lv, 3)
    assert p3[:, 0, 0].tolist() == [0b1100, 0b1101, 0b0101]
    assert np.array_equal(oracle.unpack_planes(p3, 4), lv)


@pytest.mark.parametrize("bits", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("n", [1, 31, 32, 33, 100])
def test_pack_unpack_roundtrip(bits, n):
    gen = np.random.default_rng(bits * 100 + n)
    top = (1 << bits) - 1
    level = (2 * gen.integers(0, top + 1, size=(5, n)) - top).astype(np.int16)
    planes = oracle.pack_planes(level, bits)
    assert np.array_equal(oracle.unpack_planes(planes, n), level)
    # pad bits are zero
    if n % 32:
        assert np.all(planes[:, :, -1] >> (n % 32) == 0)


def test_pack_rejects_even_or_out_of_range_levels():
    with pytest.raises(ValueError):
        oracle.pack_planes(np.array([[0]], dtype=np.int16), 2)
    with pytest.raises(ValueError):
        oracle.pack_planes(np.array([[5]], dtype=np.int16), 2)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_hrelu_limited_values_use_the_upper_levels(bits):
    # Table 1's HReLU limits the data to [0, 1]; the encoder of Eq. 15 is then applied to that value as
    # it is, so only the non-negative half of the levels occurs, and with one bit every activation is
    # +1 (the special case noted in the experiments section, which is why 1-bit uses HTanh)
    gen = np.random.default_rng(bits)
    x = gen.normal(0, 1, size=20000).astype(np.float32)
    h = np.clip(x, 0.0, 1.0)
    lv, code = oracle.quantize(h, 1.0, bits)
    top = (1 << bits) - 1
    assert lv.min() == 1 and lv.max() == top
    if bits == 1:
        assert np.all(lv == 1)
    else:
        assert len(np.unique(lv)) == (top + 1) // 2
    # Eq. 15 in float64 on the limited value, away from the rounding thresholds
    u = (top * (h.astype(np.float64) + 1.0) / 2.0)
    far = np.abs(u - np.floor(u) - 0.5) > 1e-4
    assert np.array_equal(code[far], np.floor(u[far] + 0.5).astype(code.dtype))
