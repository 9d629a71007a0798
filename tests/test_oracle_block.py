"""Pins of the residual-block part of the oracle (block_epilogue, residual_trunk) against things other
than itself: the same sums in float64, the library's batch normalisation, Table 2's real values taken
as a shortcut, special cases, and the library's float64 convolution block by block."""
import numpy as np
import torch

import oracle
import qnn_workloads as wl


def _rand_case(seed, rows=37, cols=21, bits=3):
    gen = np.random.default_rng(seed)
    acc = gen.integers(-50000, 50000, size=(rows, cols)).astype(np.int32)
    s = gen.uniform(1e-4, 1e-3, size=cols).astype(np.float32)
    b = gen.uniform(-1, 1, size=cols).astype(np.float32)
    lv = wl.odd_levels(gen, (rows, cols), bits)
    r = gen.normal(0, 2, size=(rows, cols)).astype(np.float32)
    return acc, s, b, lv, r


def test_epilogue_is_the_float64_sum_to_rounding():
    acc, s, b, lv, r = _rand_case(1)
    rs = np.float32(0.37)
    got = oracle.block_epilogue(acc, s, b, lv, rs, r)
    want = acc.astype(np.float64) * s + b + lv.astype(np.float64) * np.float64(rs) + r
    # four fp32 roundings on terms of size <= ~60: absolute error below 4 * 2^-24 * 64
    assert got.dtype == np.float32
    assert np.max(np.abs(got - want)) < 2e-5
    # every term matters at this tolerance: dropping or negating one moves the result by far more
    for wrong in (want - b, want - 2 * b, want - lv * np.float64(rs), want - r, want - 2.0 * r):
        assert np.max(np.abs(got - wrong)) > 1e-2


def test_epilogue_terms_are_optional_and_ordered():
    acc, s, b, lv, r = _rand_case(2)
    base = oracle.scale(acc, s)
    assert np.array_equal(oracle.block_epilogue(acc, s), base)
    assert np.array_equal(oracle.block_epilogue(acc, s, bias=b), base + b)
    assert np.array_equal(oracle.block_epilogue(acc, s, res_f32=r), base + r)
    zeros = np.zeros_like(b)
    assert np.array_equal(oracle.block_epilogue(acc, s, bias=zeros, res_levels=lv, res_scale=0.0), base)
    # the documented order: (((acc * scale) + bias) + level * res_scale) + res_f32, each step rounded to fp32
    rs = np.float32(1.0 / 7.0)
    step = (base + b).astype(np.float32)
    step = (step + (lv.astype(np.float32) * rs).astype(np.float32)).astype(np.float32)
    step = (step + r).astype(np.float32)
    assert np.array_equal(oracle.block_epilogue(acc, s, b, lv, rs, r), step)
    # one element by hand: 3 * 0.5 + 0.25 + (-3) * 0.125 + 1.0 = 2.375, exact in fp32
    one = oracle.block_epilogue(np.array([[3]], np.int32), np.array([0.5], np.float32), np.array([0.25], np.float32),
                                np.array([[-3]], np.int8), 0.125, np.array([[1.0]], np.float32))
    assert one[0, 0] == np.float32(2.375)


def test_table2_values_as_shortcut():
    # Table 2: the 2-bit codes stand for -1, -1/3, 1/3, 1; with res_scale = 1/3 the shortcut term is that value
    lv = np.array([[-3, -1, 1, 3]], np.int8)
    got = oracle.block_epilogue(np.zeros((1, 4), np.int32), np.ones(4, np.float32), None, lv, np.float32(1.0 / 3.0))
    np.testing.assert_allclose(got[0], [-1.0, -1.0 / 3.0, 1.0 / 3.0, 1.0], rtol=1e-7)


def test_folded_batchnorm_matches_library_batchnorm():
    # BN(z) = gamma (z - mean) / sqrt(var + eps) + beta on z = acc * s folds into one factor and one shift
    acc, s, _, _, _ = _rand_case(3, rows=64, cols=16)
    gen = np.random.default_rng(33)
    gamma, beta = gen.uniform(0.5, 2, 16), gen.normal(0, 1, 16)
    mean, var = gen.normal(0, 5, 16), gen.uniform(1, 30, 16)
    eps = 1e-5
    z = torch.from_numpy(acc.astype(np.float64) * s.astype(np.float64))
    want = torch.nn.functional.batch_norm(z, torch.from_numpy(mean), torch.from_numpy(var), torch.from_numpy(gamma),
                                          torch.from_numpy(beta), training=False, eps=eps).numpy()
    k = gamma / np.sqrt(var + eps)
    got = oracle.block_epilogue(acc, (s.astype(np.float64) * k).astype(np.float32), (beta - k * mean).astype(np.float32))
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-4)
    # and the codes of a quantizer behind it agree wherever the float64 value is clear of a threshold
    bits, clip = 3, 6.0
    top = (1 << bits) - 1
    t = np.clip(want / clip, -1, 1)
    v = top * (t + 1) / 2
    clear = np.abs(v + 0.5 - np.round(v + 0.5)) > 1e-3
    _, code = oracle.quantize(got, clip, bits)
    assert clear.mean() > 0.98
    assert np.array_equal(code[clear], np.clip(np.floor(v + 0.5), 0, top).astype(np.uint8)[clear])


def _conv64(levels, w, stride, pad):
    a = torch.from_numpy(levels.astype(np.float64)).permute(0, 3, 1, 2)
    k = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)
    return torch.nn.functional.conv2d(a, k, stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()


def test_residual_trunk_block_by_block_against_float64_library_ops():
    plan = ((16, 16, 1), (16, 32, 2), (32, 32, 1))
    net = wl.resnet18_trunk(batch=2, hw=12, bits=3, plan=plan)
    trace = oracle.residual_trunk(net["x"], net["blocks"])
    assert len(trace) == 3
    x = net["x"]
    for blk, t in zip(net["blocks"], trace):
        c1, c2, dn = blk["conv1"], blk["conv2"], blk["down"]
        a, _ = oracle.quantize(x, c1["clip"], c1["a_bits"])
        assert np.array_equal(t["a"], a)
        z1 = _conv64(a, c1["w"], c1["stride"], 1)
        assert np.array_equal(t["acc1"], z1.astype(np.int64))
        h = z1 * c1["scale"].astype(np.float64) + c1["bias"]
        hq, _ = oracle.quantize(h.astype(np.float32), c2["clip"], c2["a_bits"])
        # fp32 rounding may move a value across a threshold: allow a few in ten thousand
        assert (t["hq"] != hq).mean() < 5e-4
        z2 = _conv64(t["hq"], c2["w"], 1, 1)
        assert np.array_equal(t["acc2"], z2.astype(np.int64))
        y = z2 * c2["scale"].astype(np.float64) + c2["bias"]
        if dn is None:
            assert t["accd"] is None and a.shape == y.shape
            y = y + a * np.float64(np.float32(blk["res_scale"]))
        else:
            zd = _conv64(a, dn["w"], dn["stride"], 0)
            assert zd.shape == y.shape and np.array_equal(t["accd"], zd.astype(np.int64))
            y = y + (zd * dn["scale"].astype(np.float64) + dn["bias"])
        np.testing.assert_allclose(t["y"], y, rtol=0, atol=1e-5)
        x = t["y"]
    # the shapes of the three blocks: identity, strided with a 1x1 shortcut, identity
    assert [t["y"].shape for t in trace] == [(2, 12, 12, 16), (2, 6, 6, 32), (2, 6, 6, 32)]
    assert [t["accd"] is None for t in trace] == [True, False, True]


def test_trunk_activations_stay_in_range():
    # the workload's gains keep every quantizer busy: all levels occur, little saturation, block after block
    net = wl.resnet18_trunk(batch=1, hw=16, bits=3, plan=((32, 32, 1),) * 4)
    for t in oracle.residual_trunk(net["x"], net["blocks"]):
        for lv in (t["a"], t["hq"]):
            assert len(np.unique(lv)) == 8
            assert (np.abs(lv) == 7).mean() < 0.1


def test_relu_term_is_hrelu_in_front_of_the_quantizer():
    # Table 1: HReLU(x) = 1 for x > 1, x in between, 0 for x < 0.  With the relu term the next quantizer
    # (clamp of y / clip to [-1, 1]) sees exactly HReLU(y / clip): only the codes of the upper half occur,
    # and with 1 bit every activation is +1 -- the special case the experiments section notes.
    gen = np.random.default_rng(21)
    acc = gen.integers(-400, 400, size=(2, 5, 5, 8)).astype(np.int32)
    s = gen.uniform(0.005, 0.02, size=8).astype(np.float32)
    bias = gen.normal(0, 0.2, size=8).astype(np.float32)
    plain = oracle.block_epilogue(acc, s, bias)
    y = oracle.block_epilogue(acc, s, bias, relu=True)
    assert np.array_equal(y, np.where(plain > 0, plain, np.float32(0))) and (plain < 0).any()
    clip = 2.0
    hrelu = np.minimum(np.maximum(y.astype(np.float64) / clip, 0.0), 1.0)
    for bits in (1, 2, 3):
        lv, _ = oracle.quantize(y, clip, bits)
        top = (1 << bits) - 1
        # the quantizer's own range limit gives the same value as HReLU on these inputs
        lv_ref, _ = oracle.quantize((hrelu * clip).astype(np.float32), clip, bits)
        assert np.array_equal(lv, lv_ref)
        assert lv.min() >= 1 and lv.max() == top          # levels of the upper half only
        if bits == 1:
            assert (lv == 1).all()
