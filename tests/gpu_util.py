"""Helpers for the GPU parity tests: numpy <-> device tensors and level packing through the
library's own qnn_encode_pack (int8 level path)."""
import functools

import numpy as np
import torch

import oracle
import qnn_workloads as wl

from paper_1905_13389_amd import qnn


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def planes_to_numpy(p):
    torch.cuda.synchronize()
    return p.cpu().numpy().view(np.uint32)


def pack_levels(levels_np, bits):
    """int8 levels [..., n] -> device planes via qnn_encode_pack(dtype = int8 levels)."""
    return qnn.qnn_encode_pack(dev(levels_np.astype(np.int8)), 1.0, bits)


def levels(gen, shape, bits):
    top = (1 << bits) - 1
    return (2 * gen.integers(0, top + 1, size=shape) - top).astype(np.int8)


@functools.lru_cache(maxsize=None)
def oracle_full_batch(config):
    """The oracle's chain over the whole batch of configuration 4 ('stack4') or 5 ('stack5'), computed once
    per test session: per resolution group, the int8 levels entering every layer and the last layer's fp32
    output.  (The workload generators are seeded, so the tests rebuild the same inputs themselves.)"""
    groups = [wl.resnet18_stack()] if config == "stack4" else wl.vgg_ssd_stack()
    res = []
    for g in groups:
        trace = oracle.conv_stack(g["x"], g["layers"])
        res.append(([t["levels"].astype(np.int8) for t in trace], trace[-1]["out"]))
        del trace
    return res


def codes_explained_by_bound(got32, want64, bound, clip, bits):
    """Number of elements whose code from the fp32 value differs from the code of the float64 value; asserts that
    each of them has its float64 value within `bound` (plus the quantizer's own fp32 roundings) of a threshold."""
    top = (1 << bits) - 1
    lv_got, _ = oracle.quantize(got32, clip, bits)
    lv_ref, _ = oracle.quantize(want64.astype(np.float32), clip, bits)
    differ = lv_got != lv_ref
    if differ.any():
        thresholds = (2.0 * (np.arange(top) + 0.5) / top - 1.0) * clip
        dist = np.abs(want64[differ][:, None] - thresholds[None, :]).min(axis=1)
        slack = bound[differ] + 8 * 2.0 ** -24 * (np.abs(want64[differ]) + clip)
        assert (dist <= slack).all(), "a code differs although the value is not near a threshold"
        assert (np.abs(lv_got.astype(np.int32) - lv_ref)[differ] == 2).all(), "codes differ by more than one step"
    return int(differ.sum())
