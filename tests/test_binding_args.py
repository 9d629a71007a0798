"""Host-only checks of the Python binding: every wrapper refuses a tensor it cannot hand to the C ABI as a bare
pointer -- wrong dtype, not contiguous, wrong shape or element count, not in device memory -- before taking its
address (the C side cannot see any of that, and an undersized output buffer would be a device write out of
bounds).  No GPU and no launch: with host tensors the last check (device memory) is the one that fires when
everything else is right."""
import pytest
import torch

from paper_1905_13389_amd import qnn

I32, F32, I8, U8 = torch.int32, torch.float32, torch.int8, torch.uint8


def z(shape, dtype):
    return torch.zeros(shape, dtype=dtype)


def sliced(shape, dtype):
    """A non-contiguous view of the wanted shape (every second column of a wider tensor)."""
    wide = torch.zeros(tuple(shape[:-1]) + (2 * shape[-1],), dtype=dtype)
    return wide[..., ::2]


# every case: a callable taking a dict of tensor overrides; `good` names the tensors of a well-formed call
def gemm(t):
    return qnn.qnn_binary_gemm(t["a"], t["w"], 64, scale=t["scale"], acc=t["acc"], out=t["out"])


def conv(t):
    return qnn.qnn_conv2d(t["a"], t["w"], (2, 5, 5), 64, 1, 1, scale=t["scale"], want_out=True, next_clip=1.0,
                          next_bits=2, acc=t["acc"], out=t["out"], next_planes=t["next"])


def conv_block(t):
    return qnn.qnn_conv2d_block(t["a"], t["w"], (2, 5, 5), 64, 1, 1, t["scale"], bias=t["bias"], res_planes=t["res"],
                                res_scale=0.5, res_f32=t["res_f32"], want_out=True, acc=t["acc"], out=t["out"])


def level_conv(t):
    return qnn.qnn_level_conv2d_i8(t["a"], t["w"], 1, 1, 2, 2, scale=t["scale"], want_out=True, next_clip=1.0,
                                   next_bits=2, acc=t["acc"], out=t["out"], next_levels=t["next"])


def level_conv_fp4(t):
    return qnn.qnn_level_conv2d_block_fp4(t["a"], t["w"], 1, 1, 2, 2, t["scale"], bias=t["bias"], res_levels=t["res"],
                                          res_bits=2, res_scale=0.5, want_out=True, next_clip=1.0, next_bits=2,
                                          acc=t["acc"], out=t["out"], next_levels=t["next"])


def deconv(t):
    return qnn.qnn_deconv2d(t["a"], t["phase"], (1, 4, 4), 64, 32, 4, 4, 2, 1, 2, scale=t["scale"], bias=t["bias"],
                            want_out=True, acc=t["acc"], out=t["out"])


CASES = {
    "encode_pack": (lambda t: qnn.qnn_encode_pack(t["src"], 1.0, 2, planes=t["planes"]),
                    {"src": ((3, 64), F32), "planes": ((2, 3, 2), I32)}),
    "fc_fused": (lambda t: qnn.qnn_fc_fused(t["src"], 1.0, 2, t["w"], scale=t["scale"], acc=t["acc"], out=t["out"]),
                 {"src": ((3, 64), F32), "w": ((2, 8, 2), I32), "scale": ((8,), F32), "acc": ((3, 8), I32),
                  "out": ((3, 8), F32)}),
    "binary_gemm": (gemm, {"a": ((2, 3, 2), I32), "w": ((2, 8, 2), I32), "scale": ((8,), F32), "acc": ((3, 8), I32),
                           "out": ((3, 8), F32)}),
    "dequant_scale": (lambda t: qnn.qnn_dequant_scale(t["acc"], t["scale"], out=t["out"]),
                      {"acc": ((3, 8), I32), "scale": ((8,), F32), "out": ((3, 8), F32)}),
    "conv2d": (conv, {"a": ((2, 50, 2), I32), "w": ((2, 32, 3, 3, 2), I32), "scale": ((32,), F32),
                      "acc": ((2, 5, 5, 32), I32), "out": ((2, 5, 5, 32), F32), "next": ((2, 50, 1), I32)}),
    "conv2d_block": (conv_block, {"a": ((2, 50, 2), I32), "w": ((2, 32, 3, 3, 2), I32), "scale": ((32,), F32),
                                  "bias": ((32,), F32), "res": ((2, 50, 1), I32), "res_f32": ((2, 5, 5, 32), F32),
                                  "acc": ((2, 5, 5, 32), I32), "out": ((2, 5, 5, 32), F32)}),
    "level_conv2d_i8": (level_conv, {"a": ((2, 5, 5, 16), I8), "w": ((32, 3, 3, 16), I8), "scale": ((32,), F32),
                                     "acc": ((2, 5, 5, 32), I32), "out": ((2, 5, 5, 32), F32),
                                     "next": ((2, 5, 5, 32), I8)}),
    "level_conv2d_block_fp4": (level_conv_fp4, {"a": ((2, 5, 5, 16), U8), "w": ((32, 3, 3, 16), U8),
                                                "scale": ((32,), F32), "bias": ((32,), F32),
                                                "res": ((2, 5, 5, 16), U8), "acc": ((2, 5, 5, 32), I32),
                                                "out": ((2, 5, 5, 32), F32), "next": ((2, 5, 5, 16), U8)}),
    "deconv2d": (deconv, {"a": ((2, 16, 2), I32), "phase": ((2 * 32 * 16 * 2,), I32), "scale": ((32,), F32),
                          "bias": ((32,), F32), "acc": ((1, 8, 8, 32), I32), "out": ((1, 8, 8, 32), F32)}),
    "deconv_pack_weights": (lambda t: qnn.qnn_deconv_pack_weights(t["w"], 64, 2, phase_planes=t["phase"]),
                            {"w": ((2, 32, 4, 4, 2), I32), "phase": ((2 * 32 * 16 * 2,), I32)}),
    "maxpool_planes": (lambda t: qnn.qnn_maxpool_planes(t["p"], (2, 6, 6), 64, 2, 2, out=t["out"]),
                       {"p": ((3, 72, 2), I32), "out": ((3, 18, 2), I32)}),
    "maxpool_levels_i8": (lambda t: qnn.qnn_maxpool_levels_i8(t["l"], 2, 2, out=t["out"]),
                          {"l": ((2, 6, 6, 16), I8), "out": ((2, 3, 3, 16), I8)}),
    "maxpool_levels_fp4": (lambda t: qnn.qnn_maxpool_levels_fp4(t["l"], 2, 2, out=t["out"]),
                           {"l": ((2, 6, 6, 8), U8), "out": ((2, 3, 3, 8), U8)}),
    "plane_sum_i8": (lambda t: qnn.qnn_plane_sum_i8(t["p"], 64, levels=t["lv"]),
                     {"p": ((2, 3, 2), I32), "lv": ((3, 128), I8)}),
    "level_gemm_i8": (lambda t: qnn.qnn_level_gemm_i8(t["a"], t["w"], 64, scale=t["scale"], acc=t["acc"], out=t["out"]),
                      {"a": ((3, 128), I8), "w": ((8, 128), I8), "scale": ((8,), F32), "acc": ((3, 8), I32),
                       "out": ((3, 8), F32)}),
    "plane_sum_fp4": (lambda t: qnn.qnn_plane_sum_fp4(t["p"], 64, levels=t["lv"]),
                      {"p": ((2, 3, 2), I32), "lv": ((3, 128), U8)}),
    "level_gemm_fp4": (lambda t: qnn.qnn_level_gemm_fp4(t["a"], t["w"], 64, scale=t["scale"], acc=t["acc"], out=t["out"]),
                       {"a": ((3, 128), U8), "w": ((8, 128), U8), "scale": ((8,), F32), "acc": ((3, 8), I32),
                        "out": ((3, 8), F32)}),
    "encode_levels_i8": (lambda t: qnn.qnn_encode_levels_i8(t["src"], 1.0, 2, levels=t["lv"]),
                         {"src": ((3, 64), F32), "lv": ((3, 64), I8)}),
    "encode_levels_fp4": (lambda t: qnn.qnn_encode_levels_fp4(t["src"], 1.0, 2, levels=t["lv"]),
                          {"src": ((3, 64), F32), "lv": ((3, 32), U8)}),
    "levels_to_fp4": (lambda t: qnn.qnn_levels_to_fp4(t["lv"], out=t["out"]), {"lv": ((3, 64), I8), "out": ((3, 32), U8)}),
    "quantize_ste_backward": (lambda t: qnn.qnn_quantize_ste_backward(t["x"], t["g"], 1.0, grad_x=t["gx"]),
                              {"x": ((3, 64), F32), "g": ((3, 64), F32), "gx": ((3, 64), F32)}),
    "encoder_backward": (lambda t: qnn.qnn_encoder_backward(t["x"], t["g"], 1.0, grad_x=t["gx"]),
                         {"x": ((3, 64), F32), "g": ((2, 3, 64), F32), "gx": ((3, 64), F32)}),
    "dense_conv2d_f32": (lambda t: qnn.qnn_dense_conv2d_f32(t["x"], t["w"], 1, 1, scale=t["scale"], shift=t["shift"],
                                                            next_clip=1.0, next_bits=2, out=t["out"], next_planes=t["next"]),
                         {"x": ((2, 5, 5, 3), F32), "w": ((32, 3, 3, 3), F32), "scale": ((32,), F32), "shift": ((32,), F32),
                          "out": ((2, 5, 5, 32), F32), "next": ((2, 50, 1), I32)}),
    "dense_conv2d_f32_levels": (lambda t: qnn.qnn_dense_conv2d_f32_levels(t["x"], t["w"], 1, 1, 1.0, 2, scale=t["scale"],
                                                                          next_levels=t["next"]),
                                {"x": ((2, 5, 5, 3), F32), "w": ((32, 3, 3, 3), F32), "scale": ((32,), F32),
                                 "next": ((2, 5, 5, 32), I8)}),
    "global_avgpool_f32": (lambda t: qnn.qnn_global_avgpool_f32(t["x"], out=t["out"]),
                           {"x": ((2, 3, 3, 8), F32), "out": ((2, 8), F32)}),
    "dense_fc_f32": (lambda t: qnn.qnn_dense_fc_f32(t["x"], t["w"], t["b"], out=t["out"]),
                     {"x": ((3, 16), F32), "w": ((8, 16), F32), "b": ((8,), F32), "out": ((3, 8), F32)}),
}


def _good(spec):
    return {k: z(shape, dtype) for k, (shape, dtype) in spec.items()}


@pytest.mark.parametrize("name", sorted(CASES))
def test_well_formed_host_tensors_are_refused_as_not_device_memory(name):
    call, spec = CASES[name]
    with pytest.raises(ValueError, match="not a CUDA"):
        call(_good(spec))


@pytest.mark.parametrize("name", sorted(CASES))
def test_every_tensor_argument_is_checked(name):
    call, spec = CASES[name]
    for key, (shape, dtype) in spec.items():
        wrong_dtype = torch.float64 if dtype != torch.float64 else torch.float32
        bad = [("dtype", z(shape, wrong_dtype)), ("size", z(tuple(shape[:-1]) + (shape[-1] + 1,), dtype))]
        if not (name in ("encode_pack", "fc_fused") and key == "src"):   # their src may be a strided 2-D view
            bad.append(("strides", sliced(shape, dtype)))
        if name == "deconv_pack_weights" and key == "phase" or name == "deconv2d" and key == "phase":
            bad[1] = ("size", z((shape[0] - 1,), dtype))                 # a larger phase buffer is allowed
        for what, tensor in bad:
            args = _good(spec)
            args[key] = tensor
            with pytest.raises((ValueError, TypeError)) as e:
                call(args)
            assert "not a CUDA" not in str(e.value), "%s: a wrong %s of %r went unnoticed" % (name, what, key)


def test_encoder_inputs_may_be_rows_a_stride_apart_but_nothing_else():
    wide = torch.zeros((4, 96), dtype=F32)
    with pytest.raises(ValueError, match="not a CUDA"):
        qnn.qnn_encode_pack(wide[:, :64], 1.0, 2)              # rows 96 apart: accepted up to the device check
    with pytest.raises(ValueError, match="neither contiguous"):
        qnn.qnn_encode_pack(wide[:, ::2], 1.0, 2)              # elements of a row not adjacent
    with pytest.raises(ValueError, match="neither contiguous"):
        qnn.qnn_encode_pack(torch.zeros((2, 4, 96))[:, :, :64], 1.0, 2)   # strided views are 2-D only
    with pytest.raises(ValueError, match="2-D"):
        qnn.qnn_fc_fused(torch.zeros((2, 4, 64)), 1.0, 2, torch.zeros((2, 8, 2), dtype=I32))


def test_the_library_in_use_is_the_in_tree_build():
    import os
    here = os.path.dirname(os.path.abspath(qnn.__file__))
    assert qnn.LIB_PATH == os.path.join(here, "libqnn.so")
    qnn.lib()
    from paper_1905_13389_amd import build
    assert qnn.lib().qnn_build_id().decode() == build.source_id()
