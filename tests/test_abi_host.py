"""Host-only checks of the C ABI: the library loads, exports every symbol include/qnn.h declares,
and rejects bad arguments before any HIP call (no GPU needed, no compute launched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def qnn():
    from paper_1905_13389_amd import qnn as q
    q.lib()
    return q


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "qnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qnn_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(qnn):
    names = _declared_functions()
    assert set(names) == set(qnn.EXPORTS)
    L = ctypes.CDLL(qnn.LIB_PATH)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_empty_error(qnn):
    assert qnn.qnn_version() >= 100
    assert isinstance(qnn.lib().qnn_last_error(), bytes)


def test_conv_desc_layout_matches_header(qnn):
    # 5 int64 then 6 int32 -> 64 bytes, no padding surprises
    assert ctypes.sizeof(qnn.qnn_conv_desc) == 5 * 8 + 6 * 4


FAKE = ctypes.c_void_p(0x1000)      # 16-byte aligned, never dereferenced: all of these fail earlier
ODD = ctypes.c_void_p(0x1004)


def test_encode_pack_argument_errors(qnn):
    L = qnn.lib()
    assert L.qnn_encode_pack(FAKE, 7, 4, 64, 64, 1.0, 2, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED
    assert L.qnn_encode_pack(FAKE, 0, 4, 64, 64, 1.0, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_pack(FAKE, 0, 4, 64, 64, 1.0, 9, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_pack(FAKE, 0, -1, 64, 64, 1.0, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_pack(FAKE, 0, 4, 64, 32, 1.0, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_pack(FAKE, 0, 4, 64, 64, 0.0, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_pack(FAKE, 0, 4, 64, 64, float("nan"), 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_pack(FAKE, 0, 4, 64, 64, float("inf"), 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_pack(None, 0, 4, 64, 64, 1.0, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_pack(FAKE, 0, 4, 64, 64, 1.0, 2, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert L.qnn_encode_pack(FAKE, 2, 4, 64, 64, 1.0, 8, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED
    assert b"int8" in L.qnn_last_error()
    # empty input is a successful no-op
    assert L.qnn_encode_pack(None, 0, 0, 64, 64, 1.0, 2, None, None) == qnn.QNN_OK
    assert L.qnn_encode_pack(None, 0, 4, 0, 0, 1.0, 2, None, None) == qnn.QNN_OK


def test_binary_gemm_argument_errors(qnn):
    L = qnn.lib()
    g = L.qnn_binary_gemm
    assert g(FAKE, 0, FAKE, 2, 4, 4, 64, FAKE, None, None, None) == qnn.QNN_ERR_INVALID_ARG
    assert g(FAKE, 2, FAKE, 9, 4, 4, 64, FAKE, None, None, None) == qnn.QNN_ERR_INVALID_ARG
    assert g(FAKE, 2, FAKE, 2, -4, 4, 64, FAKE, None, None, None) == qnn.QNN_ERR_INVALID_ARG
    assert g(FAKE, 2, FAKE, 2, 4, 4, 64, None, None, None, None) == qnn.QNN_ERR_INVALID_ARG
    assert g(FAKE, 2, FAKE, 2, 4, 4, 64, None, None, FAKE, None) == qnn.QNN_ERR_INVALID_ARG  # out, no scale
    assert g(None, 2, FAKE, 2, 4, 4, 64, FAKE, None, None, None) == qnn.QNN_ERR_INVALID_ARG
    assert g(ODD, 2, FAKE, 2, 4, 4, 64, FAKE, None, None, None) == qnn.QNN_ERR_ALIGNMENT
    assert g(FAKE, 2, FAKE, 2, 4, 4, 64, ODD, None, None, None) == qnn.QNN_ERR_ALIGNMENT
    # 8x8 bits: n * 255 * 255 must stay below 2^31 -> n <= 33025
    assert g(FAKE, 8, FAKE, 8, 4, 4, 33026, FAKE, None, None, None) == qnn.QNN_ERR_RANGE
    assert b"overflows int32" in L.qnn_last_error()
    assert g(None, 2, None, 2, 0, 4, 64, FAKE, None, None, None) == qnn.QNN_OK


def test_dequant_scale_argument_errors(qnn):
    L = qnn.lib()
    f = L.qnn_dequant_scale
    assert f(None, FAKE, 4, 4, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert f(FAKE, FAKE, -1, 4, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert f(FAKE, FAKE, 4, 4, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert f(None, None, 0, 4, None, None) == qnn.QNN_OK


def test_conv2d_argument_errors(qnn):
    L = qnn.lib()

    def call(desc, a=FAKE, w=FAKE, scale=None, acc=FAKE, out=None, nxt=None, clip=0.0, nbits=0):
        return L.qnn_conv2d(ctypes.byref(desc) if desc is not None else None, a, w, scale, acc, out, nxt,
                            clip, nbits, None)

    D = qnn.qnn_conv_desc
    ok = D(1, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)
    assert call(None) == qnn.QNN_ERR_INVALID_ARG
    assert call(D(1, 8, 8, 64, 64, 3, 3, 1, 1, 0, 2)) == qnn.QNN_ERR_INVALID_ARG
    assert call(D(1, 0, 8, 64, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_ERR_INVALID_ARG
    assert call(D(1, 8, 8, 64, 64, 3, 3, 0, 1, 2, 2)) == qnn.QNN_ERR_INVALID_ARG
    assert call(D(1, 8, 8, 64, 64, 9, 9, 1, 1, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED
    assert call(D(1, 2, 2, 64, 64, 5, 5, 1, 0, 2, 2)) == qnn.QNN_ERR_INVALID_ARG  # kernel > image
    assert call(ok, acc=None) == qnn.QNN_ERR_INVALID_ARG                          # no output
    assert call(ok, acc=None, out=FAKE) == qnn.QNN_ERR_INVALID_ARG                # out without scale
    assert call(ok, scale=FAKE, nxt=FAKE, clip=1.0, nbits=0) == qnn.QNN_ERR_INVALID_ARG
    assert call(ok, scale=FAKE, nxt=FAKE, clip=-1.0, nbits=2) == qnn.QNN_ERR_INVALID_ARG
    assert call(ok, a=None) == qnn.QNN_ERR_INVALID_ARG
    assert call(ok, w=ODD) == qnn.QNN_ERR_ALIGNMENT
    # 8x8 bits with 3x3x4096 channels overflows int32
    assert call(D(1, 8, 8, 4096, 64, 3, 3, 1, 1, 8, 8)) == qnn.QNN_ERR_RANGE
    # above 4 bits the fused epilogue needs an acc or out buffer for the running sum of the plane chunks
    assert call(D(1, 8, 8, 64, 64, 3, 3, 1, 1, 5, 5), scale=FAKE, acc=None, nxt=FAKE, clip=1.0, nbits=2) \
        == qnn.QNN_ERR_UNSUPPORTED
    assert call(D(0, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_OK


def test_block_epilogue_argument_errors(qnn):
    L = qnn.lib()
    D, E = qnn.qnn_conv_desc, qnn.qnn_block_epilogue
    # pointer, pointer, int32, float, pointer, int32 (+ tail padding)
    assert ctypes.sizeof(E) == 40 and E.res_bits.offset == 16 and E.res_scale.offset == 20 and E.res_f32.offset == 24
    assert E.relu.offset == 32
    ok = D(1, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)
    F, O = FAKE.value, ODD.value

    def call(entry, epi, scale=FAKE, desc=ok):
        return entry(ctypes.byref(desc), FAKE, FAKE, scale, ctypes.byref(epi) if epi is not None else None,
                     FAKE, None, None, 0.0, 0, None)

    for entry, max_bits in ((L.qnn_conv2d_block, 8), (L.qnn_level_conv2d_block_i8, 7)):
        assert call(entry, E(F, None, 0, 0.0, None), scale=None) == qnn.QNN_ERR_INVALID_ARG   # terms without scale
        assert call(entry, E(None, F, 0, 1.0, None)) == qnn.QNN_ERR_INVALID_ARG               # res_bits too small
        assert call(entry, E(None, F, max_bits + 1, 1.0, None)) == qnn.QNN_ERR_INVALID_ARG
        assert call(entry, E(None, F, 2, float("nan"), None)) == qnn.QNN_ERR_INVALID_ARG
        assert call(entry, E(None, F, 2, float("inf"), None)) == qnn.QNN_ERR_INVALID_ARG
        assert b"res_scale" in L.qnn_last_error()
        assert call(entry, E(O, None, 0, 0.0, None)) == qnn.QNN_ERR_ALIGNMENT
        assert call(entry, E(None, O, 2, 1.0, None)) == qnn.QNN_ERR_ALIGNMENT
        assert call(entry, E(None, None, 0, 0.0, O)) == qnn.QNN_ERR_ALIGNMENT
        # a valid epilogue does not mask the convolution's own checks; an empty batch returns before any launch
        assert call(entry, E(F, F, 2, 1.0, F), desc=D(1, 8, 8, 64, 64, 3, 3, 0, 1, 2, 2)) == qnn.QNN_ERR_INVALID_ARG
        assert call(entry, E(F, F, 2, 1.0, F), desc=D(0, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_OK
        assert call(entry, None, desc=D(0, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_OK


def test_deconv_argument_errors_and_phase_words(qnn):
    L = qnn.lib()
    D = qnn.qnn_conv_desc
    # 4x4 kernel, stride 2, 64 -> 32 channels, 2 bits: 4 phases of 2x2 taps, 2*32*4*2 words each
    assert L.qnn_deconv_phase_words(2, 32, 4, 4, 64, 2) == 4 * 2 * 32 * 4 * 2
    # 3x3 kernel, stride 2, one word per tap: phases of 4, 2, 2, 1 taps; 3 channels -> 3, 6, 6, 12 words, each rounded up to 4
    assert L.qnn_deconv_phase_words(1, 3, 3, 3, 5, 2) == 12 + 8 + 8 + 4
    assert L.qnn_deconv_phase_words(0, 3, 3, 3, 5, 2) == -1
    assert L.qnn_deconv_phase_words(1, 3, 3, 3, 5, 0) == -1
    assert L.qnn_deconv_pack_weights(FAKE, 9, 8, 3, 3, 32, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_deconv_pack_weights(FAKE, 2, 8, 3, 3, 32, 2, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert L.qnn_deconv_pack_weights(None, 2, 8, 3, 3, 32, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_deconv_pack_weights(FAKE, 2, 8, 17, 3, 32, 2, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED

    def call(desc, a=FAKE, w=FAKE, scale=None, bias=None, acc=FAKE, out=None, nxt=None, clip=0.0, nbits=0):
        return L.qnn_deconv2d(ctypes.byref(desc) if desc is not None else None, a, w, scale, bias, acc, out, nxt,
                              clip, nbits, None)

    ok = D(1, 8, 8, 64, 32, 4, 4, 2, 1, 2, 2)
    assert call(None) == qnn.QNN_ERR_INVALID_ARG
    assert call(D(1, 8, 8, 64, 32, 4, 4, 2, 1, 0, 2)) == qnn.QNN_ERR_INVALID_ARG
    # above 4 bits the plane chunks need acc or out for their running sum
    assert call(D(1, 8, 8, 64, 32, 4, 4, 2, 1, 5, 2), scale=FAKE, acc=None, nxt=FAKE, clip=1.0, nbits=2) == qnn.QNN_ERR_UNSUPPORTED
    assert call(D(1, 8, 8, 64, 32, 1, 1, 2, 0, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED       # kernel below stride
    assert call(D(1, 1, 1, 64, 32, 2, 2, 2, 1, 2, 2)) == qnn.QNN_ERR_INVALID_ARG       # pad eats the whole output
    assert call(ok, acc=None) == qnn.QNN_ERR_INVALID_ARG
    assert call(ok, out=FAKE) == qnn.QNN_ERR_INVALID_ARG                               # out without scale
    assert call(ok, bias=FAKE) == qnn.QNN_ERR_INVALID_ARG                              # bias without scale
    assert call(ok, scale=FAKE, nxt=FAKE, clip=1.0, nbits=9) == qnn.QNN_ERR_INVALID_ARG
    assert call(ok, a=None) == qnn.QNN_ERR_INVALID_ARG
    assert call(ok, w=ODD) == qnn.QNN_ERR_ALIGNMENT
    assert call(ok, scale=FAKE, bias=ODD) == qnn.QNN_ERR_ALIGNMENT
    assert call(D(0, 8, 8, 64, 32, 4, 4, 2, 1, 2, 2)) == qnn.QNN_OK


def test_dilated_convolution_argument_errors(qnn):
    L = qnn.lib()
    D = qnn.qnn_conv_desc
    ok = D(1, 19, 19, 64, 64, 3, 3, 1, 6, 2, 2)
    for entry in (L.qnn_conv2d_dilated, L.qnn_level_conv2d_dilated_i8, L.qnn_level_conv2d_dilated_fp4):
        def call(desc, dil, a=FAKE, w=FAKE, scale=None, acc=FAKE, out=None, nxt=None, clip=0.0, nbits=0):
            return entry(ctypes.byref(desc) if desc is not None else None, dil, a, w, scale, acc, out, nxt, clip, nbits, None)
        assert call(None, 1) == qnn.QNN_ERR_INVALID_ARG
        assert call(ok, 0) == qnn.QNN_ERR_INVALID_ARG
        assert call(ok, -3) == qnn.QNN_ERR_INVALID_ARG
        assert call(ok, 65) == qnn.QNN_ERR_UNSUPPORTED
        assert call(ok, 16) == qnn.QNN_ERR_INVALID_ARG               # taps 32 pixels apart do not fit 19 + 2 * 6
        assert call(D(1, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2), 2, acc=None) == qnn.QNN_ERR_INVALID_ARG
        assert call(ok, 6, out=FAKE) == qnn.QNN_ERR_INVALID_ARG      # out without scale
        assert call(ok, 6, w=ODD) == qnn.QNN_ERR_ALIGNMENT
        assert call(ok, 6, a=None) == qnn.QNN_ERR_INVALID_ARG
        assert call(D(0, 19, 19, 64, 64, 3, 3, 1, 6, 2, 2), 6) == qnn.QNN_OK


def test_level_deconv_argument_errors_and_workspace(qnn):
    L = qnn.lib()
    D = qnn.qnn_conv_desc
    ok = D(2, 8, 8, 64, 32, 4, 4, 2, 1, 2, 2)
    # widened tensor: 2 x 15 x 15 pixels of 64 (int8) or 32 (fp4) bytes
    assert L.qnn_level_deconv_workspace_bytes(ctypes.byref(ok), 0) == 2 * 15 * 15 * 64
    assert L.qnn_level_deconv_workspace_bytes(ctypes.byref(ok), 1) == 2 * 15 * 15 * 32
    assert L.qnn_level_deconv_workspace_bytes(ctypes.byref(D(2, 8, 8, 64, 32, 4, 3, 2, 1, 2, 2)), 0) == -1   # not square
    assert L.qnn_level_deconv_workspace_bytes(ctypes.byref(D(2, 8, 8, 24, 32, 4, 4, 2, 1, 2, 2)), 0) == -1   # Cin % 16
    assert L.qnn_level_deconv_workspace_bytes(None, 0) == -1
    assert L.qnn_level_deconv_flip_weights(None, 32, 4, 4, 64, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_level_deconv_flip_weights(FAKE, 32, 4, 4, 24, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED
    assert L.qnn_level_deconv_flip_weights(FAKE, 32, 4, 4, 64, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert L.qnn_level_deconv_flip_weights(FAKE, 0, 4, 4, 64, FAKE, None) == qnn.QNN_ERR_INVALID_ARG

    for entry in (L.qnn_level_deconv2d_i8, L.qnn_level_deconv2d_fp4):
        def call(desc, a=FAKE, w=FAKE, ws=FAKE, scale=None, bias=None, acc=FAKE, out=None, nxt=None, clip=0.0, nbits=0):
            return entry(ctypes.byref(desc) if desc is not None else None, a, w, ws, scale, bias, acc, out, nxt, clip,
                         nbits, None)
        assert call(None) == qnn.QNN_ERR_INVALID_ARG
        assert call(D(1, 8, 8, 64, 32, 4, 4, 2, 4, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED      # pad > k - 1
        assert call(D(1, 8, 8, 64, 32, 4, 2, 2, 1, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED      # not square
        assert call(D(1, 8, 8, 64, 32, 4, 4, 0, 1, 2, 2)) == qnn.QNN_ERR_INVALID_ARG
        assert call(D(1, 1, 1, 64, 32, 2, 2, 2, 1, 2, 2)) == qnn.QNN_ERR_INVALID_ARG      # pad eats the whole output
        assert call(D(1, 8, 8, 64, 32, 4, 4, 2, 1, 0, 2)) == qnn.QNN_ERR_INVALID_ARG
        assert call(ok, acc=None) == qnn.QNN_ERR_INVALID_ARG
        assert call(ok, out=FAKE) == qnn.QNN_ERR_INVALID_ARG                              # out without scale
        assert call(ok, bias=FAKE) == qnn.QNN_ERR_INVALID_ARG                             # bias without scale
        assert call(ok, ws=None) == qnn.QNN_ERR_INVALID_ARG
        assert call(ok, ws=ODD) == qnn.QNN_ERR_ALIGNMENT
        assert call(ok, w=ODD) == qnn.QNN_ERR_ALIGNMENT
        assert call(ok, a=ODD) == qnn.QNN_ERR_ALIGNMENT
        assert call(ok, scale=FAKE, nxt=FAKE, clip=1.0, nbits=9) == qnn.QNN_ERR_INVALID_ARG
        assert call(D(0, 8, 8, 64, 32, 4, 4, 2, 1, 2, 2)) == qnn.QNN_OK
    assert L.qnn_level_deconv2d_fp4(ctypes.byref(D(1, 8, 8, 64, 32, 4, 4, 2, 1, 3, 2)), FAKE, FAKE, FAKE, None, None, FAKE,
                                    None, None, 0.0, 0, None) == qnn.QNN_ERR_UNSUPPORTED
    assert L.qnn_level_deconv2d_fp4(ctypes.byref(D(1, 8, 8, 48, 32, 4, 4, 2, 1, 2, 2)), FAKE, FAKE, FAKE, None, None, FAKE,
                                    None, None, 0.0, 0, None) == qnn.QNN_ERR_UNSUPPORTED


def test_fp4_convolution_argument_errors(qnn):
    L = qnn.lib()
    D = qnn.qnn_conv_desc

    def call(desc, a=FAKE, w=FAKE, scale=None, acc=FAKE, out=None, nxt=None, clip=0.0, nbits=0):
        return L.qnn_level_conv2d_fp4(ctypes.byref(desc), a, w, scale, acc, out, nxt, clip, nbits, None)

    assert call(D(1, 8, 8, 64, 64, 3, 3, 1, 1, 3, 2)) == qnn.QNN_ERR_UNSUPPORTED        # 3-bit codes are not fp4 values
    assert call(D(1, 8, 8, 64, 64, 3, 3, 1, 1, 9, 2)) == qnn.QNN_ERR_INVALID_ARG
    assert call(D(1, 8, 8, 48, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED        # Cin not a multiple of 32
    assert call(D(1, 8, 8, 64, 63, 3, 3, 1, 1, 2, 2), scale=FAKE, nxt=FAKE, clip=1.0, nbits=2) == qnn.QNN_ERR_UNSUPPORTED
    assert call(D(1, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2), scale=FAKE, nxt=FAKE, clip=1.0, nbits=3) == qnn.QNN_ERR_INVALID_ARG
    # 9 * 5 * 5 * 80000 >= 2^24: beyond exact fp32 accumulation (but fine for int32)
    assert call(D(1, 8, 8, 80000, 64, 5, 5, 1, 2, 2, 2)) in (qnn.QNN_ERR_RANGE, qnn.QNN_ERR_UNSUPPORTED)
    assert call(D(1, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2), w=ODD) == qnn.QNN_ERR_ALIGNMENT
    assert call(D(0, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_OK
    E = qnn.qnn_block_epilogue
    okd = D(1, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)
    blk = lambda e, d=okd: L.qnn_level_conv2d_block_fp4(ctypes.byref(d), FAKE, FAKE, FAKE, ctypes.byref(e), FAKE, None, None,
                                                         0.0, 0, None)
    assert blk(E(None, FAKE.value, 3, 1.0, None)) == qnn.QNN_ERR_UNSUPPORTED            # a 3-bit shortcut is not fp4
    assert blk(E(None, FAKE.value, 2, 1.0, None), D(1, 8, 8, 64, 63, 3, 3, 1, 1, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED
    assert blk(E(ODD.value, None, 0, 0.0, None)) == qnn.QNN_ERR_ALIGNMENT
    assert blk(E(FAKE.value, FAKE.value, 2, 1.0, FAKE.value), D(0, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_OK
    assert L.qnn_encode_levels_fp4(FAKE, 0, 64, 1.0, 3, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_levels_fp4(FAKE, 0, 63, 1.0, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encode_levels_fp4(FAKE, 2, 64, 1.0, 2, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED
    assert L.qnn_levels_to_fp4(FAKE, 63, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_levels_to_fp4(FAKE, 64, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert L.qnn_levels_to_fp4(None, 0, None, None) == qnn.QNN_OK
    assert L.qnn_maxpool_levels_fp4(FAKE, 1, 8, 8, 33, 2, 2, 0, 0, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED   # odd C
    assert L.qnn_maxpool_levels_fp4(FAKE, 1, 8, 8, 32, 2, 2, 2, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG   # pad > k / 2
    assert L.qnn_maxpool_levels_fp4(FAKE, 1, 8, 8, 32, 2, 2, 0, 0, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert L.qnn_maxpool_levels_fp4(None, 0, 8, 8, 32, 2, 2, 0, 0, None, None) == qnn.QNN_OK


def _declared_in(header, prefix="qnn_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(%s[a-z0-9_]+)\s*\(" % prefix, text)))


def test_probe_library_exports_and_argument_errors():
    # the issue-rate loops live in a library of their own (include/qnn_probe.h), outside the product library
    from paper_1905_13389_amd import probe
    L = probe.lib()
    assert set(_declared_in("qnn_probe.h")) == set(probe.EXPORTS) | {"qnn_timeline_set", "qnn_level_gemm_timeline_set"}
    for n in probe.EXPORTS:
        assert getattr(L, n) is not None
    product = ctypes.CDLL(os.path.join(os.path.dirname(probe.LIB_PATH), "libqnn.so"))
    for n in ("qnn_probe_valu", "qnn_probe_mfma", "qnn_probe_mfma_operands", "qnn_timeline_set", "qnn_level_gemm_timeline_set"):
        assert not hasattr(product, n)
    assert L.qnn_probe_valu(99, 1, 1, FAKE, None, None) < 0 and b"mode" in L.qnn_probe_last_error()
    assert L.qnn_probe_valu(0, 0, 1, FAKE, None, None) < 0
    assert L.qnn_probe_valu(0, 1, -1, FAKE, None, None) < 0
    assert L.qnn_probe_valu(0, 1, 1, None, None, None) < 0
    assert L.qnn_probe_mfma(2, 1, 1, FAKE, None) < 0
    assert L.qnn_probe_mfma(0, 70000, 1, FAKE, None) < 0
    assert L.qnn_probe_mfma(0, 1, 1, None, None) < 0
    assert L.qnn_probe_mfma_operands(2, 1, 1, FAKE, FAKE, None, None) < 0 and b"mode" in L.qnn_probe_last_error()
    assert L.qnn_probe_mfma_operands(0, 1, 1, None, FAKE, None, None) < 0 and b"operand" in L.qnn_probe_last_error()
    assert L.qnn_probe_mfma_operands(0, 1, 1, ctypes.c_void_p(FAKE.value + 4), FAKE, None, None) < 0
    assert L.qnn_probe_mfma_operands(0, 1, 1, FAKE, None, None, None) < 0


def test_timeline_library_exports_and_argument_errors():
    # the convolution kernels with wave timestamps: a diagnostic library of its own with the product's entry points
    from paper_1905_13389_amd import probe
    L = probe.timeline_lib()
    for n in probe.TIMELINE_EXPORTS:
        assert getattr(L, n) is not None
    assert L.qnn_timeline_set(None, 8, 1) < 0 and b"buffer" in L.qnn_last_error()
    assert L.qnn_timeline_set(FAKE, -1, 1) < 0
    assert L.qnn_timeline_set(None, 0, 1) == 0
    import torch
    with pytest.raises(ValueError):
        probe.qnn_timeline_set(torch.zeros((4, 3), dtype=torch.int64))
    assert L.qnn_level_gemm_timeline_set(None, 8) < 0 and b"buffer" in L.qnn_last_error()
    assert L.qnn_level_gemm_timeline_set(FAKE, -1) < 0
    assert L.qnn_level_gemm_timeline_set(None, 0) == 0
    with pytest.raises(ValueError):
        probe.qnn_level_gemm_timeline_set(torch.zeros((4, 4), dtype=torch.int64))
    # its entry points check their arguments like the product's
    from paper_1905_13389_amd import qnn as q
    assert L.qnn_level_gemm_i8(FAKE, FAKE, 4, 4, 32, None, None, None, None) == q.QNN_ERR_INVALID_ARG
    assert L.qnn_conv2d(ctypes.byref(q.qnn_conv_desc(1, 8, 8, 64, 64, 3, 3, 0, 1, 2, 2)), FAKE, FAKE, None, FAKE, None, None,
                        0.0, 0, None) == q.QNN_ERR_INVALID_ARG


def test_training_gradient_argument_errors(qnn):
    L = qnn.lib()
    assert L.qnn_quantize_ste_backward(FAKE, FAKE, -1, 1.0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_quantize_ste_backward(FAKE, FAKE, 8, 0.0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_quantize_ste_backward(FAKE, None, 8, 1.0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_quantize_ste_backward(FAKE, FAKE, 8, 1.0, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert L.qnn_quantize_ste_backward(None, None, 0, 1.0, None, None) == qnn.QNN_OK
    assert L.qnn_encoder_backward(FAKE, FAKE, 8, 1.0, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encoder_backward(FAKE, FAKE, 8, 1.0, 9, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encoder_backward(FAKE, FAKE, 8, float("nan"), 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert L.qnn_encoder_backward(ODD, FAKE, 8, 1.0, 2, FAKE, None) == qnn.QNN_ERR_ALIGNMENT
    assert L.qnn_encoder_backward(None, None, 0, 1.0, 2, None, None) == qnn.QNN_OK


def test_matrix_core_variant_argument_errors(qnn):
    L = qnn.lib()
    assert L.qnn_level_row_bytes(1) == 128 and L.qnn_level_row_bytes(128) == 128 and L.qnn_level_row_bytes(129) == 256
    ps = L.qnn_plane_sum_i8
    assert ps(FAKE, 8, 4, 64, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED       # 8-bit levels do not fit int8
    assert ps(FAKE, 2, -1, 64, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert ps(None, 2, 4, 64, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert ps(FAKE, 2, 4, 64, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert ps(None, 2, 0, 64, None, None) == qnn.QNN_OK
    g = L.qnn_level_gemm_i8
    assert g(FAKE, FAKE, 4, 4, 64, None, None, None, None) == qnn.QNN_ERR_INVALID_ARG     # no output
    assert g(FAKE, FAKE, 4, 4, 64, None, None, FAKE, None) == qnn.QNN_ERR_INVALID_ARG     # out, no scale
    assert g(None, FAKE, 4, 4, 64, FAKE, None, None, None) == qnn.QNN_ERR_INVALID_ARG
    assert g(FAKE, ODD, 4, 4, 64, FAKE, None, None, None) == qnn.QNN_ERR_ALIGNMENT
    assert g(FAKE, FAKE, 4, 4, 1 << 20, FAKE, None, None, None) == qnn.QNN_ERR_RANGE      # 127^2 n >= 2^31
    assert g(None, None, 0, 4, 64, FAKE, None, None, None) == qnn.QNN_OK
    e = L.qnn_encode_levels_i8
    assert e(FAKE, 2, 64, 1.0, 2, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED    # int8 input has no quantizer
    assert e(FAKE, 0, 64, 1.0, 8, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert e(FAKE, 0, -1, 1.0, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert e(FAKE, 0, 64, 0.0, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert e(None, 0, 64, 1.0, 2, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert e(ODD, 0, 64, 1.0, 2, FAKE, None) == qnn.QNN_ERR_ALIGNMENT
    assert e(None, 0, 0, 1.0, 2, None, None) == qnn.QNN_OK

    def conv(desc, a=FAKE, w=FAKE, scale=None, acc=FAKE, out=None, nxt=None, clip=0.0, nbits=0):
        return L.qnn_level_conv2d_i8(ctypes.byref(desc) if desc is not None else None, a, w, scale, acc, out,
                                     nxt, clip, nbits, None)

    D = qnn.qnn_conv_desc
    ok = D(1, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)
    assert conv(None) == qnn.QNN_ERR_INVALID_ARG
    assert conv(D(1, 8, 8, 64, 64, 3, 3, 1, 1, 8, 2)) == qnn.QNN_ERR_INVALID_ARG   # 8-bit levels
    assert conv(D(1, 8, 8, 24, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED   # Cin % 16
    assert conv(D(1, 8, 8, 64, 64, 7, 7, 1, 3, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED   # 49 taps
    assert conv(D(1, 8, 8, 4096, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_ERR_UNSUPPORTED  # reduction > 16 KiB
    assert conv(D(1 << 20, 64, 64, 64, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_ERR_RANGE  # 32-bit offsets
    assert conv(ok, acc=None) == qnn.QNN_ERR_INVALID_ARG
    assert conv(ok, scale=FAKE, nxt=FAKE, clip=1.0, nbits=8) == qnn.QNN_ERR_INVALID_ARG
    assert conv(ok, a=None) == qnn.QNN_ERR_INVALID_ARG
    assert conv(ok, w=ODD) == qnn.QNN_ERR_ALIGNMENT
    assert conv(D(0, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2)) == qnn.QNN_OK


def test_pool_argument_errors_and_out_size(qnn):
    L = qnn.lib()
    assert L.qnn_pool_out_size(8, 2, 2, 0, 0) == 4
    assert L.qnn_pool_out_size(75, 2, 2, 0, 0) == 37 and L.qnn_pool_out_size(75, 2, 2, 0, 1) == 38
    assert L.qnn_pool_out_size(112, 3, 2, 1, 0) == 56
    assert L.qnn_pool_out_size(4, 3, 2, 1, 1) == 3
    assert L.qnn_pool_out_size(5, 2, 2, 1, 1) == 3          # a fourth window would start in the right padding
    assert L.qnn_pool_out_size(3, 5, 1, 0, 0) == -1 and L.qnn_pool_out_size(8, 2, 2, 2, 0) == -1
    mp = L.qnn_maxpool_planes
    assert mp(FAKE, 0, 1, 8, 8, 32, 2, 2, 0, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert mp(FAKE, 2, 1, 8, 8, 32, 2, 0, 0, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert mp(FAKE, 2, 1, 8, 8, 32, 2, 2, 2, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert mp(FAKE, 2, 1, 8, 8, 32, 9, 1, 0, 0, FAKE, None) == qnn.QNN_ERR_UNSUPPORTED
    assert mp(FAKE, 2, 1, 2, 2, 32, 3, 1, 0, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert mp(None, 2, 1, 8, 8, 32, 2, 2, 0, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert mp(FAKE, 2, 1, 8, 8, 32, 2, 2, 0, 0, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert mp(None, 2, 0, 8, 8, 32, 2, 2, 0, 0, None, None) == qnn.QNN_OK
    ml = L.qnn_maxpool_levels_i8
    assert ml(FAKE, 1, 8, 8, 0, 2, 2, 0, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert ml(ODD, 1, 8, 8, 16, 2, 2, 0, 0, FAKE, None) == qnn.QNN_ERR_ALIGNMENT
    assert ml(None, 0, 8, 8, 16, 2, 2, 0, 0, None, None) == qnn.QNN_OK


def test_dense_layer_argument_errors(qnn):
    L = qnn.lib()
    assert ctypes.sizeof(qnn.qnn_dense_conv_desc) == 5 * 8 + 4 * 4
    dc = L.qnn_dense_conv2d_f32
    d = qnn.qnn_dense_conv_desc(2, 8, 8, 3, 16, 3, 3, 1, 1)
    ok = (ctypes.byref(d), FAKE, FAKE, None, None, 0)
    assert dc(None, FAKE, FAKE, None, None, 0, FAKE, None, 0.0, 0, None) == qnn.QNN_ERR_INVALID_ARG
    assert dc(*ok, None, None, 0.0, 0, None) == qnn.QNN_ERR_INVALID_ARG               # no output at all
    assert dc(*ok, None, FAKE, 1.0, 0, None) == qnn.QNN_ERR_INVALID_ARG               # planes without bits
    assert dc(*ok, None, FAKE, 1.0, 9, None) == qnn.QNN_ERR_INVALID_ARG
    assert dc(*ok, None, FAKE, 0.0, 2, None) == qnn.QNN_ERR_INVALID_ARG               # planes without a clip
    assert dc(*ok, None, FAKE, float("inf"), 2, None) == qnn.QNN_ERR_INVALID_ARG
    assert dc(ctypes.byref(d), None, FAKE, None, None, 0, FAKE, None, 0.0, 0, None) == qnn.QNN_ERR_INVALID_ARG
    assert dc(ctypes.byref(d), FAKE, FAKE, None, None, 0, ODD, None, 0.0, 0, None) == qnn.QNN_ERR_ALIGNMENT
    assert dc(ctypes.byref(d), ODD, FAKE, None, None, 0, FAKE, None, 0.0, 0, None) == qnn.QNN_ERR_ALIGNMENT
    for bad in (qnn.qnn_dense_conv_desc(2, 8, 8, 0, 16, 3, 3, 1, 1), qnn.qnn_dense_conv_desc(2, 8, 8, 3, 16, 3, 3, 0, 1),
                qnn.qnn_dense_conv_desc(2, 8, 8, 3, 16, 3, 3, 1, -1), qnn.qnn_dense_conv_desc(2, 2, 2, 3, 16, 5, 5, 1, 1),
                qnn.qnn_dense_conv_desc(-1, 8, 8, 3, 16, 3, 3, 1, 1)):
        assert dc(ctypes.byref(bad), FAKE, FAKE, None, None, 0, FAKE, None, 0.0, 0, None) == qnn.QNN_ERR_INVALID_ARG
    big = qnn.qnn_dense_conv_desc(1 << 20, 64, 64, 3, 16, 3, 3, 1, 1)                  # 2^32 output pixels
    assert dc(ctypes.byref(big), FAKE, FAKE, None, None, 0, FAKE, None, 0.0, 0, None) == qnn.QNN_ERR_RANGE
    empty = qnn.qnn_dense_conv_desc(0, 8, 8, 3, 16, 3, 3, 1, 1)
    assert dc(ctypes.byref(empty), None, None, None, None, 0, FAKE, None, 0.0, 0, None) == qnn.QNN_OK
    dl = L.qnn_dense_conv2d_f32_levels
    assert dl(*ok, None, FAKE, 1.0, 8, None) == qnn.QNN_ERR_UNSUPPORTED               # int8 levels hold 7 bits
    assert dl(*ok, None, None, 1.0, 3, None) == qnn.QNN_ERR_INVALID_ARG
    assert dl(*ok, None, ODD, 1.0, 3, None) == qnn.QNN_ERR_ALIGNMENT
    ap = L.qnn_global_avgpool_f32
    assert ap(FAKE, 2, 0, 8, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert ap(FAKE, 2, 4, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert ap(None, 2, 4, 8, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert ap(None, 0, 4, 8, None, None) == qnn.QNN_OK
    assert ap(FAKE, 1 << 40, 1 << 20, 8, FAKE, None) == qnn.QNN_ERR_RANGE
    fc = L.qnn_dense_fc_f32
    assert fc(FAKE, FAKE, None, 4, 0, 8, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert fc(FAKE, FAKE, None, 4, 8, 0, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert fc(FAKE, FAKE, None, 4, 8, 8, None, None) == qnn.QNN_ERR_INVALID_ARG
    assert fc(None, FAKE, None, 4, 8, 8, FAKE, None) == qnn.QNN_ERR_INVALID_ARG
    assert fc(FAKE, FAKE, None, 4, 8, 8, ODD, None) == qnn.QNN_ERR_ALIGNMENT
    assert fc(None, None, None, 0, 8, 8, FAKE, None) == qnn.QNN_OK


def test_fc_fused_argument_errors(qnn):
    f = qnn.lib().qnn_fc_fused
    good = dict(src=FAKE, dtype=qnn.QNN_DTYPE_F32, rows=4, n=64, stride=64, clip=1.0, a_bits=2, w=FAKE, w_bits=2, cols=8,
                scale=FAKE, acc=FAKE, out=FAKE)

    def call(**kw):
        a = dict(good, **kw)
        return f(a["src"], a["dtype"], a["rows"], a["n"], a["stride"], a["clip"], a["a_bits"], a["w"], a["w_bits"], a["cols"],
                 a["scale"], a["acc"], a["out"], None)

    assert call(dtype=7) == qnn.QNN_ERR_UNSUPPORTED
    assert call(a_bits=0) == qnn.QNN_ERR_INVALID_ARG and call(w_bits=9) == qnn.QNN_ERR_INVALID_ARG
    assert call(dtype=qnn.QNN_DTYPE_I8, a_bits=8) == qnn.QNN_ERR_UNSUPPORTED
    assert call(rows=-1) == qnn.QNN_ERR_INVALID_ARG and call(stride=63) == qnn.QNN_ERR_INVALID_ARG
    assert call(clip=0.0) == qnn.QNN_ERR_INVALID_ARG and call(clip=float("nan")) == qnn.QNN_ERR_INVALID_ARG
    assert call(acc=None, out=None) == qnn.QNN_ERR_INVALID_ARG
    assert call(scale=None) == qnn.QNN_ERR_INVALID_ARG
    assert call(src=None) == qnn.QNN_ERR_INVALID_ARG and call(w=None) == qnn.QNN_ERR_INVALID_ARG
    assert call(w=ODD) == qnn.QNN_ERR_ALIGNMENT and call(acc=ODD) == qnn.QNN_ERR_ALIGNMENT
    assert call(n=1 << 20, stride=1 << 20, a_bits=8, w_bits=8) == qnn.QNN_ERR_RANGE
    assert call(n=40000, stride=40000) == qnn.QNN_ERR_UNSUPPORTED          # planes of 4 rows do not fit LDS
    assert call(rows=0, src=None) == qnn.QNN_OK and call(cols=0) == qnn.QNN_OK
