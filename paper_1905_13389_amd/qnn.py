"""ctypes binding of libqnn.so: same names and argument order as include/qnn.h.

Marshalling only.  Tensors are torch CUDA tensors used as device-memory handles; the stream is
torch's current stream.  There is no CPU fallback: a missing library or a failing call raises.
"""
import ctypes
import os
import sys

import torch  # loads the HIP runtime that libqnn.so binds to

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqnn.so")  # the in-tree build; there is no way to point at another one

QNN_OK = 0
QNN_ERR_INVALID_ARG = -1
QNN_ERR_UNSUPPORTED = -2
QNN_ERR_ALIGNMENT = -3
QNN_ERR_RANGE = -4
QNN_ERR_LAUNCH = -5

QNN_DTYPE_F32 = 0
QNN_DTYPE_BF16 = 1
QNN_DTYPE_I8 = 2

EXPORTS = ("qnn_encode_pack", "qnn_binary_gemm", "qnn_dequant_scale", "qnn_conv2d", "qnn_conv2d_block",
           "qnn_conv2d_chain_static", "qnn_conv2d_chain_static_max_outputs", "qnn_conv2d_dilated", "qnn_level_conv2d_dilated_i8", "qnn_level_conv2d_dilated_fp4",
           "qnn_level_conv2d_block_i8", "qnn_deconv_phase_words", "qnn_deconv_pack_weights", "qnn_deconv2d",
           "qnn_quantize_ste_backward", "qnn_encoder_backward",
           "qnn_level_row_bytes", "qnn_plane_sum_i8", "qnn_level_gemm_i8",
           "qnn_encode_levels_i8", "qnn_level_conv2d_i8",
           "qnn_fp4_row_bytes", "qnn_plane_sum_fp4", "qnn_level_gemm_fp4",
           "qnn_encode_levels_fp4", "qnn_levels_to_fp4", "qnn_level_conv2d_fp4", "qnn_level_conv2d_block_fp4", "qnn_maxpool_levels_fp4",
           "qnn_level_deconv_workspace_bytes", "qnn_level_deconv_flip_weights", "qnn_level_deconv2d_i8", "qnn_level_deconv2d_fp4",
           "qnn_pool_out_size", "qnn_maxpool_planes", "qnn_maxpool_levels_i8",
           "qnn_dense_conv2d_f32", "qnn_dense_conv2d_f32_levels", "qnn_global_avgpool_f32", "qnn_dense_fc_f32", "qnn_fc_fused",
           "qnn_last_error", "qnn_version", "qnn_build_id")


class QnnError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("libqnn error %d: %s" % (code, message))
        self.code = code


class qnn_conv_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64),
                ("Cin", ctypes.c_int64), ("Cout", ctypes.c_int64),
                ("kh", ctypes.c_int32), ("kw", ctypes.c_int32), ("stride", ctypes.c_int32),
                ("pad", ctypes.c_int32), ("a_bits", ctypes.c_int32), ("w_bits", ctypes.c_int32)]


class qnn_dense_conv_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64),
                ("Cin", ctypes.c_int64), ("Cout", ctypes.c_int64),
                ("kh", ctypes.c_int32), ("kw", ctypes.c_int32), ("stride", ctypes.c_int32), ("pad", ctypes.c_int32)]


class qnn_block_epilogue(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("res_q", ctypes.c_void_p), ("res_bits", ctypes.c_int32),
                ("res_scale", ctypes.c_float), ("res_f32", ctypes.c_void_p), ("relu", ctypes.c_int32)]


_lib = None


def _built_from_current_sources():
    """True when the in-tree library exists and carries the digest of the sources as they stand now.  The file
    is searched for the digest instead of being loaded and asked: a library that has been dlopen'ed once stays
    mapped, so a stale one could not be replaced by a rebuilt one within the same process."""
    if not os.path.exists(LIB_PATH):
        return False
    with open(LIB_PATH, "rb") as f:
        return _build.source_id().encode() in f.read()


def lib():
    """The loaded C-ABI library.  Built in-tree beforehand; if the file is missing, or was built from other
    sources than the ones in csrc/ now (the library carries a hash of them), it is compiled here (hipcc
    cross-compiles without a GPU).  Any failure raises: there is no fallback."""
    global _lib
    if _lib is None:
        if not _built_from_current_sources():
            print("libqnn.so is missing or older than its sources: building", file=sys.stderr, flush=True)
            _build.build()
            if not _built_from_current_sources():
                raise RuntimeError("libqnn.so does not carry the id of the sources it was just built from")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
        L.qnn_encode_pack.argtypes = [vp, i32, i64, i64, i64, f32, i32, vp, vp]
        L.qnn_encode_pack.restype = i32
        L.qnn_binary_gemm.argtypes = [vp, i32, vp, i32, i64, i64, i64, vp, vp, vp, vp]
        L.qnn_binary_gemm.restype = i32
        L.qnn_dequant_scale.argtypes = [vp, vp, i64, i64, vp, vp]
        L.qnn_dequant_scale.restype = i32
        L.qnn_conv2d.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_conv2d.restype = i32
        L.qnn_conv2d_block.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, ctypes.POINTER(qnn_block_epilogue),
                                       vp, vp, vp, f32, i32, vp]
        L.qnn_conv2d_block.restype = i32
        L.qnn_conv2d_chain_static.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, f32, i32, vp]
        L.qnn_conv2d_chain_static.restype = i32
        L.qnn_conv2d_chain_static_max_outputs.argtypes = []
        L.qnn_conv2d_chain_static_max_outputs.restype = i64
        L.qnn_level_conv2d_block_i8.argtypes = L.qnn_conv2d_block.argtypes
        L.qnn_level_conv2d_block_i8.restype = i32
        L.qnn_dense_conv2d_f32.argtypes = [ctypes.POINTER(qnn_dense_conv_desc), vp, vp, vp, vp, i32, vp, vp, f32, i32, vp]
        L.qnn_dense_conv2d_f32.restype = i32
        L.qnn_dense_conv2d_f32_levels.argtypes = L.qnn_dense_conv2d_f32.argtypes
        L.qnn_dense_conv2d_f32_levels.restype = i32
        L.qnn_global_avgpool_f32.argtypes = [vp, i64, i64, i64, vp, vp]
        L.qnn_global_avgpool_f32.restype = i32
        L.qnn_dense_fc_f32.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
        L.qnn_dense_fc_f32.restype = i32
        L.qnn_fc_fused.argtypes = [vp, i32, i64, i64, i64, f32, i32, vp, i32, i64, vp, vp, vp, vp]
        L.qnn_fc_fused.restype = i32
        L.qnn_level_row_bytes.argtypes = [i64]
        L.qnn_level_row_bytes.restype = i64
        L.qnn_plane_sum_i8.argtypes = [vp, i32, i64, i64, vp, vp]
        L.qnn_plane_sum_i8.restype = i32
        L.qnn_level_gemm_i8.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp]
        L.qnn_level_gemm_i8.restype = i32
        L.qnn_pool_out_size.argtypes = [i64, i32, i32, i32, i32]
        L.qnn_pool_out_size.restype = i64
        L.qnn_maxpool_planes.argtypes = [vp, i32, i64, i64, i64, i64, i32, i32, i32, i32, vp, vp]
        L.qnn_maxpool_planes.restype = i32
        L.qnn_maxpool_levels_i8.argtypes = [vp, i64, i64, i64, i64, i32, i32, i32, i32, vp, vp]
        L.qnn_maxpool_levels_i8.restype = i32
        L.qnn_fp4_row_bytes.argtypes = [i64]
        L.qnn_fp4_row_bytes.restype = i64
        L.qnn_plane_sum_fp4.argtypes = [vp, i32, i64, i64, vp, vp]
        L.qnn_plane_sum_fp4.restype = i32
        L.qnn_level_gemm_fp4.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp]
        L.qnn_level_gemm_fp4.restype = i32
        L.qnn_encode_levels_i8.argtypes = [vp, i32, i64, f32, i32, vp, vp]
        L.qnn_encode_levels_i8.restype = i32
        L.qnn_level_conv2d_i8.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_level_conv2d_i8.restype = i32
        for f in (L.qnn_conv2d_dilated, L.qnn_level_conv2d_dilated_i8, L.qnn_level_conv2d_dilated_fp4):
            f.argtypes = [ctypes.POINTER(qnn_conv_desc), i32, vp, vp, vp, vp, vp, vp, f32, i32, vp]
            f.restype = i32
        L.qnn_deconv_phase_words.argtypes = [i32, i64, i32, i32, i64, i32]
        L.qnn_deconv_phase_words.restype = i64
        L.qnn_deconv_pack_weights.argtypes = [vp, i32, i64, i32, i32, i64, i32, vp, vp]
        L.qnn_deconv_pack_weights.restype = i32
        L.qnn_deconv2d.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_deconv2d.restype = i32
        L.qnn_quantize_ste_backward.argtypes = [vp, vp, i64, f32, vp, vp]
        L.qnn_quantize_ste_backward.restype = i32
        L.qnn_encoder_backward.argtypes = [vp, vp, i64, f32, i32, vp, vp]
        L.qnn_encoder_backward.restype = i32
        L.qnn_encode_levels_fp4.argtypes = [vp, i32, i64, f32, i32, vp, vp]
        L.qnn_encode_levels_fp4.restype = i32
        L.qnn_levels_to_fp4.argtypes = [vp, i64, vp, vp]
        L.qnn_levels_to_fp4.restype = i32
        L.qnn_level_conv2d_fp4.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_level_conv2d_fp4.restype = i32
        L.qnn_level_deconv_workspace_bytes.argtypes = [ctypes.POINTER(qnn_conv_desc), i32]
        L.qnn_level_deconv_workspace_bytes.restype = i64
        L.qnn_level_deconv_flip_weights.argtypes = [vp, i64, i32, i32, i64, vp, vp]
        L.qnn_level_deconv_flip_weights.restype = i32
        for f in (L.qnn_level_deconv2d_i8, L.qnn_level_deconv2d_fp4):
            f.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, vp]
            f.restype = i32
        L.qnn_level_conv2d_block_fp4.argtypes = L.qnn_conv2d_block.argtypes
        L.qnn_level_conv2d_block_fp4.restype = i32
        L.qnn_maxpool_levels_fp4.argtypes = [vp, i64, i64, i64, i64, i32, i32, i32, i32, vp, vp]
        L.qnn_maxpool_levels_fp4.restype = i32
        L.qnn_last_error.argtypes = []
        L.qnn_last_error.restype = ctypes.c_char_p
        L.qnn_version.argtypes = []
        L.qnn_version.restype = i32
        L.qnn_build_id.argtypes = []
        L.qnn_build_id.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != QNN_OK:
        raise QnnError(rc, lib().qnn_last_error().decode())


_PLANES = (torch.int32, torch.uint32)  # packed bit-vectors: uint32 words, usually held as int32 tensors
_I32 = (torch.int32,)
_F32 = (torch.float32,)
_I8 = (torch.int8,)
_U8 = (torch.uint8,)
_VALUES = (torch.float32, torch.bfloat16)


def _prod(shape):
    n = 1
    for extent in shape:
        n *= int(extent)
    return n


def _arg(name, t, dtypes, shape=None, numel=None, optional=False):
    """One tensor argument, checked before its address is taken: the C side sees a bare pointer and can tell
    neither a slice from a whole tensor nor an undersized buffer from a fitting one.  Raises on a wrong dtype,
    a non-contiguous tensor or a wrong shape / element count; _ptr, which takes the address once all arguments of
    a call have been checked against each other, refuses a tensor that is not in device memory."""
    if t is None:
        if optional:
            return None
        raise ValueError("%s: missing" % name)
    if not isinstance(t, torch.Tensor):
        raise TypeError("%s: a torch tensor is needed, got %s" % (name, type(t).__name__))
    if t.dtype not in dtypes:
        raise TypeError("%s: dtype %s, expected %s" % (name, t.dtype, " or ".join(str(d) for d in dtypes)))
    if not t.is_contiguous():
        raise ValueError("%s: not contiguous (strides %s for shape %s)" % (name, tuple(t.stride()), tuple(t.shape)))
    if shape is not None and tuple(t.shape) != tuple(int(e) for e in shape):
        raise ValueError("%s: shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    if numel is not None and t.numel() != int(numel):
        raise ValueError("%s: %d elements, expected %d" % (name, t.numel(), int(numel)))
    return t


def _out(name, t, dtype, shape, like, want=True):
    """A caller-supplied output buffer (element count checked) or a fresh one; None when not wanted."""
    if t is not None:
        return _arg(name, t, _PLANES if "planes" in name else (dtype,), numel=_prod(shape))
    if not want:
        return None
    return torch.empty(tuple(int(e) for e in shape), dtype=dtype, device=like.device)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s tensor of shape %s: not a CUDA (device) tensor" % (t.dtype, tuple(t.shape)))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


_DTYPES = {torch.float32: QNN_DTYPE_F32, torch.bfloat16: QNN_DTYPE_BF16, torch.int8: QNN_DTYPE_I8}


def qnn_version():
    return lib().qnn_version()


def _rows_view(name, src):
    """(rows, n, row_stride_elems) of an encoder input: a contiguous tensor [..., n], or a 2-D view whose rows
    are contiguous and a fixed number of elements (>= n) apart -- e.g. a column range of a wider matrix."""
    if not isinstance(src, torch.Tensor):
        raise TypeError("%s: a torch tensor is needed" % name)
    if src.dtype not in _DTYPES:
        raise TypeError("%s: dtype %s, expected float32, bfloat16 or int8" % (name, src.dtype))
    if src.dim() < 1:
        raise ValueError("%s: needs at least one dimension" % name)
    n = int(src.shape[-1])
    if src.is_contiguous():
        rows, stride = (src.numel() // n if n else 0), n
    elif src.dim() == 2 and (n <= 1 or src.stride(1) == 1) and src.stride(0) >= n:
        rows, stride = int(src.shape[0]), int(src.stride(0))
    else:
        raise ValueError("%s: neither contiguous nor a 2-D view of contiguous rows (strides %s)"
                         % (name, tuple(src.stride())))
    return rows, n, stride


def qnn_encode_pack(src, clip, bits, planes=None):
    """src: CUDA tensor [..., n] (fp32 / bf16 values, or int8 levels), contiguous, or a 2-D view with contiguous
    rows `src.stride(0)` elements apart (the C call's row_stride_elems).  Returns planes uint32-as-int32
    [bits][rows][ceil(n/32)] with rows = product of the leading dimensions."""
    rows, n, stride = _rows_view("src", src)
    nw = (n + 31) // 32
    planes = _out("planes", planes, torch.int32, (bits, rows, nw), src)
    _check(lib().qnn_encode_pack(_ptr(src), _DTYPES[src.dtype], rows, n, stride, float(clip), int(bits),
                                 _ptr(planes), _stream()))
    return planes


def _w_planes(name, t, n=None):
    _arg(name, t, _PLANES)
    if t.dim() != 3:
        raise ValueError("%s: expected [bits][rows][words], got shape %s" % (name, tuple(t.shape)))
    if n is not None and t.shape[2] != (n + 31) // 32:
        raise ValueError("%s: %d words per row, expected %d for n = %d" % (name, t.shape[2], (n + 31) // 32, n))
    return tuple(int(e) for e in t.shape)


def qnn_fc_fused(src, clip, a_bits, w_planes, want_acc=True, scale=None, acc=None, out=None):
    """src [rows][n] (fp32 / bf16 values or int8 levels; contiguous or rows a fixed stride apart), w_planes
    [w_bits][cols][nw] -> (acc int32 [rows][cols] or None, out fp32 [rows][cols] or None): qnn_encode_pack +
    qnn_binary_gemm in one launch."""
    if not isinstance(src, torch.Tensor) or src.dim() != 2:
        raise ValueError("src: expected a 2-D tensor [rows][n]")
    rows, n, stride = _rows_view("src", src)
    w_bits, cols, _ = _w_planes("w_planes", w_planes, n)
    _arg("scale", scale, _F32, shape=(cols,), optional=True)
    acc = _out("acc", acc, torch.int32, (rows, cols), src, want_acc)
    out = _out("out", out, torch.float32, (rows, cols), src, scale is not None)
    _check(lib().qnn_fc_fused(_ptr(src), _DTYPES[src.dtype], rows, n, stride, float(clip), int(a_bits), _ptr(w_planes),
                              w_bits, cols, _ptr(scale), _ptr(acc), _ptr(out), _stream()))
    return acc, out


def qnn_binary_gemm(a_planes, w_planes, n, want_acc=True, scale=None, acc=None, out=None):
    """a_planes [a_bits][rows][nw], w_planes [w_bits][cols][nw] -> (acc int32 [rows][cols] or None,
    out fp32 [rows][cols] or None)."""
    a_bits, rows, _ = _w_planes("a_planes", a_planes, n)
    w_bits, cols, _ = _w_planes("w_planes", w_planes, n)
    _arg("scale", scale, _F32, shape=(cols,), optional=True)
    acc = _out("acc", acc, torch.int32, (rows, cols), a_planes, want_acc)
    out = _out("out", out, torch.float32, (rows, cols), a_planes, scale is not None)
    _check(lib().qnn_binary_gemm(_ptr(a_planes), a_bits, _ptr(w_planes), w_bits, rows, cols, n,
                                 _ptr(acc), _ptr(scale), _ptr(out), _stream()))
    return acc, out


def qnn_level_row_bytes(n):
    return lib().qnn_level_row_bytes(int(n))


def qnn_plane_sum_i8(planes, n, levels=None):
    """planes [bits][rows][nw] -> int8 levels [rows][qnn_level_row_bytes(n)] (bit-plane-sum variant)."""
    bits, rows, _ = _w_planes("planes", planes, n)
    levels = _out("levels", levels, torch.int8, (rows, qnn_level_row_bytes(n)), planes)
    _check(lib().qnn_plane_sum_i8(_ptr(planes), bits, rows, n, _ptr(levels), _stream()))
    return levels


def _level_gemm(entry, row_bytes, dtypes, a_levels, w_levels, n, want_acc, scale, acc, out):
    _arg("a_levels", a_levels, dtypes)
    _arg("w_levels", w_levels, dtypes)
    if a_levels.dim() != 2 or w_levels.dim() != 2 or a_levels.shape[1] != row_bytes or w_levels.shape[1] != row_bytes:
        raise ValueError("level tensors must be [rows][%d] for n = %d, got %s and %s"
                         % (row_bytes, n, tuple(a_levels.shape), tuple(w_levels.shape)))
    rows, cols = int(a_levels.shape[0]), int(w_levels.shape[0])
    _arg("scale", scale, _F32, shape=(cols,), optional=True)
    acc = _out("acc", acc, torch.int32, (rows, cols), a_levels, want_acc)
    out = _out("out", out, torch.float32, (rows, cols), a_levels, scale is not None)
    _check(entry(_ptr(a_levels), _ptr(w_levels), rows, cols, n, _ptr(acc), _ptr(scale), _ptr(out), _stream()))
    return acc, out


def qnn_level_gemm_i8(a_levels, w_levels, n, want_acc=True, scale=None, acc=None, out=None):
    """int8 MFMA GEMM on levels as written by qnn_plane_sum_i8 -> (acc int32 or None, out fp32 or None)."""
    return _level_gemm(lib().qnn_level_gemm_i8, qnn_level_row_bytes(n), _I8, a_levels, w_levels, n, want_acc, scale,
                       acc, out)


def qnn_pool_out_size(size, k, stride, pad=0, ceil_mode=False):
    return int(lib().qnn_pool_out_size(int(size), int(k), int(stride), int(pad), int(bool(ceil_mode))))


def qnn_maxpool_planes(planes, shape, channels, k, stride, pad=0, ceil_mode=False, out=None):
    """planes [bits][B*H*W][cw] of an NHWC tensor of shape=(B, H, W) -> planes [bits][B*Ho*Wo][cw]."""
    B, H, W = shape
    cw = (channels + 31) // 32
    _arg("planes", planes, _PLANES)
    bits = int(planes.shape[0])
    if planes.numel() != bits * B * H * W * cw:
        raise ValueError("planes: %d words, expected [%d][%d*%d*%d][%d]" % (planes.numel(), bits, B, H, W, cw))
    ho, wo = qnn_pool_out_size(H, k, stride, pad, ceil_mode), qnn_pool_out_size(W, k, stride, pad, ceil_mode)
    out = _out("out_planes", out, torch.int32, (bits, B * max(ho, 0) * max(wo, 0), cw), planes)
    _check(lib().qnn_maxpool_planes(_ptr(planes), bits, B, H, W, channels, int(k), int(stride), int(pad),
                                    int(bool(ceil_mode)), _ptr(out), _stream()))
    return out


def _pool_levels(entry, dtypes, cfactor, levels, k, stride, pad, ceil_mode, out):
    _arg("levels", levels, dtypes)
    if levels.dim() != 4:
        raise ValueError("levels: expected [B][H][W][C], got shape %s" % (tuple(levels.shape),))
    B, H, W, cb = (int(e) for e in levels.shape)
    ho, wo = qnn_pool_out_size(H, k, stride, pad, ceil_mode), qnn_pool_out_size(W, k, stride, pad, ceil_mode)
    out = _out("out_levels", out, levels.dtype, (B, max(ho, 0), max(wo, 0), cb), levels)
    _check(entry(_ptr(levels), B, H, W, cfactor * cb, int(k), int(stride), int(pad), int(bool(ceil_mode)), _ptr(out),
                 _stream()))
    return out


def qnn_maxpool_levels_i8(levels, k, stride, pad=0, ceil_mode=False, out=None):
    """int8 levels [B][H][W][C] -> [B][Ho][Wo][C]."""
    return _pool_levels(lib().qnn_maxpool_levels_i8, _I8, 1, levels, k, stride, pad, ceil_mode, out)


def qnn_fp4_row_bytes(n):
    return int(lib().qnn_fp4_row_bytes(int(n)))


def qnn_plane_sum_fp4(planes, n, levels=None):
    """planes [bits][rows][nw], bits <= 2 -> fp4 levels, two per byte, uint8 [rows][qnn_fp4_row_bytes(n)]."""
    bits, rows, _ = _w_planes("planes", planes, n)
    levels = _out("levels", levels, torch.uint8, (rows, qnn_fp4_row_bytes(n)), planes)
    _check(lib().qnn_plane_sum_fp4(_ptr(planes), bits, rows, n, _ptr(levels), _stream()))
    return levels


def qnn_level_gemm_fp4(a_levels, w_levels, n, want_acc=True, scale=None, acc=None, out=None):
    """fp4 MFMA GEMM on levels as written by qnn_plane_sum_fp4 -> (acc int32 or None, out fp32 or None)."""
    return _level_gemm(lib().qnn_level_gemm_fp4, qnn_fp4_row_bytes(n), _U8, a_levels, w_levels, n, want_acc, scale,
                       acc, out)


def qnn_encode_levels_i8(src, clip, bits, levels=None):
    """src: CUDA fp32 / bf16 tensor, contiguous -> int8 levels of the same shape."""
    _arg("src", src, _VALUES)
    levels = _out("levels", levels, torch.int8, src.shape, src)
    _check(lib().qnn_encode_levels_i8(_ptr(src), _DTYPES[src.dtype], src.numel(), float(clip), int(bits),
                                      _ptr(levels), _stream()))
    return levels


def _block_epilogue(bias, res_q, res_bits, res_scale, res_f32, relu=False):
    return qnn_block_epilogue(_ptr(bias), _ptr(res_q), int(res_bits), float(res_scale), _ptr(res_f32), int(bool(relu)))


def _conv_out_shape(H, W, kh, kw, stride, pad, dilation=1):
    if stride < 1 or dilation < 1:
        raise ValueError("stride and dilation must be positive")
    return (H + 2 * pad - dilation * (kh - 1) - 1) // stride + 1, (W + 2 * pad - dilation * (kw - 1) - 1) // stride + 1


def _level_conv(entry, epi_args, dtypes, per_byte, a_levels, w_levels, stride, pad, a_bits, w_bits, scale, want_acc,
                want_out, next_clip, next_bits, acc, out, next_levels, dilation=None):
    """Shared by the int8 (per_byte = 1) and fp4 (per_byte = 2 channels per byte) level convolutions."""
    _arg("a_levels", a_levels, dtypes)
    _arg("w_levels", w_levels, dtypes)
    if a_levels.dim() != 4 or w_levels.dim() != 4 or a_levels.shape[3] != w_levels.shape[3]:
        raise ValueError("level tensors must be [B][H][W][C] and [Cout][kh][kw][C] with equal C, got %s and %s"
                         % (tuple(a_levels.shape), tuple(w_levels.shape)))
    B, H, W, cb = (int(e) for e in a_levels.shape)
    cout, kh, kw, _ = (int(e) for e in w_levels.shape)
    ho, wo = _conv_out_shape(H, W, kh, kw, stride, pad, 1 if dilation is None else dilation)
    _arg("scale", scale, _F32, shape=(cout,), optional=True)
    d = qnn_conv_desc(B, H, W, per_byte * cb, cout, kh, kw, stride, pad, a_bits, w_bits)
    acc = _out("acc", acc, torch.int32, (B, ho, wo, cout), a_levels, want_acc)
    out = _out("out", out, torch.float32, (B, ho, wo, cout), a_levels, want_out)
    next_levels = _out("next_levels", next_levels, a_levels.dtype, (B, ho, wo, cout // per_byte), a_levels,
                       next_clip is not None)
    epi = None
    if epi_args is not None:
        bias, res_levels, res_bits, res_scale, res_f32, relu = epi_args
        _arg("bias", bias, _F32, shape=(cout,), optional=True)
        _arg("res_levels", res_levels, dtypes, numel=B * ho * wo * (cout // per_byte), optional=True)
        _arg("res_f32", res_f32, _F32, numel=B * ho * wo * cout, optional=True)
        epi = _block_epilogue(bias, res_levels, res_bits, res_scale, res_f32, relu)
    head = (ctypes.byref(d),) + (() if dilation is None else (int(dilation),)) + (_ptr(a_levels), _ptr(w_levels), _ptr(scale))
    tail = (_ptr(acc), _ptr(out), _ptr(next_levels), float(next_clip) if next_clip is not None else 0.0,
            int(next_bits), _stream())
    _check(entry(*head, *tail) if epi is None else entry(*head, ctypes.byref(epi), *tail))
    return acc, out, next_levels


def qnn_level_conv2d_i8(a_levels, w_levels, stride, pad, a_bits, w_bits, scale=None, want_acc=True,
                        want_out=False, next_clip=None, next_bits=0, acc=None, out=None, next_levels=None):
    """a_levels int8 [B][H][W][Cin], w_levels int8 [Cout][kh][kw][Cin].  Returns (acc, out, next_levels);
    entries not requested are None."""
    return _level_conv(lib().qnn_level_conv2d_i8, None, _I8, 1, a_levels, w_levels, stride, pad, a_bits, w_bits, scale,
                       want_acc, want_out, next_clip, next_bits, acc, out, next_levels)


def qnn_level_conv2d_dilated_i8(a_levels, w_levels, stride, pad, dilation, a_bits, w_bits, scale=None, want_acc=True,
                                want_out=False, next_clip=None, next_bits=0, acc=None, out=None, next_levels=None):
    """qnn_level_conv2d_i8 with the taps `dilation` pixels apart."""
    return _level_conv(lib().qnn_level_conv2d_dilated_i8, None, _I8, 1, a_levels, w_levels, stride, pad, a_bits, w_bits,
                       scale, want_acc, want_out, next_clip, next_bits, acc, out, next_levels, dilation=dilation)


def qnn_level_conv2d_dilated_fp4(a_levels, w_levels, stride, pad, dilation, a_bits, w_bits, scale=None, want_acc=True,
                                 want_out=False, next_clip=None, next_bits=0, acc=None, out=None, next_levels=None):
    """qnn_level_conv2d_fp4 with the taps `dilation` pixels apart."""
    return _level_conv(lib().qnn_level_conv2d_dilated_fp4, None, _U8, 2, a_levels, w_levels, stride, pad, a_bits, w_bits,
                       scale, want_acc, want_out, next_clip, next_bits, acc, out, next_levels, dilation=dilation)


def qnn_level_conv2d_block_i8(a_levels, w_levels, stride, pad, a_bits, w_bits, scale, bias=None, res_levels=None,
                              res_bits=0, res_scale=0.0, res_f32=None, want_acc=True, want_out=False,
                              next_clip=None, next_bits=0, acc=None, out=None, next_levels=None, relu=False):
    """qnn_level_conv2d_i8 with the residual-block terms: bias fp32 [Cout], res_levels int8 [B][Ho][Wo][Cout]
    with its factor res_scale, res_f32 fp32 [B][Ho][Wo][Cout], relu (max(y, 0) after them)."""
    return _level_conv(lib().qnn_level_conv2d_block_i8, (bias, res_levels, res_bits, res_scale, res_f32, relu), _I8, 1,
                       a_levels, w_levels, stride, pad, a_bits, w_bits, scale, want_acc, want_out, next_clip, next_bits,
                       acc, out, next_levels)


def _conv_w_planes(t, cin):
    _arg("w_planes", t, _PLANES)
    if t.dim() != 5 or t.shape[4] != (cin + 31) // 32:
        raise ValueError("w_planes: expected [w_bits][Cout][kh][kw][%d], got shape %s" % ((cin + 31) // 32, tuple(t.shape)))
    return tuple(int(e) for e in t.shape)


def _act_planes(name, t, B, H, W, cin):
    _arg(name, t, _PLANES)
    bits, cw = int(t.shape[0]), (cin + 31) // 32
    if t.numel() != bits * B * H * W * cw:
        raise ValueError("%s: %d words, expected [%d][%d*%d*%d][%d]" % (name, t.numel(), bits, B, H, W, cw))
    return bits


def qnn_deconv_pack_weights(w_planes, cin, stride, phase_planes=None):
    """w_planes [w_bits][Cout][kh][kw][cw] -> the phase-ordered sub-kernel planes qnn_deconv2d reads (1-D int32)."""
    w_bits, cout, kh, kw, _ = _conv_w_planes(w_planes, cin)
    words = lib().qnn_deconv_phase_words(w_bits, cout, kh, kw, cin, stride)
    if words < 0:
        raise QnnError(QNN_ERR_INVALID_ARG, "qnn_deconv_phase_words: bad geometry")
    if phase_planes is None:
        phase_planes = torch.zeros((words,), dtype=torch.int32, device=w_planes.device)
    else:
        _arg("phase_planes", phase_planes, _PLANES)
        if phase_planes.numel() < words:
            raise ValueError("phase_planes: %d words, %d are needed" % (phase_planes.numel(), words))
    _check(lib().qnn_deconv_pack_weights(_ptr(w_planes), w_bits, cout, kh, kw, cin, stride, _ptr(phase_planes), _stream()))
    return phase_planes


def qnn_deconv2d(a_planes, phase_planes, shape, cin, cout, kh, kw, stride, pad, w_bits, scale=None, bias=None,
                 want_acc=True, want_out=False, next_clip=None, next_bits=0, acc=None, out=None, next_planes=None):
    """Transposed convolution of a_planes [a_bits][B*H*W][cw], shape = (B, H, W), with weights from
    qnn_deconv_pack_weights.  Returns (acc, out, next_planes) on the [B][Ho][Wo][Cout] output."""
    B, H, W = shape
    a_bits = _act_planes("a_planes", a_planes, B, H, W, cin)
    words = lib().qnn_deconv_phase_words(w_bits, cout, kh, kw, cin, stride)
    _arg("phase_planes", phase_planes, _PLANES)
    if words >= 0 and phase_planes.numel() < words:
        raise ValueError("phase_planes: %d words, %d are needed" % (phase_planes.numel(), words))
    ho, wo = (H - 1) * stride - 2 * pad + kh, (W - 1) * stride - 2 * pad + kw
    _arg("scale", scale, _F32, shape=(cout,), optional=True)
    _arg("bias", bias, _F32, shape=(cout,), optional=True)
    d = qnn_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad, a_bits, w_bits)
    acc = _out("acc", acc, torch.int32, (B, ho, wo, cout), a_planes, want_acc)
    out = _out("out", out, torch.float32, (B, ho, wo, cout), a_planes, want_out)
    next_planes = _out("next_planes", next_planes, torch.int32, (next_bits, B * ho * wo, (cout + 31) // 32), a_planes,
                       next_clip is not None)
    _check(lib().qnn_deconv2d(ctypes.byref(d), _ptr(a_planes), _ptr(phase_planes), _ptr(scale), _ptr(bias), _ptr(acc),
                              _ptr(out), _ptr(next_planes), float(next_clip) if next_clip is not None else 0.0,
                              int(next_bits), _stream()))
    return acc, out, next_planes


def qnn_quantize_ste_backward(x, grad_q, clip, grad_x=None):
    """x, grad_q fp32 of one shape -> grad_x fp32 (straight-through gradient of the ladder behind the range limit)."""
    _arg("x", x, _F32)
    _arg("grad_q", grad_q, _F32, shape=x.shape)
    grad_x = _out("grad_x", grad_x, torch.float32, x.shape, x)
    _check(lib().qnn_quantize_ste_backward(_ptr(x), _ptr(grad_q), x.numel(), float(clip), _ptr(grad_x), _stream()))
    return grad_x


def qnn_encoder_backward(x, grad_planes, clip, grad_x=None):
    """x fp32 [...], grad_planes fp32 [bits][...] -> grad_x fp32 (surrogate gradient of the encoder)."""
    _arg("x", x, _F32)
    _arg("grad_planes", grad_planes, _F32)
    if grad_planes.dim() < 1 or tuple(grad_planes.shape[1:]) != tuple(x.shape):
        raise ValueError("grad_planes: shape %s, expected [bits] + %s" % (tuple(grad_planes.shape), tuple(x.shape)))
    bits = int(grad_planes.shape[0])
    grad_x = _out("grad_x", grad_x, torch.float32, x.shape, x)
    _check(lib().qnn_encoder_backward(_ptr(x), _ptr(grad_planes), x.numel(), float(clip), bits, _ptr(grad_x), _stream()))
    return grad_x


def qnn_encode_levels_fp4(src, clip, bits, levels=None):
    """fp32 / bf16 [..., C] (C even) -> fp4 levels uint8 [..., C / 2], two channels per byte."""
    _arg("src", src, _VALUES)
    if src.dim() < 1 or src.shape[-1] % 2:
        raise ValueError("src: the last dimension must be even, got shape %s" % (tuple(src.shape),))
    levels = _out("levels", levels, torch.uint8, tuple(src.shape[:-1]) + (src.shape[-1] // 2,), src)
    _check(lib().qnn_encode_levels_fp4(_ptr(src), _DTYPES[src.dtype], src.numel(), float(clip), int(bits), _ptr(levels),
                                       _stream()))
    return levels


def qnn_levels_to_fp4(levels, out=None):
    """int8 levels [..., C] (C even, |level| <= 3) -> fp4 levels uint8 [..., C / 2]."""
    _arg("levels", levels, _I8)
    if levels.dim() < 1 or levels.shape[-1] % 2:
        raise ValueError("levels: the last dimension must be even, got shape %s" % (tuple(levels.shape),))
    out = _out("out", out, torch.uint8, tuple(levels.shape[:-1]) + (levels.shape[-1] // 2,), levels)
    _check(lib().qnn_levels_to_fp4(_ptr(levels), levels.numel(), _ptr(out), _stream()))
    return out


def qnn_level_conv2d_fp4(a_levels, w_levels, stride, pad, a_bits, w_bits, scale=None, want_acc=True, want_out=False,
                         next_clip=None, next_bits=0, acc=None, out=None, next_levels=None):
    """a_levels uint8 [B][H][W][Cin/2], w_levels uint8 [Cout][kh][kw][Cin/2] (fp4, two channels per byte).
    Returns (acc, out, next_levels [B][Ho][Wo][Cout/2]); entries not requested are None."""
    return _level_conv(lib().qnn_level_conv2d_fp4, None, _U8, 2, a_levels, w_levels, stride, pad, a_bits, w_bits, scale,
                       want_acc, want_out, next_clip, next_bits, acc, out, next_levels)


def qnn_level_deconv_flip_weights(w_levels, flipped=None):
    """w_levels int8 [Cout][kh][kw][Cin] or uint8 fp4 [Cout][kh][kw][Cin/2] -> the same tensor with the taps in
    flipped order, as qnn_level_deconv2d_i8 / _fp4 read it."""
    _arg("w_levels", w_levels, (torch.int8, torch.uint8))
    if w_levels.dim() != 4:
        raise ValueError("w_levels must be [Cout][kh][kw][C], got %s" % (tuple(w_levels.shape),))
    cout, kh, kw, cb = (int(e) for e in w_levels.shape)
    flipped = _out("flipped", flipped, w_levels.dtype, (cout, kh, kw, cb), w_levels, True)
    _check(lib().qnn_level_deconv_flip_weights(_ptr(w_levels), cout, kh, kw, cb, _ptr(flipped), _stream()))
    return flipped


def _level_deconv(entry, dtypes, per_byte, a_levels, flipped_w, stride, pad, a_bits, w_bits, scale, bias, want_acc, want_out,
                  next_clip, next_bits, acc, out, next_levels, workspace):
    _arg("a_levels", a_levels, dtypes)
    _arg("flipped_w", flipped_w, dtypes)
    if a_levels.dim() != 4 or flipped_w.dim() != 4 or a_levels.shape[3] != flipped_w.shape[3]:
        raise ValueError("level tensors must be [B][H][W][C] and [Cout][kh][kw][C] with equal C, got %s and %s"
                         % (tuple(a_levels.shape), tuple(flipped_w.shape)))
    B, H, W, cb = (int(e) for e in a_levels.shape)
    cout, kh, kw, _ = (int(e) for e in flipped_w.shape)
    ho, wo = (H - 1) * stride - 2 * pad + kh, (W - 1) * stride - 2 * pad + kw
    if ho < 1 or wo < 1:
        raise ValueError("transposed convolution with an empty output")
    d = qnn_conv_desc(B, H, W, per_byte * cb, cout, kh, kw, stride, pad, a_bits, w_bits)
    need = lib().qnn_level_deconv_workspace_bytes(ctypes.byref(d), int(per_byte == 2))
    if need < 0:
        raise QnnError(QNN_ERR_UNSUPPORTED, lib().qnn_last_error().decode())
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=a_levels.device)
    else:
        _arg("workspace", workspace, _U8)
        if workspace.numel() < need:
            raise ValueError("workspace: %d bytes, %d are needed" % (workspace.numel(), need))
    _arg("scale", scale, _F32, shape=(cout,), optional=True)
    _arg("bias", bias, _F32, shape=(cout,), optional=True)
    acc = _out("acc", acc, torch.int32, (B, ho, wo, cout), a_levels, want_acc)
    out = _out("out", out, torch.float32, (B, ho, wo, cout), a_levels, want_out)
    next_levels = _out("next_levels", next_levels, a_levels.dtype, (B, ho, wo, cout // per_byte), a_levels,
                       next_clip is not None)
    _check(entry(ctypes.byref(d), _ptr(a_levels), _ptr(flipped_w), _ptr(workspace), _ptr(scale), _ptr(bias), _ptr(acc),
                 _ptr(out), _ptr(next_levels), float(next_clip) if next_clip is not None else 0.0, int(next_bits), _stream()))
    return acc, out, next_levels


def qnn_level_deconv2d_i8(a_levels, flipped_w, stride, pad, a_bits, w_bits, scale=None, bias=None, want_acc=True,
                          want_out=False, next_clip=None, next_bits=0, acc=None, out=None, next_levels=None, workspace=None):
    """Transposed convolution on int8 levels: a_levels [B][H][W][Cin], flipped_w from qnn_level_deconv_flip_weights.
    workspace: uint8 tensor of qnn_level_deconv_workspace_bytes bytes (made here when None).  Returns (acc, out,
    next_levels) on the [B][Ho][Wo][Cout] output."""
    return _level_deconv(lib().qnn_level_deconv2d_i8, _I8, 1, a_levels, flipped_w, stride, pad, a_bits, w_bits, scale, bias,
                         want_acc, want_out, next_clip, next_bits, acc, out, next_levels, workspace)


def qnn_level_deconv2d_fp4(a_levels, flipped_w, stride, pad, a_bits, w_bits, scale=None, bias=None, want_acc=True,
                           want_out=False, next_clip=None, next_bits=0, acc=None, out=None, next_levels=None, workspace=None):
    """qnn_level_deconv2d_i8 on fp4 levels, two channels per byte (1- and 2-bit codes)."""
    return _level_deconv(lib().qnn_level_deconv2d_fp4, _U8, 2, a_levels, flipped_w, stride, pad, a_bits, w_bits, scale, bias,
                         want_acc, want_out, next_clip, next_bits, acc, out, next_levels, workspace)


def qnn_level_conv2d_block_fp4(a_levels, w_levels, stride, pad, a_bits, w_bits, scale, bias=None, res_levels=None,
                               res_bits=0, res_scale=0.0, res_f32=None, want_acc=True, want_out=False,
                               next_clip=None, next_bits=0, acc=None, out=None, next_levels=None, relu=False):
    """qnn_level_conv2d_fp4 with the residual-block terms; res_levels uint8 fp4 [B][Ho][Wo][Cout/2]."""
    return _level_conv(lib().qnn_level_conv2d_block_fp4, (bias, res_levels, res_bits, res_scale, res_f32, relu), _U8, 2,
                       a_levels, w_levels, stride, pad, a_bits, w_bits, scale, want_acc, want_out, next_clip, next_bits,
                       acc, out, next_levels)


def qnn_maxpool_levels_fp4(levels, k, stride, pad=0, ceil_mode=False, out=None):
    """levels uint8 [B][H][W][C/2] (fp4) -> pooled uint8 [B][Ho][Wo][C/2]."""
    return _pool_levels(lib().qnn_maxpool_levels_fp4, _U8, 2, levels, k, stride, pad, ceil_mode, out)


def _dense_conv(entry, x, w, stride, pad, scale, shift, relu, want_out, out, quant_name, quant_dtype, quant_shape,
                quant, want_quant, next_clip, next_bits):
    _arg("x", x, _F32)
    _arg("w", w, _F32)
    if x.dim() != 4 or w.dim() != 4 or x.shape[3] != w.shape[3]:
        raise ValueError("expected x [B][H][W][Cin] and w [Cout][kh][kw][Cin], got %s and %s"
                         % (tuple(x.shape), tuple(w.shape)))
    B, H, W, cin = (int(e) for e in x.shape)
    cout, kh, kw, _ = (int(e) for e in w.shape)
    ho, wo = _conv_out_shape(H, W, kh, kw, stride, pad)
    ho, wo = max(ho, 0), max(wo, 0)
    _arg("scale", scale, _F32, shape=(cout,), optional=True)
    _arg("shift", shift, _F32, shape=(cout,), optional=True)
    out = _out("out", out, torch.float32, (B, ho, wo, cout), x, want_out)
    quant = _out(quant_name, quant, quant_dtype, quant_shape(B, ho, wo, cout), x, want_quant)
    d = qnn_dense_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad)
    _check(entry(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(scale), _ptr(shift), int(bool(relu)), _ptr(out), _ptr(quant),
                 float(next_clip or 0.0), int(next_bits), _stream()))
    return out, quant


def qnn_dense_conv2d_f32(x, w, stride, pad, scale=None, shift=None, relu=False, want_out=True, next_clip=None,
                         next_bits=0, out=None, next_planes=None):
    """x fp32 [B][H][W][Cin], w fp32 [Cout][kh][kw][Cin] -> (out fp32 [B][Ho][Wo][Cout] or None,
    next planes int32 [next_bits][B*Ho*Wo][ceil(Cout/32)] or None)."""
    return _dense_conv(lib().qnn_dense_conv2d_f32, x, w, stride, pad, scale, shift, relu, want_out, out, "next_planes",
                       torch.int32, lambda B, ho, wo, cout: (next_bits, B * ho * wo, (cout + 31) // 32), next_planes,
                       bool(next_bits), next_clip, next_bits)


def qnn_dense_conv2d_f32_levels(x, w, stride, pad, next_clip, next_bits, scale=None, shift=None, relu=False, want_out=False,
                                out=None, next_levels=None):
    """As qnn_dense_conv2d_f32 with the quantized output as int8 levels [B][Ho][Wo][Cout]: (out or None, levels)."""
    return _dense_conv(lib().qnn_dense_conv2d_f32_levels, x, w, stride, pad, scale, shift, relu, want_out, out,
                       "next_levels", torch.int8, lambda B, ho, wo, cout: (B, ho, wo, cout), next_levels, True, next_clip,
                       next_bits)


def qnn_global_avgpool_f32(x, out=None):
    """x fp32 [B][H][W][C] (or [B][hw][C]) -> fp32 [B][C]."""
    _arg("x", x, _F32)
    if x.dim() < 2:
        raise ValueError("x: expected [B][...][C]")
    B, C = int(x.shape[0]), int(x.shape[-1])
    hw = _prod(x.shape[1:-1])
    out = _out("out", out, torch.float32, (B, C), x)
    _check(lib().qnn_global_avgpool_f32(_ptr(x), B, hw, C, _ptr(out), _stream()))
    return out


def qnn_dense_fc_f32(x, w, bias=None, out=None):
    """x fp32 [rows][n], w fp32 [cols][n], bias fp32 [cols] or None -> fp32 [rows][cols]."""
    _arg("x", x, _F32)
    _arg("w", w, _F32)
    if x.dim() != 2 or w.dim() != 2 or x.shape[1] != w.shape[1]:
        raise ValueError("expected x [rows][n] and w [cols][n], got %s and %s" % (tuple(x.shape), tuple(w.shape)))
    rows, n = (int(e) for e in x.shape)
    cols = int(w.shape[0])
    _arg("bias", bias, _F32, shape=(cols,), optional=True)
    out = _out("out", out, torch.float32, (rows, cols), x)
    _check(lib().qnn_dense_fc_f32(_ptr(x), _ptr(w), _ptr(bias), rows, cols, n, _ptr(out), _stream()))
    return out


def qnn_dequant_scale(acc, scale, out=None):
    """acc int32 [..., cols], scale fp32 [cols] -> fp32 of acc's shape."""
    _arg("acc", acc, _I32)
    if acc.dim() < 1:
        raise ValueError("acc: expected [..., cols]")
    rows, cols = _prod(acc.shape[:-1]), int(acc.shape[-1])
    _arg("scale", scale, _F32, shape=(cols,))
    out = _out("out", out, torch.float32, acc.shape, acc)
    _check(lib().qnn_dequant_scale(_ptr(acc), _ptr(scale), rows, cols, _ptr(out), _stream()))
    return out


def _conv(entry, epi_args, a_planes, w_planes, shape, cin, stride, pad, scale, want_acc, want_out, next_clip, next_bits,
          acc, out, next_planes, dilation=None):
    B, H, W = shape
    w_bits, cout, kh, kw, _ = _conv_w_planes(w_planes, cin)
    a_bits = _act_planes("a_planes", a_planes, B, H, W, cin)
    ho, wo = _conv_out_shape(H, W, kh, kw, stride, pad, 1 if dilation is None else dilation)
    _arg("scale", scale, _F32, shape=(cout,), optional=True)
    d = qnn_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad, a_bits, w_bits)
    acc = _out("acc", acc, torch.int32, (B, ho, wo, cout), a_planes, want_acc)
    out = _out("out", out, torch.float32, (B, ho, wo, cout), a_planes, want_out)
    next_planes = _out("next_planes", next_planes, torch.int32, (next_bits, B * ho * wo, (cout + 31) // 32), a_planes,
                       next_clip is not None)
    epi = None
    if epi_args is not None:
        bias, res_planes, res_scale, res_f32, relu = epi_args
        _arg("bias", bias, _F32, shape=(cout,), optional=True)
        _arg("res_planes", res_planes, _PLANES, optional=True)
        res_bits = int(res_planes.shape[0]) if res_planes is not None else 0
        if res_planes is not None and res_planes.numel() != res_bits * B * ho * wo * ((cout + 31) // 32):
            raise ValueError("res_planes: %d words, expected [%d][%d][%d]"
                             % (res_planes.numel(), res_bits, B * ho * wo, (cout + 31) // 32))
        _arg("res_f32", res_f32, _F32, numel=B * ho * wo * cout, optional=True)
        epi = _block_epilogue(bias, res_planes, res_bits, res_scale, res_f32, relu)
    head = (ctypes.byref(d),) + (() if dilation is None else (int(dilation),)) + (_ptr(a_planes), _ptr(w_planes), _ptr(scale))
    tail = (_ptr(acc), _ptr(out), _ptr(next_planes), float(next_clip) if next_clip is not None else 0.0,
            int(next_bits), _stream())
    _check(entry(*head, *tail) if epi is None else entry(*head, ctypes.byref(epi), *tail))
    return acc, out, next_planes


def qnn_conv2d(a_planes, w_planes, shape, cin, stride, pad, scale=None, want_acc=True, want_out=False,
               next_clip=None, next_bits=0, acc=None, out=None, next_planes=None):
    """a_planes [a_bits][B*H*W][cw] for an NHWC tensor of shape=(B, H, W); w_planes
    [w_bits][Cout][kh][kw][cw].  Returns (acc, out, next_planes); entries not requested are None."""
    return _conv(lib().qnn_conv2d, None, a_planes, w_planes, shape, cin, stride, pad, scale, want_acc, want_out,
                 next_clip, next_bits, acc, out, next_planes)


def qnn_conv2d_dilated(a_planes, w_planes, shape, cin, stride, pad, dilation, scale=None, want_acc=True, want_out=False,
                       next_clip=None, next_bits=0, acc=None, out=None, next_planes=None):
    """qnn_conv2d with the taps `dilation` pixels apart."""
    return _conv(lib().qnn_conv2d_dilated, None, a_planes, w_planes, shape, cin, stride, pad, scale, want_acc, want_out,
                 next_clip, next_bits, acc, out, next_planes, dilation=dilation)


def qnn_conv2d_block(a_planes, w_planes, shape, cin, stride, pad, scale, bias=None, res_planes=None, res_scale=0.0,
                     res_f32=None, want_acc=True, want_out=False, next_clip=None, next_bits=0, acc=None, out=None,
                     next_planes=None, relu=False):
    """qnn_conv2d with the residual-block terms: bias fp32 [Cout], res_planes [res_bits][B*Ho*Wo][ceil(Cout/32)]
    with its factor res_scale, res_f32 fp32 [B][Ho][Wo][Cout], relu (max(y, 0) after them)."""
    return _conv(lib().qnn_conv2d_block, (bias, res_planes, res_scale, res_f32, relu), a_planes, w_planes, shape, cin,
                 stride, pad, scale, want_acc, want_out, next_clip, next_bits, acc, out, next_planes)


def qnn_conv2d_chain_static_max_outputs():
    return int(lib().qnn_conv2d_chain_static_max_outputs())


def qnn_conv2d_chain_static(a_planes, w_planes, shape, cin, stride, pad, scale, next_clip, next_bits, next_planes=None):
    """qnn_conv2d from planes to the next layer's planes with no acc / out buffer at any bit width (the running sum
    of wide bit widths lives in the library's own fixed device array; the call allocates nothing when next_planes
    is passed in).  Returns next_planes [next_bits][B*Ho*Wo][ceil(Cout/32)]."""
    B, H, W = shape
    w_bits, cout, kh, kw, _ = _conv_w_planes(w_planes, cin)
    a_bits = _act_planes("a_planes", a_planes, B, H, W, cin)
    ho, wo = _conv_out_shape(H, W, kh, kw, stride, pad)
    _arg("scale", scale, _F32, shape=(cout,))
    d = qnn_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad, a_bits, w_bits)
    next_planes = _out("next_planes", next_planes, torch.int32, (next_bits, B * ho * wo, (cout + 31) // 32), a_planes)
    _check(lib().qnn_conv2d_chain_static(ctypes.byref(d), _ptr(a_planes), _ptr(w_planes), _ptr(scale), _ptr(next_planes),
                                         float(next_clip), int(next_bits), _stream()))
    return next_planes
