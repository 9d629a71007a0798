"""CPU oracle for the encoding-decomposition QNN hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy front for oracle/qnn_oracle.c plus the layer-chaining loop.  Only
tests/, the smoke check and the benchmark's cpu_baseline leg may import this package;
the GPU library never does and shares no code with it.

Every function cites the passage of the paper it follows; the C file's header lists
what pins each of them.  layer_graph composes quantize / conv2d / scale / maxpool over a node list; its pin (the
library's float64 convolution and pooling on the decoded real values, node by node, on a small instance of the
detection graph) is in tests/test_oracle_graph.py.  maxpool / pool_out_size are plain numpy here; their pins (the library
pooling routine on the same integers, commutation with the quantizer, brute force) are in
tests/test_oracle_pool.py.  block_epilogue / residual_trunk are numpy float32 here; their pins (the same
sums in float64, the library's batch normalisation, Table 2's real values as the shortcut, the library's
float64 convolution block by block) are in tests/test_oracle_block.py.  deconv2d is plain numpy; its pins
(the library's transposed convolution in float64, the adjoint identity with conv2d, brute force) are in
tests/test_oracle_deconv.py.  quantize_ste_backward /
encoder_backward are numpy float64; their pins (Eq. 12-13's printed values, finite differences of the sines,
the sines' signs against the quantizer's planes) are in tests/test_oracle_training.py.  dense_conv2d /
dense_layer / global_avgpool / dense_fc (the unquantized ends of a network) are numpy float64; their pins
(brute-force loops, the library's float64 convolution, shifted copies through one-hot kernels, tap counts
of all-ones tensors, the integer convolution on integer-valued inputs) are in tests/test_oracle_dense.py.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = ctypes.CDLL(path)
        i64, i32, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_float
        p = ctypes.c_void_p
        L.oracle_quantize16.argtypes = [p, i64, f32, i32, p, p]
        L.oracle_pack_planes.argtypes = [p, i64, i64, i32, p]
        L.oracle_unpack_planes.argtypes = [p, i64, i64, i32, p]
        L.oracle_gemm.argtypes = [p, p, i64, i64, i64, p]
        L.oracle_gemm8.argtypes = [p, p, i64, i64, i64, p]
        L.oracle_gemm8_one.argtypes = [p, p, i64]
        L.oracle_gemm8_one.restype = ctypes.c_int32
        L.oracle_conv2d8.argtypes = [p, p, i64, i64, i64, i64, i64, i32, i32, i32, i32, p]
        L.oracle_conv2d8_dilated.argtypes = [p, p, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, p]
        L.oracle_scale.argtypes = [p, p, i64, i64, p]
        L.oracle_xnor_bitcount_dot.argtypes = [p, p, i64]
        L.oracle_xnor_bitcount_dot.restype = ctypes.c_int32
        L.oracle_multibranch_gemm.argtypes = [p, i32, p, i32, i64, i64, i64, p, p]
        L.oracle_num_threads.restype = ctypes.c_int
        _LIB = L
    return _LIB


def num_threads():
    """Threads the row-parallel oracle loops use (reported with the CPU baseline)."""
    return int(lib().oracle_num_threads())


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s failed with code %d" % (what, rc))


def quantize(x, clip, bits):
    """Range limit + linear quantizer (Table 1 HTanh, Eq. 15, Eq. 10).

    x: float32 array of any shape.  Returns (levels int16, codes uint8), same shape.
    level = (2^bits - 1) * q_bits(HTanh(x / clip)), an odd integer.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    level = np.empty(x.shape, dtype=np.int16)
    code = np.empty(x.shape, dtype=np.uint8)
    _check(lib().oracle_quantize16(_ptr(x), x.size, float(np.float32(clip)), int(bits),
                                   _ptr(level), _ptr(code)), "quantize")
    return level, code


def pack_planes(levels, bits):
    """Levels [rows][n] -> bit-planes [bits][rows][ceil(n/32)] uint32 (Eq. 4-6, Eq. 10)."""
    lv = np.ascontiguousarray(levels, dtype=np.int16)
    assert lv.ndim == 2
    rows, n = lv.shape
    nw = (n + 31) // 32
    planes = np.zeros((bits, rows, nw), dtype=np.uint32)
    _check(lib().oracle_pack_planes(_ptr(lv), rows, n, int(bits), _ptr(planes)), "pack_planes")
    return planes


def unpack_planes(planes, n):
    """Decode bit-planes back to levels: v = sum_j 2^j c_j, c_j in {-1,+1} (Eq. 10)."""
    pl = np.ascontiguousarray(planes, dtype=np.uint32)
    bits, rows, nw = pl.shape
    assert nw == (n + 31) // 32
    level = np.empty((rows, n), dtype=np.int16)
    _check(lib().oracle_unpack_planes(_ptr(pl), rows, n, bits, _ptr(level)), "unpack_planes")
    return level


def gemm(a_levels, w_levels):
    """acc[r][c] = sum_t a[r][t] * w[c][t] on decoded levels (Eq. 1-2).  int32 out."""
    a = np.ascontiguousarray(a_levels)
    w = np.ascontiguousarray(w_levels)
    rows, n = a.shape
    cols, n2 = w.shape
    assert n == n2
    acc = np.empty((rows, cols), dtype=np.int32)
    if a.dtype == np.int8 and w.dtype == np.int8:
        _check(lib().oracle_gemm8(_ptr(a), _ptr(w), rows, cols, n, _ptr(acc)), "gemm8")
    else:
        a = np.ascontiguousarray(a, dtype=np.int16)
        w = np.ascontiguousarray(w, dtype=np.int16)
        _check(lib().oracle_gemm(_ptr(a), _ptr(w), rows, cols, n, _ptr(acc)), "gemm")
    return acc


def gemm_one(a_row, w_row):
    """One GEMM output (for sampled checks at sizes where the full loop is slow)."""
    a = np.ascontiguousarray(a_row, dtype=np.int8)
    w = np.ascontiguousarray(w_row, dtype=np.int8)
    assert a.shape == w.shape and a.ndim == 1
    return int(lib().oracle_gemm8_one(_ptr(a), _ptr(w), a.size))


def conv2d(a_levels, w_levels, stride, pad, dilation=1):
    """Zero-padded convolution on decoded levels.  a: [B][H][W][Cin] int8, w:
    [Cout][kh][kw][Cin] int8 -> int32 [B][Ho][Wo][Cout] (Section "Model Decomposition").
    dilation > 1: the taps are that many pixels apart (the dilated layer of the detection network)."""
    a = np.ascontiguousarray(a_levels, dtype=np.int8)
    w = np.ascontiguousarray(w_levels, dtype=np.int8)
    B, H, W, Cin = a.shape
    Cout, kh, kw, Cin2 = w.shape
    assert Cin == Cin2
    if dilation == 1:
        Ho = (H + 2 * pad - kh) // stride + 1
        Wo = (W + 2 * pad - kw) // stride + 1
        acc = np.empty((B, Ho, Wo, Cout), dtype=np.int32)
        _check(lib().oracle_conv2d8(_ptr(a), _ptr(w), B, H, W, Cin, Cout, kh, kw, stride, pad,
                                    _ptr(acc)), "conv2d")
        return acc
    Ho = (H + 2 * pad - dilation * (kh - 1) - 1) // stride + 1
    Wo = (W + 2 * pad - dilation * (kw - 1) - 1) // stride + 1
    assert Ho >= 1 and Wo >= 1
    acc = np.empty((B, Ho, Wo, Cout), dtype=np.int32)
    _check(lib().oracle_conv2d8_dilated(_ptr(a), _ptr(w), B, H, W, Cin, Cout, kh, kw, stride, pad, dilation,
                                        _ptr(acc)), "conv2d (dilated)")
    return acc


def scale(acc, scale_vec):
    """out = (float)acc * scale[c]: the decoder's scale factor (1/alpha^2 of Section
    "M-bit Encoding Functions", Eq. 18), one fp32 factor per output channel."""
    a = np.ascontiguousarray(acc, dtype=np.int32)
    s = np.ascontiguousarray(scale_vec, dtype=np.float32)
    cols = a.shape[-1]
    assert s.shape == (cols,)
    out = np.empty(a.shape, dtype=np.float32)
    _check(lib().oracle_scale(_ptr(a), _ptr(s), a.size // cols, cols, _ptr(out)), "scale")
    return out


def xnor_bitcount_dot(a_words, b_words, n):
    """Binary dot of two {-1,+1}^n bit-vectors: 2*bitcount(xnor) - n (self-test helper)."""
    a = np.ascontiguousarray(a_words, dtype=np.uint32)
    b = np.ascontiguousarray(b_words, dtype=np.uint32)
    return int(lib().oracle_xnor_bitcount_dot(_ptr(a), _ptr(b), n))


def multibranch_gemm(a_planes, w_planes, n, want_branches=False):
    """Literal M x K multi-branch binary product (Eq. 9 + Eq. 10, Fig. 1) on planes as
    written by pack_planes (self-test helper; the GEMM oracle is gemm())."""
    ap = np.ascontiguousarray(a_planes, dtype=np.uint32)
    wp = np.ascontiguousarray(w_planes, dtype=np.uint32)
    a_bits, rows, nw = ap.shape
    w_bits, cols, nw2 = wp.shape
    assert nw == nw2 == (n + 31) // 32
    acc = np.empty((rows, cols), dtype=np.int32)
    br = np.empty((rows, cols, w_bits, a_bits), dtype=np.int32) if want_branches else None
    _check(lib().oracle_multibranch_gemm(_ptr(ap), a_bits, _ptr(wp), w_bits, rows, cols, n,
                                         _ptr(acc), _ptr(br) if want_branches else None),
           "multibranch_gemm")
    return (acc, br) if want_branches else acc


def conv_stack(x, layers):
    """Chain of quantized convolutions (inference by multi-branch binary layers one after
    another: Introduction; Section "Quantized Networks Training").

    x: float32 [B][H][W][C].  layers: list of dicts with keys w (int8 levels
    [Cout][kh][kw][Cin]), scale (float32 [Cout]), clip (float), a_bits, stride, pad.
    Per layer: quantize(x, clip, a_bits) -> conv2d -> scale -> next x.
    Returns a list of per-layer dicts {levels, acc, out}.
    """
    trace = []
    cur = np.ascontiguousarray(x, dtype=np.float32)
    for L in layers:
        assert 1 <= L["a_bits"] <= 7, "int8 level path holds up to 7 bits"
        lv, _ = quantize(cur, L["clip"], L["a_bits"])
        acc = conv2d(lv.astype(np.int8), L["w"], L["stride"], L["pad"])
        out = scale(acc, L["scale"])
        trace.append({"levels": lv, "acc": acc, "out": out})
        cur = out
    return trace


def layer_graph(x, clip0, bits, nodes):
    """A network of quantized layers given as a list of nodes in execution order (the detection network of the
    experiments section is such a graph: a backbone whose maps feed both the next layer and the detector's heads).

    x: float32 [B][H][W][C], quantized once with (clip0, bits) (Table 1 range limit, Eq. 15); the result is node
    "input".  Every node names its source node:
      conv  levels(src) -> conv2d (zero padding; "dilation" if the node has one) -> scale -> out (float32); unless the node is a head, out is
            quantized with (clip, a_bits) and the levels are what its consumers read
      pool  max-pooling of the source's levels (taken on the codes: the quantizer is monotone)
    Returns {name: {"levels" (or None for heads), "acc", "out"}} with "input" included.
    """
    assert 1 <= bits <= 7, "int8 level path holds up to 7 bits"
    lv, _ = quantize(np.ascontiguousarray(x, dtype=np.float32), clip0, bits)
    values = {"input": {"levels": lv, "acc": None, "out": None}}
    for nd in nodes:
        src = values[nd["src"]]["levels"]
        assert src is not None, "a head's output feeds nothing"
        if nd["kind"] == "pool":
            values[nd["name"]] = {"levels": maxpool(src, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"]),
                                  "acc": None, "out": None}
            continue
        acc = conv2d(src.astype(np.int8), nd["w"], nd["stride"], nd["pad"], nd.get("dilation", 1))
        out = scale(acc, nd["scale"])
        lv = None
        if not nd["head"]:
            lv, _ = quantize(out, nd["clip"], nd["a_bits"])
        values[nd["name"]] = {"levels": lv, "acc": acc, "out": out}
    return values


def deconv2d(a_levels, w_levels, stride, pad):
    """Transposed convolution ("deconvolution", Section "Model Decomposition": deconvolution layers
    reduce to the same vector products) on decoded levels, written as its definition: every input
    pixel (i, j) adds a[b][i][j][:] . w[co][ky][kx][:] to output pixel (i stride + ky - pad,
    j stride + kx - pad); contributions that fall outside the output are dropped.
    a: [B][H][W][Cin], w: [Cout][kh][kw][Cin] -> int32 [B][Ho][Wo][Cout], Ho = (H - 1) stride - 2 pad + kh."""
    a = np.ascontiguousarray(a_levels).astype(np.int64)
    w = np.ascontiguousarray(w_levels).astype(np.int64)
    B, H, W, Cin = a.shape
    Cout, kh, kw, Cin2 = w.shape
    assert Cin == Cin2
    Ho, Wo = (H - 1) * stride - 2 * pad + kh, (W - 1) * stride - 2 * pad + kw
    assert Ho >= 1 and Wo >= 1
    full = np.zeros((B, (H - 1) * stride + kh, (W - 1) * stride + kw, Cout), dtype=np.int64)
    for ky in range(kh):
        for kx in range(kw):
            contrib = a @ w[:, ky, kx, :].T                       # [B][H][W][Cout]
            full[:, ky:ky + (H - 1) * stride + 1:stride, kx:kx + (W - 1) * stride + 1:stride, :] += contrib
    out = full[:, pad:pad + Ho, pad:pad + Wo, :]
    assert np.abs(out).max() < 2 ** 31
    return np.ascontiguousarray(out.astype(np.int32))


def block_epilogue(acc, scale_vec, bias=None, res_levels=None, res_scale=None, res_f32=None, relu=False):
    """What a residual block adds between the decoder's scale factor and the next quantizer (the
    ResNet-18 of the experiments section has shortcuts and batch normalisation; the derivation itself
    leaves the bias out): a per-channel shift -- a folded batch-norm -- and the shortcut term, either
    quantized levels times one real factor or an fp32 tensor.  fp32 throughout, one rounding per step,
    in this order:
        y = (float)acc * scale[c];  y = y + bias[c];  y = y + ((float)res_level * res_scale);
        y = y + res_f32;  y = max(y, 0) if relu -- the lower limit of HReLU (Table 1); the next quantizer's clip
        is the upper one, so that the encoder sees clamp(y / clip, 0, 1).
    numpy float32 array arithmetic is one IEEE single-precision operation per element per operator.
    """
    y = scale(acc, scale_vec)
    if bias is not None:
        b = np.ascontiguousarray(bias, dtype=np.float32)
        assert b.shape == (y.shape[-1],)
        y = y + b
    if res_levels is not None:
        lv = np.asarray(res_levels)
        assert lv.shape == y.shape
        y = y + lv.astype(np.float32) * np.float32(res_scale)
    if res_f32 is not None:
        r = np.asarray(res_f32)
        assert r.dtype == np.float32 and r.shape == y.shape
        y = y + r
    if relu:
        y = np.maximum(y, np.float32(0.0))
    assert y.dtype == np.float32
    return y


def residual_trunk(x, blocks):
    """Chain of two-convolution residual blocks (the ResNet-18 shape of the experiments section) on
    quantized layers.  x: float32 [B][H][W][C].  Each block: dict with conv1, conv2 and down (None or
    a 1x1 convolution), every convolution a dict with w (int8 levels), scale, bias (float32 [Cout]),
    stride, pad, clip (of the quantizer in front of it), a_bits.

        a  = quantize(x, conv1.clip)                      block input, shared by conv1 and the shortcut
        h  = epilogue(conv(a, conv1))                     scale + bias
        hq = quantize(h, conv2.clip)
        y  = epilogue(conv(hq, conv2), shortcut)          shortcut: a's levels times res_scale (identity
                                                          block) or the fp32 output of down(a)
    and y is the next block's x.  Returns per block {a, acc1, hq, acc2, accd, shortcut, y}.
    """
    trace = []
    cur = np.ascontiguousarray(x, dtype=np.float32)
    for blk in blocks:
        c1, c2, dn = blk["conv1"], blk["conv2"], blk["down"]
        assert 1 <= c1["a_bits"] <= 7 and 1 <= c2["a_bits"] <= 7
        a, _ = quantize(cur, c1["clip"], c1["a_bits"])
        acc1 = conv2d(a.astype(np.int8), c1["w"], c1["stride"], c1["pad"])
        h = block_epilogue(acc1, c1["scale"], c1["bias"])
        hq, _ = quantize(h, c2["clip"], c2["a_bits"])
        acc2 = conv2d(hq.astype(np.int8), c2["w"], c2["stride"], c2["pad"])
        if dn is None:
            accd, shortcut = None, None
            y = block_epilogue(acc2, c2["scale"], c2["bias"], res_levels=a, res_scale=blk["res_scale"])
        else:
            accd = conv2d(a.astype(np.int8), dn["w"], dn["stride"], dn["pad"])
            shortcut = block_epilogue(accd, dn["scale"], dn["bias"])
            y = block_epilogue(acc2, c2["scale"], c2["bias"], res_f32=shortcut)
        trace.append({"a": a, "acc1": acc1, "hq": hq, "acc2": acc2, "accd": accd, "shortcut": shortcut, "y": y})
        cur = y
    return trace


def _range_limited(x, clip):
    """t = x * (1 / clip) in fp32, as the quantizer forms it, and the mask of -1 <= t <= 1."""
    inv = np.float32(1.0) / np.float32(clip)
    t = np.ascontiguousarray(x, dtype=np.float32) * inv
    return t.astype(np.float64), (t >= -1.0) & (t <= 1.0), np.float64(inv)


def quantize_ste_backward(x, grad_q, clip):
    """Straight-through gradient of the hard ladder q_k behind the range limit (Section "Quantized
    Networks Training"; Table 1 HTanh): q_k(HTanh(x / clip)) is differentiated as if q_k were the
    identity, so the gradient passes with slope 1 / clip where -1 <= x / clip <= 1 and is 0 outside.
    With clip = 1 this is also the gradient of Binarize(x) = sign(HTanh(x)) (Eq. 14).  float64 out."""
    _, inside, inv = _range_limited(x, clip)
    g = np.asarray(grad_q, dtype=np.float64)
    return np.where(inside, g * inv, 0.0)


def encoder_backward(x, grad_planes, clip, bits):
    """Surrogate gradient of the M-bit encoder (Eq. 12-13 for M = 2).  Plane m of M (m = 1 lowest) is
    the sign of a sine: +sin(pi K t / 2^M) for m = M and -sin(pi K t / 2^m) below, K = 2^M - 1,
    t = HTanh(x / clip); its derivative is taken as that of the sine inside [-1, 1] and 0 outside:
        d plane_M / dt = +(pi K / 2^M) cos(pi K t / 2^M),  d plane_m / dt = -(pi K / 2^m) cos(pi K t / 2^m).
    grad_planes: [bits][...] gradients w.r.t. each plane (index m - 1).  Returns d loss / d x, float64."""
    t, inside, inv = _range_limited(x, clip)
    g = np.asarray(grad_planes, dtype=np.float64)
    assert g.shape == (bits,) + t.shape
    K = float((1 << bits) - 1)
    total = np.zeros(t.shape, dtype=np.float64)
    for m in range(1, bits + 1):
        coef = np.pi * K / float(1 << m)
        sign = 1.0 if m == bits else -1.0
        total += g[m - 1] * (sign * coef * np.cos(coef * t))
    return np.where(inside, total * inv, 0.0)


def pool_out_size(size, k, stride, pad, ceil_mode):
    """Output extent of a pooling window sweep: floor or ceil of (size + 2 pad - k) / stride, plus 1;
    in ceil mode a last window that would start beyond the image and its left padding is dropped."""
    span = size + 2 * pad - k
    if span < 0:
        raise ValueError("pooling window larger than the padded image")
    if ceil_mode:
        out = -(-span // stride) + 1
        if (out - 1) * stride >= size + pad:
            out -= 1
    else:
        out = span // stride + 1
    return out


def maxpool(levels, k, stride, pad=0, ceil_mode=False):
    """Max-pooling of a quantized activation tensor, taken on the decoded levels.

    The linear quantizer (Eq. 15 after the range limit of Table 1) is monotone non-decreasing, so the
    maximum over a window of the quantized values is the quantized maximum: pooling the levels (or,
    equally, the codes) is exact.  levels: integer [B][H][W][C].  Window elements outside the image
    (padding, ceil-mode overhang) are ignored.  Plain definition: for every window offset, an
    elementwise maximum of the shifted view.
    """
    a = np.asarray(levels)
    B, H, W, C = a.shape
    if pad * 2 > k:
        raise ValueError("pad must be at most half the window")
    ho = pool_out_size(H, k, stride, pad, ceil_mode)
    wo = pool_out_size(W, k, stride, pad, ceil_mode)
    lowest = np.iinfo(np.int32).min
    out = np.full((B, ho, wo, C), lowest, dtype=np.int32)
    for oy in range(ho):
        for ox in range(wo):
            for ky in range(k):
                for kx in range(k):
                    y, x = oy * stride - pad + ky, ox * stride - pad + kx
                    if 0 <= y < H and 0 <= x < W:
                        out[:, oy, ox, :] = np.maximum(out[:, oy, ox, :], a[:, y, x, :])
    if (out == lowest).any():
        raise ValueError("a pooling window holds no image element")
    return out.astype(a.dtype)


def dense_conv2d(x, w, stride, pad):
    """Unquantized convolution in float64, written as its definition: out[b][ho][wo][co] = sum over
    (ky, kx, ci) of x[b][ho stride + ky - pad][wo stride + kx - pad][ci] w[co][ky][kx][ci], taps outside
    the image contribute 0.  The networks of the experiments section keep their first and last layers
    unquantized (the ResNet-18 workload says so); this is the first one.
    x: [B][H][W][Cin], w: [Cout][kh][kw][Cin] -> float64 [B][Ho][Wo][Cout]."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    B, H, W, Cin = x.shape
    Cout, kh, kw, Cin2 = w.shape
    assert Cin == Cin2 and stride >= 1 and pad >= 0
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    assert Ho >= 1 and Wo >= 1
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin))
    xp[:, pad:pad + H, pad:pad + W, :] = x
    out = np.zeros((B, Ho, Wo, Cout))
    for ky in range(kh):
        for kx in range(kw):
            view = xp[:, ky:ky + (Ho - 1) * stride + 1:stride, kx:kx + (Wo - 1) * stride + 1:stride, :]
            out += view @ w[:, ky, kx, :].T
    return out


def dense_layer(x, w, stride, pad, scale_vec=None, shift=None, relu=False):
    """dense_conv2d, then per output channel y = conv * scale[c] + shift[c] (a folded batch normalisation)
    and optionally max(y, 0), all in float64; the absolute sum sum |x| |w| of every output comes back as
    well, since the float32 rounding error of any summation order is bounded by a multiple of it."""
    y = dense_conv2d(x, w, stride, pad)
    mag = dense_conv2d(np.abs(np.asarray(x, dtype=np.float64)), np.abs(np.asarray(w, dtype=np.float64)), stride, pad)
    if scale_vec is not None:
        sv = np.asarray(scale_vec, dtype=np.float64)
        y, mag = y * sv, mag * np.abs(sv)
    if shift is not None:
        sh = np.asarray(shift, dtype=np.float64)
        y, mag = y + sh, mag + np.abs(sh)
    if relu:
        y = np.maximum(y, 0.0)
    return y, mag


def global_avgpool(x):
    """Mean over the image positions of every channel, float64: [B][H][W][C] -> [B][C] (the pooling in
    front of ResNet-18's classifier)."""
    x = np.asarray(x, dtype=np.float64)
    B, H, W, C = x.shape
    total = np.zeros((B, C))
    for i in range(H):
        for j in range(W):
            total += x[:, i, j, :]
    return total / (H * W)


def dense_fc(x, w, bias=None):
    """Unquantized fully connected layer in float64: out[b][o] = sum_i x[b][i] w[o][i] + bias[o] (Eq. 1
    without quantization; the last layer of the ResNet-18 workload).  Also returns sum |x| |w| + |bias|."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    out, mag = x @ w.T, np.abs(x) @ np.abs(w).T
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        out, mag = out + b, mag + np.abs(b)
    return out, mag
