"""Seeded synthetic inputs for the five benchmark / parity configurations.

Shared by the CPU oracle's tests and the GPU library's tests and benchmark, so both
sides see identical tensors.  This module holds no arithmetic of the method beyond
naming the level set (odd integers in [-(2^b - 1), 2^b - 1], Eq. 10 of the paper):
it only draws random numbers and names shapes.

The paper evaluates on CIFAR-10, ImageNet and VOC; none of those (nor trained
weights) are used here.  The binary-product path is data independent in time, so
tensors with the networks' layer shapes and the stated value distributions stand in.

Seeds: numpy Generator(PCG64(190513389 + 1000 * config_index + tensor_index)).
"""
import numpy as np

BASE_SEED = 190513389


def rng(config_index, tensor_index):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config_index + tensor_index))


def odd_levels(gen, shape, bits, dtype=np.int8):
    """Uniform draw over the 2^bits odd levels {-(2^b-1), ..., -1, 1, ..., 2^b-1}."""
    top = (1 << bits) - 1
    u = gen.integers(0, top + 1, size=shape, dtype=np.int64)
    return (2 * u - top).astype(dtype)


def channel_scales(gen, cols, lo=0.01, hi=0.1):
    return gen.uniform(lo, hi, size=cols).astype(np.float32)


# --------------------------------------------------------------------------- config 1
def fc_2x2(config_index=0):
    """Single FC layer, 2-bit weights and activations: A [64][512], W [256][512]."""
    a = odd_levels(rng(config_index, 0), (64, 512), 2)
    w = odd_levels(rng(config_index, 1), (256, 512), 2)
    s = channel_scales(rng(config_index, 2), 256)
    return {"a": a, "w": w, "scale": s, "a_bits": 2, "w_bits": 2}


# --------------------------------------------------------------------------- config 2
def gemm_square(w_bits, a_bits, size=4096, config_index=1):
    """Square binary-decomposed GEMM operands: A [size][size], W [size][size] levels."""
    a = odd_levels(rng(config_index, 10 * a_bits + 0), (size, size), a_bits)
    w = odd_levels(rng(config_index, 10 * w_bits + 1), (size, size), w_bits)
    s = channel_scales(rng(config_index, 2), size)
    return {"a": a, "w": w, "scale": s, "a_bits": a_bits, "w_bits": w_bits}


def gemm_float_activations(rows, n, config_index=1, tensor_index=5):
    """fp32 activations ~N(0,1) for the encode step of the GEMM workload."""
    return rng(config_index, tensor_index).standard_normal((rows, n), dtype=np.float32)


# --------------------------------------------------------------------------- config 3
def resnet_conv_2x2(batch=64, hw=56, cin=64, cout=64, config_index=2):
    """ResNet-18-shaped 3x3 conv, stride 1, pad 1; fp32 NHWC input ~N(0,1), clip = 3 sigma
    (sigma = float64 std of the generated tensor, rounded once to fp32)."""
    x = rng(config_index, 0).standard_normal((batch, hw, hw, cin), dtype=np.float32)
    w = odd_levels(rng(config_index, 1), (cout, 3, 3, cin), 2)
    s = channel_scales(rng(config_index, 2), cout)
    clip = float(np.float32(3.0 * np.std(x.astype(np.float64))))
    return {"x": x, "w": w, "scale": s, "clip": clip, "a_bits": 2, "w_bits": 2,
            "stride": 1, "pad": 1}


# --------------------------------------------------------------------------- configs 4, 5
def _uniform_level_variance(bits):
    # variance of a uniform draw over the odd levels of `bits` bits: (4^b - 1) / 3
    return (4.0 ** bits - 1.0) / 3.0


def _gaussian_level_variance(bits, clip_sigmas=3.0):
    # variance, in level units, of a unit-variance Gaussian put through a `bits`-bit ladder
    # that clips at clip_sigmas: slope^2 plus the rounding noise of a step of 2 levels
    top = (1 << bits) - 1
    return (top / clip_sigmas) ** 2 + 1.0 / 3.0


def _stack_layer(gen_w, gen_s, cin, cout, bits, stride, clip):
    w = odd_levels(gen_w, (cout, 3, 3, cin), bits)
    n = 9 * cin
    # keep the post-scale activations near unit variance so that a fixed clip of 3.0 keeps
    # exercising every level (and a little saturation) layer after layer
    g = gen_s.uniform(0.5, 1.5, size=cout)
    s = (g / np.sqrt(n * _uniform_level_variance(bits) * _gaussian_level_variance(bits)))
    return {"w": w, "scale": s.astype(np.float32), "clip": float(clip), "a_bits": bits,
            "w_bits": bits, "stride": stride, "pad": 1, "cin": cin, "cout": cout}


RESNET18_PLAN = (
    # (cin, cout, stride) for the 16 quantized 3x3 convs; the stem conv and the FC head are
    # unquantized in the source network and are not part of this workload.
    (64, 64, 1), (64, 64, 1), (64, 64, 1), (64, 64, 1),
    (64, 128, 2), (128, 128, 1), (128, 128, 1), (128, 128, 1),
    (128, 256, 2), (256, 256, 1), (256, 256, 1), (256, 256, 1),
    (256, 512, 2), (512, 512, 1), (512, 512, 1), (512, 512, 1),
)


def resnet18_stack(batch=256, hw=56, bits=3, config_index=3, plan=RESNET18_PLAN):
    """ResNet-18-shaped chain of quantized 3x3 convs; input at the stem's output shape."""
    x = rng(config_index, 0).standard_normal((batch, hw, hw, plan[0][0]), dtype=np.float32)
    layers = []
    for li, (cin, cout, stride) in enumerate(plan):
        layers.append(_stack_layer(rng(config_index, 10 + 2 * li), rng(config_index, 11 + 2 * li),
                                   cin, cout, bits, stride, 3.0))
    return {"x": x, "layers": layers}


VGG_SSD_PLAN = (
    # resolution groups of the VGG16-backbone detection stack: (hw, [(cin, cout), ...])
    (300, ((64, 64),)),
    (150, ((64, 128), (128, 128))),
    (75, ((128, 256), (256, 256), (256, 256))),
    (38, ((256, 512), (512, 512), (512, 512))),
    (19, ((512, 512), (512, 512), (512, 512))),
)


def vgg_ssd_stack(batch=32, bits=4, config_index=4, plan=VGG_SSD_PLAN):
    """Detection-style stack: per resolution group a fresh N(0,1) fp32 input (clip = 3 sigma)
    feeding a chain of 3x3 stride-1 convs (pooling between groups is not modelled)."""
    groups = []
    t = 0
    for gi, (hw, chans) in enumerate(plan):
        x = rng(config_index, 100 + gi).standard_normal((batch, hw, hw, chans[0][0]),
                                                        dtype=np.float32)
        clip0 = float(np.float32(3.0 * np.std(x.astype(np.float64))))
        layers = []
        for li, (cin, cout) in enumerate(chans):
            L = _stack_layer(rng(config_index, 10 + 2 * t), rng(config_index, 11 + 2 * t),
                             cin, cout, bits, 1, clip0 if li == 0 else 3.0)
            layers.append(L)
            t += 1
        groups.append({"x": x, "layers": layers})
    return groups


# --------------------------------------------------------------------------- detection network as one chain
def _graph_conv(ci, t, name, src, cin, cout, k, bits, stride, pad, head=False, dilation=1):
    """A convolution node: weights uniform over the odd levels, per-channel scale that keeps unit-variance inputs at
    unit variance (heads: raw box / class scores of unit variance), input quantizer clipping at 3.0."""
    gen_w, gen_s = rng(ci, 10 + 2 * t), rng(ci, 11 + 2 * t)
    n = k * k * cin
    g = gen_s.uniform(0.5, 1.5, size=cout)
    s = g / np.sqrt(n * _uniform_level_variance(bits) * _gaussian_level_variance(bits))
    return {"kind": "conv", "name": name, "src": src, "w": odd_levels(gen_w, (cout, k, k, cin), bits),
            "scale": s.astype(np.float32), "clip": 3.0, "a_bits": bits, "w_bits": bits, "k": k, "stride": stride,
            "pad": pad, "cin": cin, "cout": cout, "head": head, "dilation": dilation}


def _graph_pool(name, src, k, stride, pad=0, ceil_mode=False):
    return {"kind": "pool", "name": name, "src": src, "k": k, "stride": stride, "pad": pad, "ceil_mode": ceil_mode, "head": False}


def vgg_ssd_chained(batch=32, bits=4, image=300, config_index=8, heads=True):
    """The detection network of the benchmark's fifth configuration as ONE graph on one input tensor: the twelve
    3x3 convolutions of the VGG16 backbone from its second layer on, joined by 2x2 stride-2 max-pooling (ceil mode
    at 75 -> 38), then the layers an SSD-style detector puts on top: a 3x3 stride-1 pooling, a 3x3 and a 1x1
    convolution with 1024 channels, four pairs of 1x1 / 3x3 convolutions that take the map from 19x19 down to
    1x1 (two with stride 2, two without padding), and a 3x3 localisation and a 3x3 class-score convolution on each
    of the six maps the detector reads (4 or 6 boxes per position, 21 classes).  The 3x3 convolution to 1024 channels
    has its taps 6 pixels apart (padding 6), as in the published network.  Every quantizer clips at 3.0 except the
    first (3 sigma of the input); heads write fp32 scores and feed nothing.
    Returns {"x", "clip0", "bits", "nodes"}: nodes in execution order, each naming its source node ("input" first)."""
    ci = config_index
    x = rng(ci, 0).standard_normal((batch, image, image, 64), dtype=np.float32)
    clip0 = float(np.float32(3.0 * np.std(x.astype(np.float64))))
    nodes, t = [], 0

    def conv(name, src, cin, cout, k=3, stride=1, pad=1, head=False, dilation=1):
        nonlocal t
        nodes.append(_graph_conv(ci, t, name, src, cin, cout, k, bits, stride, pad, head, dilation))
        t += 1
        return name

    def pool(name, src, k=2, stride=2, pad=0, ceil_mode=False):
        nodes.append(_graph_pool(name, src, k, stride, pad, ceil_mode))
        return name

    cur = conv("conv1_2", "input", 64, 64)
    cur = pool("pool1", cur)
    cur = conv("conv2_1", cur, 64, 128)
    cur = conv("conv2_2", cur, 128, 128)
    cur = pool("pool2", cur)
    cur = conv("conv3_1", cur, 128, 256)
    cur = conv("conv3_2", cur, 256, 256)
    cur = conv("conv3_3", cur, 256, 256)
    cur = pool("pool3", cur, ceil_mode=True)
    cur = conv("conv4_1", cur, 256, 512)
    cur = conv("conv4_2", cur, 512, 512)
    f1 = cur = conv("conv4_3", cur, 512, 512)
    cur = pool("pool4", cur)
    cur = conv("conv5_1", cur, 512, 512)
    cur = conv("conv5_2", cur, 512, 512)
    cur = conv("conv5_3", cur, 512, 512)
    cur = pool("pool5", cur, k=3, stride=1, pad=1)
    cur = conv("conv6", cur, 512, 1024, pad=6, dilation=6)
    f2 = cur = conv("conv7", cur, 1024, 1024, k=1, pad=0)
    cur = conv("conv8_1", cur, 1024, 256, k=1, pad=0)
    f3 = cur = conv("conv8_2", cur, 256, 512, stride=2)
    cur = conv("conv9_1", cur, 512, 128, k=1, pad=0)
    f4 = cur = conv("conv9_2", cur, 128, 256, stride=2)
    cur = conv("conv10_1", cur, 256, 128, k=1, pad=0)
    f5 = cur = conv("conv10_2", cur, 128, 256, pad=0)
    cur = conv("conv11_1", cur, 256, 128, k=1, pad=0)
    f6 = cur = conv("conv11_2", cur, 128, 256, pad=0)
    if heads:
        for src, cin, boxes in ((f1, 512, 4), (f2, 1024, 6), (f3, 512, 6), (f4, 256, 6), (f5, 256, 4), (f6, 256, 4)):
            conv("loc_" + src, src, cin, 4 * boxes, head=True)
            conv("conf_" + src, src, cin, 21 * boxes, head=True)
    return {"x": x, "clip0": clip0, "bits": bits, "nodes": nodes}


# --------------------------------------------------------------------------- whole network
CIFAR_VGG_PLAN = (
    # The CIFAR-10 network of the paper's Table 3 (the BinaryConnect / BNN architecture it cites:
    # 2x128C3 - MP2 - 2x256C3 - MP2 - 2x512C3 - MP2 - 2x1024FC - 10), from its second layer on: the
    # first convolution reads the real-valued image and is not part of the quantized path.
    ("conv", 128, 128), ("pool",),
    ("conv", 128, 256), ("conv", 256, 256), ("pool",),
    ("conv", 256, 512), ("conv", 512, 512), ("pool",),
    ("fc", 4 * 4 * 512, 1024), ("fc", 1024, 1024), ("fc", 1024, 10),
)


def cifar_vgg_network(batch=8, bits=2, config_index=5, plan=CIFAR_VGG_PLAN):
    """Input at the first layer's output shape [batch][32][32][128] ~ N(0,1), clip = 3 sigma; every
    later quantizer clips at 3.0.  Ops: dicts with kind conv (as _stack_layer), pool (2x2 stride 2)
    or fc (w int8 levels [cout][n], scale fp32 [cout], clip of its input quantizer)."""
    x = rng(config_index, 0).standard_normal((batch, 32, 32, plan[0][1]), dtype=np.float32)
    clip0 = float(np.float32(3.0 * np.std(x.astype(np.float64))))
    ops, t, first = [], 0, True
    for op in plan:
        if op[0] == "pool":
            ops.append({"kind": "pool", "k": 2, "stride": 2})
            continue
        gw, gs = rng(config_index, 10 + 2 * t), rng(config_index, 11 + 2 * t)
        t += 1
        clip = clip0 if first else 3.0
        first = False
        if op[0] == "conv":
            L = _stack_layer(gw, gs, op[1], op[2], bits, 1, clip)
            L["kind"] = "conv"
        else:
            n, cout = op[1], op[2]
            g = gs.uniform(0.5, 1.5, size=cout)
            s = g / np.sqrt(n * _uniform_level_variance(bits) * _gaussian_level_variance(bits))
            L = {"kind": "fc", "w": odd_levels(gw, (cout, n), bits), "scale": s.astype(np.float32),
                 "clip": float(clip), "a_bits": bits, "w_bits": bits, "n": n, "cout": cout}
        ops.append(L)
    return {"x": x, "ops": ops}


# --------------------------------------------------------------------------- residual trunk
RESNET18_BLOCKS = (
    # (cin, cout, stride of the block's first convolution); a block whose shape changes takes its
    # shortcut through a 1x1 convolution of the same stride, the others add their own input
    (64, 64, 1), (64, 64, 1), (64, 128, 2), (128, 128, 1),
    (128, 256, 2), (256, 256, 1), (256, 512, 2), (512, 512, 1),
)


def _block_conv(ci, t, cin, cout, k, bits, stride, clip, gain):
    L = _stack_layer(rng(ci, 10 + 3 * t), rng(ci, 11 + 3 * t), cin, cout, bits, stride, clip)
    if k == 1:
        L["w"] = odd_levels(rng(ci, 10 + 3 * t), (cout, 1, 1, cin), bits)
        L["scale"] = (L["scale"] * 3.0).astype(np.float32)      # a ninth of the taps
        L["pad"] = 0
    L["scale"] = (L["scale"] * np.float32(gain)).astype(np.float32)
    L["bias"] = rng(ci, 12 + 3 * t).uniform(-0.2, 0.2, size=cout).astype(np.float32)
    return L


def resnet18_trunk(batch=256, hw=56, bits=3, config_index=6, plan=RESNET18_BLOCKS):
    """The residual trunk of ResNet-18 (8 two-convolution blocks, 16 3x3 convolutions and 3 1x1
    shortcut convolutions) on quantized layers, input at the stem's output shape.  Every convolution
    has a per-channel scale and shift (a folded batch-norm); the second convolution of a block and
    the shortcut each carry a gain of 0.7 so that their sum keeps unit variance block after block."""
    x = rng(config_index, 0).standard_normal((batch, hw, hw, plan[0][0]), dtype=np.float32)
    top = (1 << bits) - 1
    blocks, t = [], 0
    for cin, cout, stride in plan:
        blk = {"conv1": _block_conv(config_index, t, cin, cout, 3, bits, stride, 3.0, 1.0),
               "conv2": _block_conv(config_index, t + 1, cout, cout, 3, bits, 1, 3.0, 0.7),
               "down": None, "res_scale": float(np.float32(0.7 * 3.0 / top))}
        if stride != 1 or cin != cout:
            blk["down"] = _block_conv(config_index, t + 2, cin, cout, 1, bits, stride, 3.0, 0.7)
        t += 3
        blocks.append(blk)
    return {"x": x, "blocks": blocks}


def resnet18_ends(batch=256, image=224, classes=1000, config_index=7):
    """The unquantized ends of ResNet-18 around the trunk: the 7x7 stride-2 first convolution (3 -> 64
    channels, folded batch-norm scale and shift, ReLU) on an N(0,1) image batch, and the classifier
    (512 -> classes) behind the global average pooling.  Weights N(0, 1/fan_in): post-scale outputs of
    about unit variance, so the first quantizer's clip of 3 sees a realistic spread."""
    g = [rng(config_index, t) for t in range(6)]
    return {"image": g[0].standard_normal((batch, image, image, 3), dtype=np.float32),
            "stem_w": (g[1].standard_normal((64, 7, 7, 3), dtype=np.float32) / np.float32(np.sqrt(147.0))),
            "stem_scale": g[2].uniform(0.8, 1.2, size=64).astype(np.float32),
            "stem_shift": g[3].normal(0.0, 0.2, size=64).astype(np.float32),
            "fc_w": (g[4].standard_normal((classes, 512), dtype=np.float32) / np.float32(np.sqrt(512.0))),
            "fc_b": g[5].normal(0.0, 0.1, size=classes).astype(np.float32)}
