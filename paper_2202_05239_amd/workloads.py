"""Seeded synthetic workloads: operands and layer lists of the five benchmark configurations.

This module only *draws inputs* (numpy, PCG64) and writes down layer shapes; it holds
none of the fixed-point layer arithmetic and imports neither the GPU library nor the
CPU oracle, both of which consume what it produces.

Synthetic tensors stand in for ImageNet crops (224x224x3) and for trained weights:
shapes are those of the paper's models (ResNet18, ResNet50 with the stride on the 3x3
of the bottleneck, one MobileNetV2 inverted-residual block), value formats are the
paper's 8-bit fixed point (Eq. 2 unsigned 0..255, Eq. 9 signed -127..127) and the
per-layer fractional lengths are drawn from the seed inside the range the paper
reports for trained models (Table 3, Fig. 2b, Fig. 6: anything from 0 to 8 occurs).

Draw order for every configuration: fractional length of the input (if drawn), the
input tensor, then per layer in execution order FL_w, FL_y, W, bias (and, for the
ResNet-50 configuration, the clip draw).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 220205239


def seed_of(config_index: int) -> int:
    return BASE_SEED + 1000 * config_index


@dataclass
class LayerSpec:
    """One layer of a fixed-point network, or a single stand-alone layer call.

    op: 'conv' (dense conv / GEMM), 'dwconv', 'maxpool', 'gpool' (global sum pool).
    src / dst / res: tensor ids (0 = network input); res = -1 when there is no residual.
    *_type: 'u8', 's8' or 's32'.  clip_lo/clip_hi are in output LSBs (2^-fl_y).
    w: int8 [Cout][R][S][Cin] for 'conv', [R][S][C] for 'dwconv', None for pools.
    dst2 > 0 ('conv' only): a second output tensor holding the same result in the format
    fl_y2 / clip_lo2 / clip_hi2 / y2_type, for a sibling consumer with a private fractional
    length (paper Sec. 4.3).
    """
    op: str
    name: str = ""
    src: int = 0
    dst: int = 1
    res: int = -1
    Cin: int = 0
    Cout: int = 0
    R: int = 1
    S: int = 1
    stride: int = 1
    pad: int = 0
    fl_x: int = 0
    fl_w: int = 0
    fl_y: int = 0
    clip_lo: int = 0
    clip_hi: int = 255
    x_type: str = "u8"
    y_type: str = "u8"
    res_type: str = "u8"
    fl_res: int = 0
    w: Optional[np.ndarray] = None
    bias: Optional[np.ndarray] = None
    in_hw: Tuple[int, int] = (0, 0)
    out_hw: Tuple[int, int] = (0, 0)
    dst2: int = -1
    fl_y2: int = 0
    clip_lo2: int = 0
    clip_hi2: int = 255
    y2_type: str = "u8"

    @property
    def macs_per_image(self) -> int:
        P, Q = self.out_hw
        if self.op == "conv":
            return P * Q * self.Cout * self.R * self.S * self.Cin
        if self.op == "dwconv":
            return P * Q * self.Cout * self.R * self.S
        return 0


@dataclass
class Net:
    name: str
    in_hw: Tuple[int, int]
    in_c: int
    x_type: str
    fl_x: int
    layers: List[LayerSpec] = field(default_factory=list)

    @property
    def macs_per_image(self) -> int:
        return sum(L.macs_per_image for L in self.layers)


# ---------------------------------------------------------------------------------
# elementary draws
# ---------------------------------------------------------------------------------

def draw_weight(rng, shape, std, fl_w):
    """int8 weights: a normal draw with standard deviation `std`, written in 8-bit
    signed fixed point with fractional length fl_w (symmetric range -127..127)."""
    w = np.rint(rng.normal(0.0, std, size=shape) * 2.0 ** fl_w)
    return np.clip(w, -127, 127).astype(np.int8)


def draw_bias(rng, n, fl_acc, std=0.1):
    """int32 bias at the accumulator scale fl_acc = FL_x + FL_w."""
    return np.rint(rng.normal(0.0, std, size=n) * 2.0 ** fl_acc).astype(np.int32)


def draw_u8(rng, shape):
    return rng.integers(0, 256, size=shape, dtype=np.uint8)


def draw_s8_normal(rng, shape, fl):
    x = np.rint(rng.standard_normal(size=shape, dtype=np.float32) * np.float32(2.0 ** fl))
    return np.clip(x, -127, 127).astype(np.int8)


def _out(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


# ---------------------------------------------------------------------------------
# configuration 0: one GEMM (1x1-conv equivalent)
# ---------------------------------------------------------------------------------

def config0(seed=None):
    """M=256, K=64, N=64; uint8 activations FL 4, int8 weights FL 7, FL_y 4 (shift 7)."""
    rng = np.random.default_rng(seed_of(0) if seed is None else seed)
    M, K, N = 256, 64, 64
    x = draw_u8(rng, (M, K))
    L = LayerSpec(op="conv", name="gemm", Cin=K, Cout=N, fl_x=4, fl_w=7, fl_y=4,
                  clip_lo=0, clip_hi=255, x_type="u8", y_type="u8",
                  in_hw=(1, M), out_hw=(1, M))
    w = draw_weight(rng, (N, K), 0.05, 7)
    L.w = w.reshape(N, 1, 1, K)
    L.bias = draw_bias(rng, N, 4 + 7)
    return x, L


# ---------------------------------------------------------------------------------
# configuration 1: one ResNet-18-style 3x3 layer
# ---------------------------------------------------------------------------------

def config1(seed=None, batch=32):
    """NHWC batch x 56 x 56 x 64 -> 64, 3x3 stride 1 pad 1, FL_x 5, FL_w 8, FL_y 5,
    clip level 6.0 in output LSBs = 6.0 * 2^5 = 192."""
    rng = np.random.default_rng(seed_of(1) if seed is None else seed)
    x = draw_u8(rng, (batch, 56, 56, 64))
    L = LayerSpec(op="conv", name="conv3x3_56x56x64", Cin=64, Cout=64, R=3, S=3, stride=1, pad=1,
                  fl_x=5, fl_w=8, fl_y=5, clip_lo=0, clip_hi=192, x_type="u8", y_type="u8",
                  in_hw=(56, 56), out_hw=(56, 56))
    L.w = draw_weight(rng, (64, 3, 3, 64), float(np.sqrt(2.0 / 576.0)), 8)
    L.bias = draw_bias(rng, 64, 5 + 8)
    return x, L


# ---------------------------------------------------------------------------------
# configuration 2: MobileNetV2 inverted-residual block
# ---------------------------------------------------------------------------------

def config2(seed=None, batch=64, hw=56, c=24, expand=6, with_residual=False):
    """1x1 expand (uint8 out) -> 3x3 depthwise (uint8 out) -> 1x1 project (int8 out).

    The block input is the signed output of a previous projection.  Every fractional
    length is drawn uniformly from 3..8.  with_residual adds the block input as the
    residual operand of the projection (the identity shortcut of the block)."""
    rng = np.random.default_rng(seed_of(2) if seed is None else seed)
    fl_in = int(rng.integers(3, 9))
    x = draw_s8_normal(rng, (batch, hw, hw, c), fl_in)
    ce = c * expand
    net = Net(name="mbv2_block", in_hw=(hw, hw), in_c=c, x_type="s8", fl_x=fl_in)

    fl_w = int(rng.integers(3, 9)); fl_y = int(rng.integers(3, 9))
    L1 = LayerSpec(op="conv", name="expand1x1", src=0, dst=1, Cin=c, Cout=ce, fl_x=fl_in, fl_w=fl_w,
                   fl_y=fl_y, clip_lo=0, clip_hi=255, x_type="s8", y_type="u8",
                   in_hw=(hw, hw), out_hw=(hw, hw))
    L1.w = draw_weight(rng, (ce, 1, 1, c), 0.05, fl_w)
    L1.bias = draw_bias(rng, ce, fl_in + fl_w)

    fl_x2 = fl_y
    fl_w = int(rng.integers(3, 9)); fl_y = int(rng.integers(3, 9))
    L2 = LayerSpec(op="dwconv", name="dw3x3", src=1, dst=2, Cin=ce, Cout=ce, R=3, S=3, stride=1, pad=1,
                   fl_x=fl_x2, fl_w=fl_w, fl_y=fl_y, clip_lo=0, clip_hi=255, x_type="u8", y_type="u8",
                   in_hw=(hw, hw), out_hw=(hw, hw))
    L2.w = draw_weight(rng, (3, 3, ce), 0.05, fl_w)
    L2.bias = draw_bias(rng, ce, fl_x2 + fl_w)

    fl_x3 = fl_y
    fl_w = int(rng.integers(3, 9)); fl_y = int(rng.integers(3, 9))
    L3 = LayerSpec(op="conv", name="project1x1", src=2, dst=3, Cin=ce, Cout=c, fl_x=fl_x3, fl_w=fl_w,
                   fl_y=fl_y, clip_lo=-127, clip_hi=127, x_type="u8", y_type="s8",
                   in_hw=(hw, hw), out_hw=(hw, hw))
    L3.w = draw_weight(rng, (c, 1, 1, ce), 0.05, fl_w)
    L3.bias = draw_bias(rng, c, fl_x3 + fl_w)
    if with_residual:
        L3.res, L3.res_type, L3.fl_res = 0, "s8", fl_in
    net.layers = [L1, L2, L3]
    return x, net


# ---------------------------------------------------------------------------------
# configurations 3 and 4: whole ResNet forward passes
# ---------------------------------------------------------------------------------

class _NetBuilder:
    """Book-keeping for tensor ids, shapes, types and fractional lengths."""

    def __init__(self, name, rng, hw, c, x_type, fl_x, fl_w_range, fl_a_range, clip_draw):
        self.rng = rng
        self.net = Net(name=name, in_hw=(hw, hw), in_c=c, x_type=x_type, fl_x=fl_x)
        self.t = {0: dict(hw=(hw, hw), c=c, type=x_type, fl=fl_x)}
        self.next_id = 1
        self.fl_w_range = fl_w_range
        self.fl_a_range = fl_a_range
        self.clip_draw = clip_draw

    def _new(self, hw, c, type_, fl):
        i = self.next_id
        self.next_id += 1
        self.t[i] = dict(hw=hw, c=c, type=type_, fl=fl)
        return i

    def conv(self, name, src, cout, k, stride, pad, relu=True, res=-1, raw=False, dual=False):
        """dual=True: the layer also writes its result in a second, separately drawn format and
        the method returns both tensor ids."""
        rng, s = self.rng, self.t[src]
        cin = s["c"]
        K = k * k * cin
        fl_w = int(rng.integers(self.fl_w_range[0], self.fl_w_range[1] + 1))
        fl_y = int(rng.integers(self.fl_a_range[0], self.fl_a_range[1] + 1))
        w = draw_weight(rng, (cout, k, k, cin), float(np.sqrt(2.0 / K)), fl_w)
        bias = draw_bias(rng, cout, s["fl"] + fl_w)
        hw = (_out(s["hw"][0], k, stride, pad), _out(s["hw"][1], k, stride, pad))
        if raw:
            y_type, lo, hi, fl_y = "s32", 0, 0, s["fl"] + fl_w
        elif relu:
            y_type, lo, hi = "u8", 0, 255
            if self.clip_draw and int(rng.integers(0, 4)) == 0:
                hi = int(rng.integers(96, 255))
        else:
            y_type, lo, hi = "s8", -127, 127
        dst = self._new(hw, cout, y_type, fl_y)
        L = LayerSpec(op="conv", name=name, src=src, dst=dst, res=res, Cin=cin, Cout=cout, R=k, S=k,
                      stride=stride, pad=pad, fl_x=s["fl"], fl_w=fl_w, fl_y=fl_y, clip_lo=lo,
                      clip_hi=hi, x_type=s["type"], y_type=y_type, w=w, bias=bias,
                      in_hw=s["hw"], out_hw=hw)
        if res >= 0:
            L.res_type, L.fl_res = self.t[res]["type"], self.t[res]["fl"]
        self.net.layers.append(L)
        if dual:
            fl_y2 = int(rng.integers(self.fl_a_range[0], self.fl_a_range[1] + 1))
            if fl_y2 == fl_y:
                fl_y2 = fl_y + 1
            L.fl_y2, L.y2_type, L.clip_lo2, L.clip_hi2 = fl_y2, y_type, lo, hi
            if relu and self.clip_draw and int(rng.integers(0, 4)) == 0:
                L.clip_hi2 = int(rng.integers(96, 255))
            L.dst2 = self._new(hw, cout, y_type, fl_y2)
            return dst, L.dst2
        return dst

    def dwconv(self, name, src, k, stride, pad):
        """Depthwise layer followed by the unsigned quantiser (ReLU + clip)."""
        rng, s = self.rng, self.t[src]
        c = s["c"]
        fl_w = int(rng.integers(self.fl_w_range[0], self.fl_w_range[1] + 1))
        fl_y = int(rng.integers(self.fl_a_range[0], self.fl_a_range[1] + 1))
        w = draw_weight(rng, (k, k, c), float(np.sqrt(2.0 / (k * k))), fl_w)
        bias = draw_bias(rng, c, s["fl"] + fl_w)
        hw = (_out(s["hw"][0], k, stride, pad), _out(s["hw"][1], k, stride, pad))
        hi = 255
        if self.clip_draw and int(rng.integers(0, 4)) == 0:
            hi = int(rng.integers(96, 255))
        dst = self._new(hw, c, "u8", fl_y)
        self.net.layers.append(LayerSpec(
            op="dwconv", name=name, src=src, dst=dst, Cin=c, Cout=c, R=k, S=k, stride=stride, pad=pad,
            fl_x=s["fl"], fl_w=fl_w, fl_y=fl_y, clip_lo=0, clip_hi=hi, x_type=s["type"], y_type="u8",
            w=w, bias=bias, in_hw=s["hw"], out_hw=hw))
        return dst

    def maxpool(self, name, src, k=3, stride=2, pad=1):
        s = self.t[src]
        hw = (_out(s["hw"][0], k, stride, pad), _out(s["hw"][1], k, stride, pad))
        dst = self._new(hw, s["c"], s["type"], s["fl"])
        self.net.layers.append(LayerSpec(
            op="maxpool", name=name, src=src, dst=dst, Cin=s["c"], Cout=s["c"], R=k, S=k, stride=stride,
            pad=pad, fl_x=s["fl"], fl_y=s["fl"], x_type=s["type"], y_type=s["type"],
            in_hw=s["hw"], out_hw=hw))
        return dst

    def gpool(self, name, src):
        """Global pool as an integer sum followed by a rounding shift by ceil(log2(H*W))
        (the remaining factor 2^sh / (H*W) is taken to be folded into the next layer's
        effective weights, the way the paper folds every full-precision scale)."""
        s = self.t[src]
        n = s["hw"][0] * s["hw"][1]
        sh = int(np.ceil(np.log2(n)))
        dst = self._new((1, 1), s["c"], "u8", s["fl"])
        self.net.layers.append(LayerSpec(
            op="gpool", name=name, src=src, dst=dst, Cin=s["c"], Cout=s["c"], R=s["hw"][0], S=s["hw"][1],
            fl_x=s["fl"], fl_w=sh, fl_y=s["fl"], clip_lo=0, clip_hi=255, x_type=s["type"], y_type="u8",
            in_hw=s["hw"], out_hw=(1, 1)))
        return dst


def _resnet_input(rng, batch, hw=224):
    return draw_s8_normal(rng, (batch, hw, hw, 3), 5)


def resnet18(rng, hw=224, classes=1000, widths=(64, 128, 256, 512), clip_draw=False):
    b = _NetBuilder("resnet18", rng, hw, 3, "s8", 5, (5, 9), (2, 6), clip_draw)
    t = b.conv("conv1", 0, widths[0], 7, 2, 3)
    t = b.maxpool("maxpool", t)
    for si, c in enumerate(widths):
        for bi in range(2):
            stride = 2 if (si > 0 and bi == 0) else 1
            pre = "s%db%d." % (si + 1, bi + 1)
            short = t
            if stride != 1 or b.t[t]["c"] != c:
                short = b.conv(pre + "ds", t, c, 1, stride, 0, relu=False)
            u = b.conv(pre + "conv_a", t, c, 3, stride, 1)
            t = b.conv(pre + "conv_b", u, c, 3, 1, 1, res=short)
    t = b.gpool("gpool", t)
    b.conv("fc", t, classes, 1, 1, 0, raw=True)
    return b.net


def resnet50b(rng, hw=224, classes=1000, widths=(64, 128, 256, 512), depths=(3, 4, 6, 3),
              clip_draw=True, private_fl=False):
    """private_fl=True: every block output is written in two formats, one per child (the next
    block's first convolution, and its shortcut or downsample branch), each with its own
    fractional length (paper Sec. 4.3)."""
    b = _NetBuilder("resnet50b" + ("_private_fl" if private_fl else ""), rng, hw, 3, "s8", 5, (5, 9), (2, 6),
                    clip_draw)
    t = b.conv("conv1", 0, 64, 7, 2, 3)
    t = t2 = b.maxpool("maxpool", t)
    n_blocks = sum(depths)
    done = 0
    for si, (c, d) in enumerate(zip(widths, depths)):
        for bi in range(d):
            stride = 2 if (si > 0 and bi == 0) else 1
            pre = "s%db%d." % (si + 1, bi + 1)
            short = t2
            if bi == 0:
                short = b.conv(pre + "ds", t2, 4 * c, 1, stride, 0, relu=False)
            u = b.conv(pre + "conv_a", t, c, 1, 1, 0)
            u = b.conv(pre + "conv_b", u, c, 3, stride, 1)
            done += 1
            if private_fl and done < n_blocks:
                t, t2 = b.conv(pre + "conv_c", u, 4 * c, 1, 1, 0, res=short, dual=True)
            else:
                t = t2 = b.conv(pre + "conv_c", u, 4 * c, 1, 1, 0, res=short)
    t = b.gpool("gpool", t)
    b.conv("fc", t, classes, 1, 1, 0, raw=True)
    return b.net


def mobilenet_v2(rng, hw=224, classes=1000, clip_draw=True):
    """MobileNetV2 body in fixed point (paper Sec. 5 / Appx: ReLU6 replaced by the unsigned
    quantiser, linear bottleneck outputs signed): 3x3/2 stem, 17 inverted-residual blocks
    (1x1 expand, 3x3 depthwise, 1x1 linear projection, identity shortcut when shapes match),
    1x1 to 1280 channels, global pool, classifier."""
    b = _NetBuilder("mobilenet_v2", rng, hw, 3, "s8", 5, (5, 9), (2, 6), clip_draw)
    t = b.conv("stem", 0, 32, 3, 2, 1)
    cfg = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1))
    blk = 0
    for expand, c, n, stride in cfg:
        for i in range(n):
            blk += 1
            pre = "b%d." % blk
            st = stride if i == 0 else 1
            cin = b.t[t]["c"]
            u = t
            if expand != 1:
                u = b.conv(pre + "expand", u, cin * expand, 1, 1, 0)
            u = b.dwconv(pre + "dw", u, 3, st, 1)
            shortcut = t if (st == 1 and cin == c) else -1
            t = b.conv(pre + "project", u, c, 1, 1, 0, relu=False, res=shortcut)
    t = b.conv("head", t, 1280, 1, 1, 0)
    t = b.gpool("gpool", t)
    b.conv("fc", t, classes, 1, 1, 0, raw=True)
    return b.net


def mobilenet_v1(rng, hw=224, classes=1000, clip_draw=True):
    """MobileNetV1 body in fixed point: 3x3/2 stem, 13 depthwise-separable blocks (3x3 depthwise,
    1x1 pointwise, each followed by the unsigned quantiser), global pool, classifier."""
    b = _NetBuilder("mobilenet_v1", rng, hw, 3, "s8", 5, (5, 9), (2, 6), clip_draw)
    t = b.conv("stem", 0, 32, 3, 2, 1)
    cfg = ((64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2), (512, 1), (512, 1), (512, 1), (512, 1),
           (512, 1), (1024, 2), (1024, 1))
    for i, (c, stride) in enumerate(cfg):
        t = b.dwconv("b%d.dw" % (i + 1), t, 3, stride, 1)
        t = b.conv("b%d.pw" % (i + 1), t, c, 1, 1, 0)
    t = b.gpool("gpool", t)
    b.conv("fc", t, classes, 1, 1, 0, raw=True)
    return b.net


def mobilenet_v1_forward(seed=None, batch=64, hw=224):
    """Whole fixed-point MobileNetV1 forward (beyond the five baseline configs)."""
    rng = np.random.default_rng(seed_of(6) if seed is None else seed)
    x = _resnet_input(rng, batch, hw)
    return x, mobilenet_v1(rng, hw)


def mobilenet_v2_forward(seed=None, batch=64, hw=224):
    """Whole fixed-point MobileNetV2 forward (beyond the five baseline configs)."""
    rng = np.random.default_rng(seed_of(5) if seed is None else seed)
    x = _resnet_input(rng, batch, hw)
    return x, mobilenet_v2(rng, hw)


def config3(seed=None, batch=64, hw=224):
    rng = np.random.default_rng(seed_of(3) if seed is None else seed)
    x = _resnet_input(rng, batch, hw)
    return x, resnet18(rng, hw)


def config4(seed=None, batch=256, hw=224):
    rng = np.random.default_rng(seed_of(4) if seed is None else seed)
    x = _resnet_input(rng, batch, hw)
    return x, resnet50b(rng, hw)


def resnet50_private_fl(seed=None, batch=256, hw=224):
    """ResNet-50 in which the two children of every block output keep private fractional
    lengths: the block's last convolution writes both formats."""
    rng = np.random.default_rng(seed_of(8) if seed is None else seed)
    x = _resnet_input(rng, batch, hw)
    return x, resnet50b(rng, hw, private_fl=True)


# ---------------------------------------------------------------------------------
# free-form random layers for parity sweeps
# ---------------------------------------------------------------------------------

def random_conv_case(rng, B, H, W, Cin, Cout, R, S, stride, pad, x_type="u8", y_type="u8",
                     res_type=None, shift=None, w_std=None, clip=None, depthwise=False):
    """One random layer with operands: returns (x, LayerSpec, res or None).  Magnitudes
    are chosen so that outputs spread over the whole clip range."""
    K = R * S * (1 if depthwise else Cin)
    fl_x = int(rng.integers(0, 9))
    fl_w = int(rng.integers(0, 9))
    s = int(rng.integers(0, 13)) if shift is None else shift
    fl_y = fl_x + fl_w - s
    if s <= 0:
        # no down-shift: keep operands tiny so that results do not all saturate
        x = rng.integers(0, 4, size=(B, H, W, Cin), dtype=np.uint8) if x_type == "u8" else \
            rng.integers(-3, 4, size=(B, H, W, Cin), dtype=np.int8)
    else:
        x = draw_u8(rng, (B, H, W, Cin)) if x_type == "u8" else \
            rng.integers(-128, 128, size=(B, H, W, Cin), dtype=np.int8)
    if w_std is None:
        # accumulator spread of a few hundred output LSBs
        w_std = min(40.0, max(0.6, 2.0 ** s * 60.0 / (74.0 * np.sqrt(K))))
    wshape = (R, S, Cin) if depthwise else (Cout, R, S, Cin)
    w = np.clip(np.rint(rng.normal(0, w_std, size=wshape)), -127, 127).astype(np.int8)
    nb = Cin if depthwise else Cout
    bias = np.rint(rng.normal(0, 2.0 ** max(s, 0) * 20.0, size=nb)).astype(np.int32)
    if y_type == "u8":
        lo, hi = (0, 255) if clip is None else clip
    elif y_type == "s8":
        lo, hi = (-127, 127) if clip is None else clip
    else:
        lo, hi = 0, 0
    P, Q = _out(H, R, stride, pad), _out(W, S, stride, pad)
    L = LayerSpec(op="dwconv" if depthwise else "conv", Cin=Cin, Cout=nb, R=R, S=S, stride=stride,
                  pad=pad, fl_x=fl_x, fl_w=fl_w, fl_y=fl_y, clip_lo=lo, clip_hi=hi, x_type=x_type,
                  y_type=y_type, w=w, bias=bias, in_hw=(H, W), out_hw=(P, Q))
    res = None
    if res_type is not None:
        L.res_type = res_type
        L.fl_res = int(rng.integers(max(0, fl_x + fl_w - 6), fl_x + fl_w + 4))
        shape = (B, P, Q, nb)
        if res_type == "u8":
            res = draw_u8(rng, shape)
        elif res_type == "s8":
            res = rng.integers(-127, 128, size=shape, dtype=np.int8)
        else:
            res = rng.integers(-2 ** 20, 2 ** 20, size=shape, dtype=np.int32)
        L.res = 0
    return x, L, res


# ----------------------------------------------------------------------------- floating-point side
# Inputs of the steps upstream of the integer layers: tensors to quantise, Gaussian samples of
# the toy experiment, and the trained-model quantities of a Conv-BN block.  Drawn values only.

def fp_tensor(seed, n, std=1.0, mean=0.0):
    """n float32 values ~ N(mean, std)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(n) * std + mean).astype(np.float32)


def toy_samples(seed=None, n=10000):
    """The unit-variance zero-mean Gaussian samples of the toy experiment (scaled by the caller
    to each standard deviation), float32."""
    rng = np.random.default_rng(seed_of(7) if seed is None else seed)
    return rng.standard_normal(n).astype(np.float32)


@dataclass
class FpBlock:
    """Floating-point quantities of one Conv-BN block: W [Cout][K] (K = R*S*Cin flattened in
    the integer layers' weight order), the BN scale gamma, shift beta, running mean mu and
    running standard deviation sigma, the clipping levels and fractional lengths of its input
    quantiser (alpha_in, fl_in) and of its child's (alpha_out, fl_out)."""
    W: np.ndarray
    gamma: np.ndarray
    beta: np.ndarray
    mu: np.ndarray
    sigma: np.ndarray
    alpha_in: float
    fl_in: int
    alpha_out: float
    fl_out: int


def fp_conv_bn_block(seed, cout, k):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((cout, k)) * np.sqrt(2.0 / k)).astype(np.float32)
    gamma = rng.uniform(0.4, 1.6, cout).astype(np.float32)
    gamma *= rng.choice(np.array([-1.0, 1.0], np.float32), cout, p=[0.1, 0.9])
    beta = (rng.standard_normal(cout) * 0.3).astype(np.float32)
    mu = (rng.standard_normal(cout) * 0.5).astype(np.float32)
    sigma = rng.uniform(0.5, 2.0, cout).astype(np.float32)
    alpha_in = float(np.float32(rng.uniform(2.0, 8.0)))
    alpha_out = float(np.float32(rng.uniform(2.0, 8.0)))
    return FpBlock(W, gamma, beta, mu, sigma, alpha_in, int(rng.integers(3, 7)), alpha_out,
                   int(rng.integers(3, 7)))
