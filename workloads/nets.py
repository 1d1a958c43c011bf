"""Layer lists of the five synthetic early-exit networks and their random weights.

The architectures are the public ResNet-18 / ResNet-50 / MobileNetV2 layer
shapes (plus a three-stage toy net); weights are seeded random numbers.  The
result of `build_net` is a blob (see blob.py) whose calibration fields (shift,
res_shift, gap_shift, frac_bits, logit_scale, thr) still hold placeholder
values; they are filled in later from a calibration record.
"""
import math
import numpy as np

from . import rng
from .blob import (HEADER_DT, STAGE_DT, OP_DT, EXIT_DT, MAGIC, DT_I8, DT_BF16, OP_CONV, OP_DWCONV,
                   OP_MAXPOOL, OP_AVGPOOL, Blob, f32_to_bf16_bits)

BASE_SEED = 0x220913443000
RELU6_Q = 96  # int8 stand-in for the ReLU6 ceiling (per-tensor power-of-two scales carry no absolute unit)


class _Net:
    def __init__(self, dtype, in_h, in_w, in_c, n_classes):
        self.dtype, self.in_shape, self.n_classes = dtype, (in_h, in_w, in_c), n_classes
        self.stages = []   # list of dict(ops=[...], shapes={id: (h,w,c)}, out=id)
        self._cur = None

    # -- stage construction -------------------------------------------------
    def begin_stage(self):
        prev = self.stages[-1] if self.stages else None
        shape0 = self.in_shape if prev is None else prev["shapes"][prev["out"]]
        self._cur = dict(ops=[], shapes={0: shape0}, out=None)
        return 0

    def end_stage(self, out):
        self._cur["out"] = out
        self.stages.append(self._cur)
        self._cur = None

    def _new(self, shape):
        tid = len(self._cur["shapes"])
        self._cur["shapes"][tid] = shape
        return tid

    def _act(self, act):
        if act == "relu":
            return 0, 127, 0.0, math.inf
        if act == "relu6":
            return 0, RELU6_Q, 0.0, 6.0
        return -128, 127, -math.inf, math.inf

    def new_concat(self, h, w, c_tot):
        """A tensor that several ops fill slice by slice along the channels (`into=(tensor, c_off)`)."""
        return self._new((h, w, c_tot))

    def _dst(self, shape, into):
        """Destination tensor id, channel offset and total channels of an op producing `shape`."""
        if into is None:
            return self._new(shape), 0, shape[2]
        tid, c_off = into
        h, w, c_tot = self._cur["shapes"][tid]
        assert (h, w) == shape[:2] and 0 <= c_off and c_off + shape[2] <= c_tot
        return tid, c_off, c_tot

    def conv(self, src, co, k, stride, pad, act="relu", res=-1, into=None):
        """k and pad are ints (square kernel) or (rows, columns) pairs."""
        h, w, ci = self._cur["shapes"][src]
        kh, kw = (k, k) if isinstance(k, int) else k
        ph, pw = (pad, pad) if isinstance(pad, int) else pad
        ho, wo = (h + 2 * ph - kh) // stride + 1, (w + 2 * pw - kw) // stride + 1
        dst, c_off, c_tot = self._dst((ho, wo, co), into)
        lo, hi, flo, fhi = self._act(act)
        self._cur["ops"].append(dict(kind=OP_CONV, src=src, dst=dst, res=res, h_in=h, w_in=w, c_in=ci,
                                     h_out=ho, w_out=wo, c_out=co, kh=kh, kw=kw, stride=stride, pad=ph, pad_w=pw,
                                     c_off=c_off, c_tot=c_tot, lo=lo, hi=hi, f_lo=flo, f_hi=fhi))
        return dst

    def dwconv(self, src, k, stride, pad, act="relu6"):
        h, w, c = self._cur["shapes"][src]
        ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
        dst = self._new((ho, wo, c))
        lo, hi, flo, fhi = self._act(act)
        self._cur["ops"].append(dict(kind=OP_DWCONV, src=src, dst=dst, res=-1, h_in=h, w_in=w, c_in=c,
                                     h_out=ho, w_out=wo, c_out=c, kh=k, kw=k, stride=stride, pad=pad, pad_w=pad,
                                     c_off=0, c_tot=c, lo=lo, hi=hi, f_lo=flo, f_hi=fhi))
        return dst

    def _pool(self, kind, src, k, stride, pad, into):
        h, w, c = self._cur["shapes"][src]
        ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
        dst, c_off, c_tot = self._dst((ho, wo, c), into)
        self._cur["ops"].append(dict(kind=kind, src=src, dst=dst, res=-1, h_in=h, w_in=w, c_in=c,
                                     h_out=ho, w_out=wo, c_out=c, kh=k, kw=k, stride=stride, pad=pad, pad_w=pad,
                                     c_off=c_off, c_tot=c_tot, lo=-128, hi=127, f_lo=-math.inf, f_hi=math.inf))
        return dst

    def maxpool(self, src, k, stride, pad, into=None):
        return self._pool(OP_MAXPOOL, src, k, stride, pad, into)

    def avgpool(self, src, k, stride, pad, into=None):
        return self._pool(OP_AVGPOOL, src, k, stride, pad, into)


# ---------------------------------------------------------------------------
# architectures
# ---------------------------------------------------------------------------
def _tiny(dtype):
    net = _Net(dtype, 32, 32, 3, 10)
    for ch in (16, 32, 64):
        t = net.begin_stage()
        t = net.conv(t, ch, 3, 2, 1)
        t = net.conv(t, ch, 3, 1, 1)
        net.end_stage(t)
    return net


def _resnet_stem(net):
    t = net.begin_stage()
    t = net.conv(t, 64, 7, 2, 3)
    return net.maxpool(t, 3, 2, 1)


def _resnet18(dtype, in_hw=224, n_classes=1000):
    net = _Net(dtype, in_hw, in_hw, 3, n_classes)
    cin = 64
    for s, (ch, nblk) in enumerate(zip((64, 128, 256, 512), (2, 2, 2, 2))):
        t = _resnet_stem(net) if s == 0 else net.begin_stage()
        for b in range(nblk):
            stride = 2 if (b == 0 and s > 0) else 1
            short = t
            if stride != 1 or cin != ch:
                short = net.conv(t, ch, 1, stride, 0, act="linear")
            u = net.conv(t, ch, 3, stride, 1)
            t = net.conv(u, ch, 3, 1, 1, res=short)
            cin = ch
        net.end_stage(t)
    return net


def _resnet50(dtype, in_hw=224, n_classes=1000, blocks=(3, 4, 6, 3)):
    net = _Net(dtype, in_hw, in_hw, 3, n_classes)
    cin = 64
    for s, (mid, nblk) in enumerate(zip((64, 128, 256, 512), blocks)):
        t = _resnet_stem(net) if s == 0 else net.begin_stage()
        for b in range(nblk):
            stride = 2 if (b == 0 and s > 0) else 1
            short = t
            if b == 0:
                short = net.conv(t, 4 * mid, 1, stride, 0, act="linear")
            u = net.conv(t, mid, 1, 1, 0)
            u = net.conv(u, mid, 3, stride, 1)
            t = net.conv(u, 4 * mid, 1, 1, 0, res=short)
            cin = 4 * mid
        net.end_stage(t)
    return net


def _resnet50_eq(dtype, in_hw=224, n_classes=1000, exits_after=(4, 8, 12, 16)):
    """The same bottleneck backbone with its exits where the cumulative work crosses quarters of the total
    (Sec. IV "Benchmarks": exits placed equidistantly in FLOPs) instead of at the ends of the four resolution
    groups: after bottleneck blocks 4, 8, 12 and 16 (28 %, 53 %, 75 %, 100 % of the MACs: the closest block ends)."""
    net = _Net(dtype, in_hw, in_hw, 3, n_classes)
    t = _resnet_stem(net)
    done = 0
    for g, (mid, nblk) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for b in range(nblk):
            stride = 2 if (b == 0 and g > 0) else 1
            short = t
            if b == 0:
                short = net.conv(t, 4 * mid, 1, stride, 0, act="linear")
            u = net.conv(t, mid, 1, 1, 0)
            u = net.conv(u, mid, 3, stride, 1)
            t = net.conv(u, 4 * mid, 1, 1, 0, res=short)
            done += 1
            if done in exits_after:
                net.end_stage(t)
                if done != exits_after[-1]:
                    t = net.begin_stage()
    return net


def _inception(dtype, in_hw=304, n_classes=1000):
    """Inception-v3-style network with four exits (the paper's second benchmark, Sec. IV): the public layer shapes
    -- factorised 1x7 / 7x1 and 1x3 / 3x1 convolutions, 5x5 convolutions, average-pool branches, channel concatenation --
    with exits after the 35x35 group, in the middle and at the end of the 17x17 group, and at the end.  The input is
    304 x 304 instead of 299 x 299 (a sample is then a whole number of 16-byte chunks); the grids stay 35, 17 and 8."""
    net = _Net(dtype, in_hw, in_hw, 3, n_classes)
    shape = lambda t: net._cur["shapes"][t]

    def block_a(t, pool_ch):
        h, w, _ = shape(t)
        cat = net.new_concat(h, w, 64 + 64 + 96 + pool_ch)
        net.conv(t, 64, 1, 1, 0, into=(cat, 0))
        u = net.conv(t, 48, 1, 1, 0)
        net.conv(u, 64, 5, 1, 2, into=(cat, 64))
        u = net.conv(t, 64, 1, 1, 0)
        u = net.conv(u, 96, 3, 1, 1)
        net.conv(u, 96, 3, 1, 1, into=(cat, 128))
        u = net.avgpool(t, 3, 1, 1)
        net.conv(u, pool_ch, 1, 1, 0, into=(cat, 224))
        return cat

    def reduce_a(t):
        h, w, c = shape(t)
        ho, wo = (h - 3) // 2 + 1, (w - 3) // 2 + 1
        cat = net.new_concat(ho, wo, 384 + 96 + c)
        net.conv(t, 384, 3, 2, 0, into=(cat, 0))
        u = net.conv(t, 64, 1, 1, 0)
        u = net.conv(u, 96, 3, 1, 1)
        net.conv(u, 96, 3, 2, 0, into=(cat, 384))
        net.maxpool(t, 3, 2, 0, into=(cat, 480))
        return cat

    def block_b(t, c7):
        h, w, _ = shape(t)
        cat = net.new_concat(h, w, 768)
        net.conv(t, 192, 1, 1, 0, into=(cat, 0))
        u = net.conv(t, c7, 1, 1, 0)
        u = net.conv(u, c7, (1, 7), 1, (0, 3))
        net.conv(u, 192, (7, 1), 1, (3, 0), into=(cat, 192))
        u = net.conv(t, c7, 1, 1, 0)
        u = net.conv(u, c7, (7, 1), 1, (3, 0))
        u = net.conv(u, c7, (1, 7), 1, (0, 3))
        u = net.conv(u, c7, (7, 1), 1, (3, 0))
        net.conv(u, 192, (1, 7), 1, (0, 3), into=(cat, 384))
        u = net.avgpool(t, 3, 1, 1)
        net.conv(u, 192, 1, 1, 0, into=(cat, 576))
        return cat

    def reduce_b(t):
        h, w, c = shape(t)
        ho, wo = (h - 3) // 2 + 1, (w - 3) // 2 + 1
        cat = net.new_concat(ho, wo, 320 + 192 + c)
        u = net.conv(t, 192, 1, 1, 0)
        net.conv(u, 320, 3, 2, 0, into=(cat, 0))
        u = net.conv(t, 192, 1, 1, 0)
        u = net.conv(u, 192, (1, 7), 1, (0, 3))
        u = net.conv(u, 192, (7, 1), 1, (3, 0))
        net.conv(u, 192, 3, 2, 0, into=(cat, 320))
        net.maxpool(t, 3, 2, 0, into=(cat, 512))
        return cat

    def block_c(t):
        h, w, _ = shape(t)
        cat = net.new_concat(h, w, 2048)
        net.conv(t, 320, 1, 1, 0, into=(cat, 0))
        u = net.conv(t, 384, 1, 1, 0)
        net.conv(u, 384, (1, 3), 1, (0, 1), into=(cat, 320))
        net.conv(u, 384, (3, 1), 1, (1, 0), into=(cat, 704))
        u = net.conv(t, 448, 1, 1, 0)
        u = net.conv(u, 384, 3, 1, 1)
        net.conv(u, 384, (1, 3), 1, (0, 1), into=(cat, 1088))
        net.conv(u, 384, (3, 1), 1, (1, 0), into=(cat, 1472))
        u = net.avgpool(t, 3, 1, 1)
        net.conv(u, 192, 1, 1, 0, into=(cat, 1856))
        return cat

    t = net.begin_stage()
    t = net.conv(t, 32, 3, 2, 0)
    t = net.conv(t, 32, 3, 1, 0)
    t = net.conv(t, 64, 3, 1, 1)
    t = net.maxpool(t, 3, 2, 0)
    t = net.conv(t, 80, 1, 1, 0)
    t = net.conv(t, 192, 3, 1, 0)
    t = net.maxpool(t, 3, 2, 0)
    for pool_ch in (32, 64, 64):
        t = block_a(t, pool_ch)
    net.end_stage(t)
    t = net.begin_stage()
    t = reduce_a(t)
    for c7 in (128, 160):
        t = block_b(t, c7)
    net.end_stage(t)
    t = net.begin_stage()
    for c7 in (160, 192):
        t = block_b(t, c7)
    net.end_stage(t)
    t = net.begin_stage()
    t = reduce_b(t)
    for _ in range(2):
        t = block_c(t)
    net.end_stage(t)
    return net


def _mobilenetv2(dtype, in_hw=224, n_classes=1000):
    net = _Net(dtype, in_hw, in_hw, 3, n_classes)
    cfg = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
    exits_after = (6, 13, 17)
    t = net.begin_stage()
    t = net.conv(t, 32, 3, 2, 1, act="relu6")
    cin, blk = 32, 0
    for (e, c, n, s) in cfg:
        for i in range(n):
            stride = s if i == 0 else 1
            u = t
            if e != 1:
                u = net.conv(u, cin * e, 1, 1, 0, act="relu6")
            u = net.dwconv(u, 3, stride, 1, act="relu6")
            use_res = (stride == 1 and cin == c)
            t = net.conv(u, c, 1, 1, 0, act="linear", res=t if use_res else -1)
            cin = c
            blk += 1
            if blk in exits_after:
                if blk == exits_after[-1]:
                    t = net.conv(t, 1280, 1, 1, 0, act="relu6")   # final head's 1x1 expansion
                    net.end_stage(t)
                else:
                    net.end_stage(t)
                    t = net.begin_stage()
    return net


def _zoo(dtype):
    """Test network: every kernel path and awkward shape (odd image sizes, channel counts that are not
    multiples of 16, 1x1 / 3x3 / 5x5 / 7x7 kernels, strides, residuals, depthwise, max-pool)."""
    net = _Net(dtype, 36, 44, 3, 37)
    t = net.begin_stage()
    t = net.conv(t, 16, 3, 2, 1)
    t = net.conv(t, 24, 1, 1, 0)
    t = net.conv(t, 32, 3, 1, 1)
    t = net.maxpool(t, 3, 2, 1)
    net.end_stage(t)
    t = net.begin_stage()
    short = net.conv(t, 128, 1, 2, 0, act="linear")
    u = net.conv(t, 64, 1, 1, 0)
    u = net.conv(u, 64, 3, 2, 1)
    t = net.conv(u, 128, 1, 1, 0, res=short)
    u = net.dwconv(t, 3, 1, 1, act="relu6")
    u = net.conv(u, 128, 1, 1, 0, act="linear", res=t)
    u = net.dwconv(u, 3, 2, 1, act="relu6")
    t = net.conv(u, 48, 1, 1, 0, act="linear")
    net.end_stage(t)
    t = net.begin_stage()
    t = net.conv(t, 64, 5, 1, 2)
    t = net.conv(t, 80, 7, 2, 3)
    t = net.conv(t, 256, 1, 1, 0, act="relu6")
    net.end_stage(t)
    return net


def random_net(seed, dtype):
    """A small random network for parity fuzzing: one or two segments of randomly chosen layers -- square and
    rectangular kernels with their own padding per axis, strides, residuals, depthwise, max / average pooling and
    concatenations whose slices come from convolutions and pooling -- with requantisation shifts guessed from the
    reduction length, so that outputs are neither all zero nor all saturated.  Data only: no arithmetic of the method."""
    r = np.random.default_rng(0xFA57 + seed)
    es = 1 if dtype == DT_I8 else 2
    pick = lambda seq: seq[int(r.integers(len(seq)))]
    c0 = pick([3, 4, 8, 16, 32, 48])
    net = _Net(dtype, int(r.integers(6, 20)), 16 if c0 == 3 else pick([8, 12, 16]), c0, 10)     # a sample is whole 16-byte chunks
    for _ in range(int(r.integers(1, 3))):
        t0 = net.begin_stage()
        shapes = net._cur["shapes"]
        avail = [t0]
        for _ in range(int(r.integers(5, 12))):
            src = pick(avail)
            h, w, c = shapes[src]
            kind = pick(["conv"] * 5 + ["pool", "dw", "cat"])
            chunked = (c * es) % 16 == 0
            if kind == "conv" or (kind in ("pool", "dw") and not chunked) or (kind == "cat" and min(h, w) < 2):
                kh, kw = pick([(1, 1), (3, 3), (1, 3), (3, 1), (1, 7), (7, 1), (5, 5), (2, 2), (3, 5)])
                stride = pick([1, 1, 2])
                ph, pw = (kh // 2, kw // 2) if r.integers(3) else (0, 0)
                if (h + 2 * ph - kh) // stride + 1 < 1 or (w + 2 * pw - kw) // stride + 1 < 1:
                    ph, pw = kh // 2, kw // 2
                co = pick([4, 8, 12, 16, 24, 32, 40, 64, 80, 136])
                ho, wo = (h + 2 * ph - kh) // stride + 1, (w + 2 * pw - kw) // stride + 1
                res = [t for t in avail if shapes[t] == (ho, wo, co)]
                avail.append(net.conv(src, co, (kh, kw), stride, (ph, pw), act=pick(["relu", "relu", "linear", "relu6"]),
                                      res=pick(res) if res and r.integers(2) else -1))
            elif kind == "pool":
                k, stride, pad = 3, pick([1, 2]), pick([0, 1])
                if (min(h, w) + 2 * pad - k) // stride + 1 < 1:
                    pad, stride = 1, 1
                avail.append((net.maxpool if r.integers(2) else net.avgpool)(src, k, stride, pad))
            elif kind == "dw":
                avail.append(net.dwconv(src, 3, pick([1, 2]), 1, act=pick(["relu6", "relu"])))
            else:                                       # concatenation of 2-3 convolution branches and, maybe, a pooled copy
                widths = [pick([16, 32, 48]) // es * es for _ in range(int(r.integers(2, 4)))]
                pooled = chunked and bool(r.integers(2))
                cat = net.new_concat(h, w, sum(widths) + (c if pooled else 0))
                off = 0
                for wd in widths:
                    kh, kw = pick([(1, 1), (3, 3), (1, 3), (3, 1), (1, 7), (5, 5)])
                    u = net.conv(src, pick([8, 16, 24]), 1, 1, 0) if r.integers(2) else src
                    net.conv(u, wd, (kh, kw), 1, (kh // 2, kw // 2), into=(cat, off))
                    off += wd
                if pooled:
                    (net.maxpool if r.integers(2) else net.avgpool)(src, 3, 1, 1, into=(cat, off))
                avail.append(cat)
        net.end_stage(net.conv(avail[-1], 32, 1, 1, 0))       # segment outputs (what the exit heads read): 32 channels
    blob = _assemble(net, dtype, BASE_SEED + 0x5000 + seed)
    for op in blob.ops:
        if int(op["kind"]) in (OP_CONV, OP_DWCONV):
            k_red = int(op["kh"]) * int(op["kw"]) * (int(op["c_in"]) if int(op["kind"]) == OP_CONV else 1)
            op["shift"] = max(0, int(math.ceil(math.log2(2.0 * 74 * 50 * math.sqrt(k_red) / 127))))
            op["res_shift"] = min(int(op["shift"]), 6) if int(op["res"]) >= 0 else 0
    for e in blob.exits:
        e["frac_bits"], e["thr"] = 10, 0.5
    return blob


def single_layer_net(kind, h, w, c, k, stride, pad, dtype, seed=0, co=None, act="linear"):
    """One segment that is one layer on the input tensor ("maxpool", "avgpool", "dw", or "conv" with `co` output
    channels), so that a test sees the layer's own output: for edge shapes and hand-picked input values.  Data only."""
    net = _Net(dtype, h, w, c, 10)
    t0 = net.begin_stage()
    if kind == "dw":
        out = net.dwconv(t0, k, stride, pad, act="linear")
    elif kind == "conv":
        out = net.conv(t0, co, k, stride, pad, act=act)
    else:
        out = (net.maxpool if kind == "maxpool" else net.avgpool)(t0, k, stride, pad)
    net.end_stage(out)
    blob = _assemble(net, dtype, BASE_SEED + 0x6000 + seed)
    for op in blob.ops:
        if int(op["kind"]) == OP_DWCONV:
            op["shift"] = 7
        elif int(op["kind"]) == OP_CONV:
            op["shift"] = max(0, int(math.ceil(math.log2(2.0 * 74 * 74 * math.sqrt(int(op["kh"]) * int(op["kw"]) * c) / 127))))
    for e in blob.exits:
        e["frac_bits"], e["thr"] = 10, 0.5
    return blob


def inverted_residual_net(h, w, ci, ce, co, stride, seed=0, blocks=1):
    """One segment of `blocks` inverted-residual blocks (1x1 expansion to `ce` channels -- none when ce = 0 --, 3x3 depthwise with the given stride
    in the first block, 1x1 projection to `co` channels (an int, or one value per block), with the block's input as residual where shapes allow) on an
    h x w x ci input, int8: the fused-block kernel's shapes alone, for edge cases.  Data only."""
    net = _Net(DT_I8, h, w, ci, 10)
    t = net.begin_stage()
    cin = ci
    cos = [co] * blocks if isinstance(co, int) else list(co)          # output channels per block
    for i in range(blocks):
        s_i = stride if i == 0 else 1
        u = net.conv(t, ce, 1, 1, 0, act="relu6") if ce else t         # ce = 0: no expansion, the depthwise layer reads the block's input
        u = net.dwconv(u, 3, s_i, 1, act="relu6")
        t = net.conv(u, cos[i], 1, 1, 0, act="linear", res=t if (s_i == 1 and cin == cos[i]) else -1)
        cin = cos[i]
    net.end_stage(t)
    blob = _assemble(net, DT_I8, BASE_SEED + 0x7000 + seed)
    for op in blob.ops:
        if int(op["kind"]) == OP_DWCONV:
            op["shift"] = 7
        elif int(op["kind"]) == OP_CONV:
            op["shift"] = max(0, int(math.ceil(math.log2(2.0 * 74 * 40 * math.sqrt(int(op["c_in"])) / 127))))
    for e in blob.exits:
        e["frac_bits"], e["thr"] = 10, 0.5
    return blob


def stem_net(h, w, seed=0):
    """The first layers of a ResNet-style network alone on an h x w x 3 input, int8: 7x7 stride-2 convolution to 64 channels, 3x3 stride-2
    max-pool, and a 1x1 convolution to 32 channels as the segment's output: the fused first-layer kernel's shapes, for edge cases.  Data only."""
    net = _Net(DT_I8, h, w, 3, 10)
    t = net.begin_stage()
    t = net.conv(t, 64, 7, 2, 3)
    t = net.maxpool(t, 3, 2, 1)
    net.end_stage(net.conv(t, 32, 1, 1, 0))
    blob = _assemble(net, DT_I8, BASE_SEED + 0x7c00 + seed)
    for op in blob.ops:
        if int(op["kind"]) == OP_CONV:
            fan_in = int(op["c_in"]) * int(op["kh"]) * int(op["kw"])
            op["shift"] = max(0, int(math.ceil(math.log2(2.0 * 74 * 40 * math.sqrt(fan_in) / 127))))
    for e in blob.exits:
        e["frac_bits"], e["thr"] = 10, 0.5
    return blob


def bottleneck_net(h, w, ci, seed=0, blocks=1, mid=64, stages=1):
    """`stages` segments (each with an exit) of `blocks` bottleneck blocks (1x1 to `mid` channels, 3x3 stride 1, 1x1 to 4 * mid channels with a residual:
    the block's input where it has 4 * mid channels, else a 1x1 convolution of it) on an h x w x ci input, int8: the fused-block
    kernel's shapes alone, for edge cases.  Data only."""
    net = _Net(DT_I8, h, w, ci, 10)
    cin = ci
    for _ in range(stages):
        t = net.begin_stage()
        for i in range(blocks):
            # a segment behind the first starts with a convolution on its shortcut, as ResNet-50's groups do (the segment's input is then read by convolutions only)
            short = t if cin == 4 * mid and not (stages > 1 and i == 0) else net.conv(t, 4 * mid, 1, 1, 0, act="linear")
            u = net.conv(t, mid, 1, 1, 0)
            u = net.conv(u, mid, 3, 1, 1)
            t = net.conv(u, 4 * mid, 1, 1, 0, res=short)
            cin = 4 * mid
        net.end_stage(t)
    blob = _assemble(net, DT_I8, BASE_SEED + 0x7800 + seed)
    for op in blob.ops:
        if int(op["kind"]) == OP_CONV:
            fan_in = int(op["c_in"]) * int(op["kh"]) * int(op["kw"])
            op["shift"] = max(0, int(math.ceil(math.log2(2.0 * 74 * 40 * math.sqrt(fan_in) / 127))))
            if int(op["res"]) >= 0:
                op["res_shift"] = max(0, int(op["shift"]) - 1)
    for e in blob.exits:
        e["frac_bits"], e["thr"] = 10, 0.5
    return blob


CONFIGS = {
    # name: (architecture, dtype, seed offset)
    "tiny_i8": (_tiny, DT_I8, 1),
    "resnet18_i8": (_resnet18, DT_I8, 2),
    "mobilenetv2_i8": (_mobilenetv2, DT_I8, 3),
    "resnet50_i8": (_resnet50, DT_I8, 4),
    "resnet50_bf16": (_resnet50, DT_BF16, 5),
    "resnet50_eq_i8": (_resnet50_eq, DT_I8, 6),          # exits equidistant in work
    "inception_i8": (_inception, DT_I8, 7),
    "inception_small_i8": (lambda dt: _inception(dt, 80, 100), DT_I8, 16),
    "inception_small_bf16": (lambda dt: _inception(dt, 80, 100), DT_BF16, 17),
    # reduced-size variants for fast tests (same layer types, smaller images / fewer classes)
    "tiny_bf16": (_tiny, DT_BF16, 11),
    "resnet18_small_i8": (lambda dt: _resnet18(dt, 64, 100), DT_I8, 12),
    "resnet50_small_i8": (lambda dt: _resnet50(dt, 64, 100, (1, 2, 2, 1)), DT_I8, 14),
    "resnet50_small_bf16": (lambda dt: _resnet50(dt, 64, 100, (1, 2, 2, 1)), DT_BF16, 15),
    "mobilenetv2_small_i8": (lambda dt: _mobilenetv2(dt, 64, 100), DT_I8, 13),
    "zoo_i8": (_zoo, DT_I8, 21),
    "zoo_bf16": (_zoo, DT_BF16, 22),
}


# ---------------------------------------------------------------------------
# blob assembly
# ---------------------------------------------------------------------------
def _align(n, a=64):
    return (n + a - 1) // a * a


def _int8_weights(seed, stream, count):
    """int8 uniform over [-127, 127]."""
    raw = rng.uniform_bytes(seed, stream, 2 * count).view("<u2")
    return (raw % np.uint16(255)).astype(np.int16).__sub__(127).astype(np.int8)


def _int32_bias(seed, stream, count, bits):
    raw = rng.raw_u64(seed, stream, count)
    span = np.uint64((1 << (bits + 1)) + 1)
    return ((raw >> np.uint64(16)) % span).astype(np.int64).__sub__(1 << bits).astype(np.int32)


def build_net(name):
    """Assemble the un-calibrated blob of configuration `name` (a key of CONFIGS)."""
    arch, dtype, off = CONFIGS[name]
    return _assemble(arch(dtype), dtype, BASE_SEED + off)


def _assemble(net, dtype, seed):
    """Blob of a layer list: records, seeded random weights and biases."""
    n_stages = len(net.stages)
    n_ops = sum(len(s["ops"]) for s in net.stages)
    stages = np.zeros(n_stages, STAGE_DT)
    ops = np.zeros(n_ops, OP_DT)
    exits = np.zeros(n_stages, EXIT_DT)
    stages_off = 128
    ops_off = stages_off + stages.nbytes
    exits_off = ops_off + ops.nbytes
    data_off = _align(exits_off + exits.nbytes)
    chunks, cursor, stream = [], data_off, 1

    def put(arr):
        nonlocal cursor
        off0 = cursor
        b = np.ascontiguousarray(arr).view(np.uint8).ravel()
        pad = _align(b.size) - b.size
        chunks.append(b)
        if pad:
            chunks.append(np.zeros(pad, np.uint8))
        cursor += b.size + pad
        return off0

    def weights(count, fan_in):
        nonlocal stream
        stream += 1
        if dtype == DT_I8:
            return _int8_weights(seed, stream, count)
        w = rng.normal_f64(seed, stream, count) * math.sqrt(2.0 / fan_in)
        return f32_to_bf16_bits(w.astype(np.float32))

    def bias(count, k_red):
        nonlocal stream
        stream += 1
        if dtype == DT_I8:
            return _int32_bias(seed, stream, count, 10 + int(math.ceil(0.5 * math.log2(k_red))))
        return np.zeros(count, np.float32)

    oi = 0
    for s, st in enumerate(net.stages):
        oh, ow, oc = st["shapes"][st["out"]]
        stages[s] = (oi, len(st["ops"]), len(st["shapes"]), st["out"], oh, ow, oc, 0)
        for op in st["ops"]:
            rec = ops[oi]
            for k, v in op.items():
                rec[k] = v
            rec["shift"], rec["res_shift"] = 0, 0
            if op["kind"] == OP_CONV:
                kred = op["kh"] * op["kw"] * op["c_in"]
                rec["w_off"] = put(weights(op["c_out"] * kred, kred))
                rec["b_off"] = put(bias(op["c_out"], kred))
            elif op["kind"] == OP_DWCONV:
                kred = op["kh"] * op["kw"]
                rec["w_off"] = put(weights(op["c_out"] * kred, kred))
                rec["b_off"] = put(bias(op["c_out"], kred))
            oi += 1
        e = exits[s]
        e["h"], e["w"], e["c"], e["n_cls"] = oh, ow, oc, net.n_classes
        e["gap_shift"] = int(math.ceil(math.log2(oh * ow))) if oh * ow > 1 else 0
        e["frac_bits"], e["logit_scale"], e["thr"] = 8, 1.0, 2.0
        e["w_off"] = put(weights(net.n_classes * oc, oc))
        e["b_off"] = put(bias(net.n_classes, oc))

    header = np.zeros(1, HEADER_DT)
    header[0]["magic"] = MAGIC
    header[0]["version"], header[0]["dtype"] = 2, dtype
    header[0]["n_stages"], header[0]["n_ops"] = n_stages, n_ops
    header[0]["in_h"], header[0]["in_w"], header[0]["in_c"] = net.in_shape
    header[0]["n_classes"] = net.n_classes
    header[0]["stages_off"], header[0]["ops_off"] = stages_off, ops_off
    header[0]["exits_off"], header[0]["data_off"] = exits_off, data_off
    header[0]["total_bytes"] = cursor
    head = np.concatenate([header.view(np.uint8), stages.view(np.uint8), ops.view(np.uint8), exits.view(np.uint8)])
    head = np.concatenate([head, np.zeros(data_off - head.size, np.uint8)])
    return Blob(np.concatenate([head] + chunks).tobytes())


def apply_calibration(blob, rec):
    """Write a calibration record (per-layer shifts, logit scaling, exit thresholds) into a blob."""
    assert len(rec["ops"]) == len(blob.ops) and len(rec["exits"]) == blob.n_stages
    for op, r in zip(blob.ops, rec["ops"]):
        op["shift"], op["res_shift"] = r["shift"], r["res_shift"]
    for e, r in zip(blob.exits, rec["exits"]):
        e["gap_shift"], e["frac_bits"] = r["gap_shift"], r["frac_bits"]
        e["logit_scale"] = np.uint32(r["logit_scale_bits"]).view(np.float32)
        e["thr"] = np.uint32(r["thr_bits"]).view(np.float32)
    return blob


def load_net(name):
    """The calibrated blob of configuration `name` (needs workloads/calib/<name>.json)."""
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "calib", f"{name}.json")
    with open(path) as f:
        rec = json.load(f)
    return apply_calibration(build_net(name), rec)
