"""Declarative descriptions of the ensemble members used as synthetic workloads.

A member is a flat list of operations over numbered NHWC tensors plus a list
of parameter tensors living in one flat fp32 blob.  The description is pure
data: the CPU oracle and the GPU library each read it and implement every
operation on their own.  Shapes follow the public architecture papers
(ResNet, DenseNet, Inception-v3, EfficientNet, VGG, Xception, MobileNetV2); only the shapes matter for the
throughput study, the weights are random (see synth.weights).

Operation semantics (tensor = H x W x C, channel slices [c0, c0+n)):

  CONV     dst[:, :, dst_c0:+cout] = act( bn( conv(pre(src[:, :, src_c0:+cin])) + bias ) + res )
           weights [kh][kw][cin][cout]; with r = g > 1 groups output channel co sees the input
           channels of group co // (cout/g) only and the weights are [kh][kw][cin/g][cout]; zero padding (pt rows above, pl columns
           left; the output size is the dst tensor's H x W); `pre` applies an
           inference batch-norm followed by ReLU to the in-bounds input values.
  DWCONV   depthwise: one kh x kw filter per channel, weights [kh][kw][c].
  MAXPOOL  window maximum over the in-bounds part of the window.
  AVGPOOL  window mean over the in-bounds part of the window.
  GAP      mean over all pixels (optionally of relu(bn(x)) when `pre`).
  FC       dst = src . W[cin][cout] + bias   (src is a 1 x 1 x cin tensor).
  SE       squeeze-excite: s = mean over pixels; g = sigmoid(W2^T silu(W1^T s + b1) + b2);
           dst = src * g  (per channel).

  bn(x) = gamma * (x - mean) / sqrt(var + 1e-5) + beta, parameters stored as
  four consecutive vectors [gamma, beta, mean, var].
"""
import math

CONV, DWCONV, MAXPOOL, AVGPOOL, GAP, FC, SE = 1, 2, 3, 4, 5, 6, 7
ACT_NONE, ACT_RELU, ACT_SILU = 0, 1, 2
BN_EPS = 1e-5

OP_FIELDS = (
    "kind", "src", "src_c0", "cin", "dst", "dst_c0", "cout",
    "kh", "kw", "sh", "sw", "pt", "pl", "act", "res", "res_c0", "pre", "r",
    "off_w", "off_b", "off_bn", "off_pre", "off_w2", "off_b2",
)

_ACT = {None: ACT_NONE, "none": ACT_NONE, "relu": ACT_RELU, "silu": ACT_SILU}


class Net:
    """Builder and container of one member description."""

    def __init__(self, name, in_h, in_w, classes, dtype="bf16", in_c=3):
        self.name = name
        self.in_h, self.in_w, self.in_c = in_h, in_w, in_c
        self.classes = classes
        self.dtype = dtype
        self.tensors = [(in_h, in_w, in_c)]
        self.ops = []
        self.params = []       # dicts: role, offset, size, + generation arguments
        self.blob_size = 0
        self.out_tensor = -1

    # ---- bookkeeping -------------------------------------------------
    def tensor(self, h, w, c):
        self.tensors.append((int(h), int(w), int(c)))
        return len(self.tensors) - 1

    def _param(self, role, size, **kw):
        off = self.blob_size
        self.params.append(dict(role=role, offset=off, size=int(size), index=len(self.params), **kw))
        self.blob_size += int(size)
        return off

    def _op(self, **kw):
        op = {f: 0 for f in OP_FIELDS}
        op.update(res=-1, off_w=-1, off_b=-1, off_bn=-1, off_pre=-1, off_w2=-1, off_b2=-1)
        op.update(kw)
        self.ops.append(op)
        return op

    def _bn(self, c, gamma):
        return self._param("bn", 4 * c, channels=c, gamma=float(gamma))

    @staticmethod
    def _out(size, k, s, p_lo, p_hi):
        return (size + p_lo + p_hi - k) // s + 1

    # ---- operations --------------------------------------------------
    def conv(self, src, cout, k, stride=1, pad="same", bn=True, act="relu", bias=None,
             res=None, pre=False, gamma=1.0, gain=2.0, dst=None, src_slice=None, groups=1):
        kh, kw = (k, k) if isinstance(k, int) else k
        h, w, c_all = self.tensors[src]
        c0, cin = (0, c_all) if src_slice is None else src_slice
        if pad == "same":
            ph, pw = (kh - 1) // 2, (kw - 1) // 2
        elif pad == "valid":
            ph, pw = 0, 0
        else:
            ph, pw = pad
        ho, wo = self._out(h, kh, stride, ph, ph), self._out(w, kw, stride, pw, pw)
        if dst is None:
            dt, d0 = self.tensor(ho, wo, cout), 0
        else:
            dt, d0 = dst
            assert self.tensors[dt][:2] == (ho, wo), (self.tensors[dt], ho, wo)
            assert d0 + cout <= self.tensors[dt][2]
        if bias is None:
            bias = not bn
        assert cin % groups == 0 and cout % groups == 0
        fan_in = kh * kw * cin // groups
        off_w = self._param("conv_w", fan_in * cout, std=math.sqrt(gain / fan_in))
        off_b = self._param("bias", cout) if bias else -1
        off_bn = self._bn(cout, gamma) if bn else -1
        off_pre = self._bn(cin, 1.0) if pre else -1
        rt, r0 = (-1, 0) if res is None else (res if isinstance(res, tuple) else (res, 0))
        if rt >= 0:
            assert self.tensors[rt][:2] == (ho, wo) and r0 + cout <= self.tensors[rt][2]
        self._op(kind=CONV, src=src, src_c0=c0, cin=cin, dst=dt, dst_c0=d0, cout=cout,
                 kh=kh, kw=kw, sh=stride, sw=stride, pt=ph, pl=pw, act=_ACT[act],
                 res=rt, res_c0=r0, pre=int(pre), r=groups if groups > 1 else 0, off_w=off_w, off_b=off_b,
                 off_bn=off_bn, off_pre=off_pre)
        return dt

    def dwconv(self, src, k, stride=1, bn=True, act="silu", gain=2.0):
        h, w, c = self.tensors[src]
        p = (k - 1) // 2
        ho, wo = self._out(h, k, stride, p, p), self._out(w, k, stride, p, p)
        dt = self.tensor(ho, wo, c)
        off_w = self._param("conv_w", k * k * c, std=math.sqrt(gain / (k * k)))
        off_b = -1 if bn else self._param("bias", c)
        off_bn = self._bn(c, 1.0) if bn else -1
        self._op(kind=DWCONV, src=src, cin=c, dst=dt, cout=c, kh=k, kw=k, sh=stride, sw=stride,
                 pt=p, pl=p, act=_ACT[act], off_w=off_w, off_b=off_b, off_bn=off_bn)
        return dt

    def pool(self, kind, src, k, stride, pad=0, dst=None):
        h, w, c = self.tensors[src]
        ho, wo = self._out(h, k, stride, pad, pad), self._out(w, k, stride, pad, pad)
        if dst is None:
            dt, d0 = self.tensor(ho, wo, c), 0
        else:
            dt, d0 = dst
            assert self.tensors[dt][:2] == (ho, wo) and d0 + c <= self.tensors[dt][2]
        self._op(kind=kind, src=src, cin=c, dst=dt, dst_c0=d0, cout=c, kh=k, kw=k,
                 sh=stride, sw=stride, pt=pad, pl=pad)
        return dt

    def maxpool(self, src, k, stride, pad=0, dst=None):
        return self.pool(MAXPOOL, src, k, stride, pad, dst)

    def avgpool(self, src, k, stride, pad=0, dst=None):
        return self.pool(AVGPOOL, src, k, stride, pad, dst)

    def gap(self, src, pre=False):
        h, w, c = self.tensors[src]
        dt = self.tensor(1, 1, c)
        off_pre = self._bn(c, 1.0) if pre else -1
        self._op(kind=GAP, src=src, cin=c, dst=dt, cout=c, kh=h, kw=w, sh=1, sw=1,
                 pre=int(pre), off_pre=off_pre)
        return dt

    def fc(self, src, cout, gain=1.0):
        h, w, c = self.tensors[src]
        assert (h, w) == (1, 1)
        dt = self.tensor(1, 1, cout)
        off_w = self._param("conv_w", c * cout, std=math.sqrt(gain / c))
        off_b = self._param("bias", cout)
        self._op(kind=FC, src=src, cin=c, dst=dt, cout=cout, kh=1, kw=1, sh=1, sw=1,
                 off_w=off_w, off_b=off_b)
        self.out_tensor = dt
        return dt

    def se(self, src, r):
        h, w, c = self.tensors[src]
        dt = self.tensor(h, w, c)
        off_w = self._param("conv_w", c * r, std=math.sqrt(2.0 / c))
        off_b = self._param("bias", r)
        off_w2 = self._param("conv_w", r * c, std=math.sqrt(2.0 / r))
        off_b2 = self._param("bias", c)
        self._op(kind=SE, src=src, cin=c, dst=dt, cout=c, kh=h, kw=w, sh=1, sw=1, r=r,
                 off_w=off_w, off_b=off_b, off_w2=off_w2, off_b2=off_b2)
        return dt

    # ---- derived figures --------------------------------------------
    def macs(self):
        """Multiply-accumulates per image of the convolutions and FC layers."""
        total = 0
        for op in self.ops:
            ho, wo, _ = self.tensors[op["dst"]]
            if op["kind"] == CONV:
                total += ho * wo * op["cout"] * op["kh"] * op["kw"] * op["cin"] // max(1, op["r"])
            elif op["kind"] == DWCONV:
                total += ho * wo * op["cout"] * op["kh"] * op["kw"]
            elif op["kind"] == FC:
                total += op["cin"] * op["cout"]
            elif op["kind"] == SE:
                total += 2 * op["cin"] * op["r"]
        return total

    def n_weights(self):
        return sum(p["size"] for p in self.params if p["role"] in ("conv_w", "bias"))


# ----------------------------------------------------------------------
# Architectures
# ----------------------------------------------------------------------

RES_ALPHA = 0.25   # gamma of the last norm of every residual branch (keeps the stream variance bounded)


def tiny_a(classes=10, size=32):
    n = Net("tiny_a", size, size, classes, dtype="fp32")
    t = n.conv(0, 16, 3)
    t = n.maxpool(t, 2, 2)
    t = n.conv(t, 32, 3)
    t = n.gap(t)
    n.fc(t, classes)
    return n


def tiny_b(classes=10, size=32):
    n = Net("tiny_b", size, size, classes, dtype="fp32")
    t = n.conv(0, 8, 5, bn=False)
    t = n.avgpool(t, 2, 2)
    t = n.conv(t, 16, 3, bn=False)
    t = n.gap(t)
    n.fc(t, classes)
    return n


def _resnet_stem(n, width=64):
    t = n.conv(0, width, 7, stride=2)
    return n.maxpool(t, 3, 2, 1)


def resnet_basic(name, blocks, classes=1000, size=224, widths=(64, 128, 256, 512), dtype="bf16"):
    n = Net(name, size, size, classes, dtype)
    t = _resnet_stem(n, widths[0])
    cin = widths[0]
    for si, (w, nb) in enumerate(zip(widths, blocks)):
        for bi in range(nb):
            s = 2 if (bi == 0 and si > 0) else 1
            idt = t
            if s != 1 or cin != w:
                idt = n.conv(t, w, 1, stride=s, act=None)
            u = n.conv(t, w, 3, stride=s)
            t = n.conv(u, w, 3, gamma=RES_ALPHA, res=idt)
            cin = w
    t = n.gap(t)
    n.fc(t, classes)
    return n


def resnet_bottleneck(name, blocks, classes=1000, size=224, widths=(64, 128, 256, 512), dtype="bf16"):
    """Bottleneck residual network; the stride sits on the 3x3 convolution."""
    n = Net(name, size, size, classes, dtype)
    t = _resnet_stem(n, 64)
    cin = 64
    for si, (w, nb) in enumerate(zip(widths, blocks)):
        for bi in range(nb):
            s = 2 if (bi == 0 and si > 0) else 1
            idt = t
            if s != 1 or cin != 4 * w:
                idt = n.conv(t, 4 * w, 1, stride=s, act=None)
            u = n.conv(t, w, 1)
            u = n.conv(u, w, 3, stride=s)
            t = n.conv(u, 4 * w, 1, gamma=RES_ALPHA, res=idt)
            cin = 4 * w
    t = n.gap(t)
    # the residual stream's spread grows about 6 % per block; the head is scaled so that the
    # logits keep a spread of about 3 whatever the depth (no saturated softmax)
    n.fc(t, classes, gain=0.25 * 1.126 ** (16 - sum(blocks)))
    return n


def resnext50(classes=1000, size=224, dtype="bf16", groups=32, width=4):
    """ResNeXt-50 (32x4d)-shaped member: the bottleneck network with a grouped 3x3 convolution of
    `groups` groups, `width` channels per group in the first stage (doubling per stage)."""
    n = Net("resnext50", size, size, classes, dtype)
    t = _resnet_stem(n, 64)
    cin = 64
    for si, (w, nb) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        gw = groups * width * 2 ** si
        for bi in range(nb):
            s = 2 if (bi == 0 and si > 0) else 1
            idt = t
            if s != 1 or cin != 4 * w:
                idt = n.conv(t, 4 * w, 1, stride=s, act=None)
            u = n.conv(t, gw, 1)
            u = n.conv(u, gw, 3, stride=s, groups=groups)
            t = n.conv(u, 4 * w, 1, gamma=RES_ALPHA, res=idt)
            cin = 4 * w
    t = n.gap(t)
    n.fc(t, classes, gain=0.25)
    return n


def resnet18(**kw):
    return resnet_basic("resnet18", (2, 2, 2, 2), **kw)


def resnet34(**kw):
    return resnet_basic("resnet34", (3, 4, 6, 3), **kw)


def resnet50(**kw):
    return resnet_bottleneck("resnet50", (3, 4, 6, 3), **kw)


def resnet101(**kw):
    return resnet_bottleneck("resnet101", (3, 4, 23, 3), **kw)


def resnet152(**kw):
    return resnet_bottleneck("resnet152", (3, 8, 36, 3), **kw)


def densenet(name, blocks, growth=32, bn_size=4, classes=1000, size=224, dtype="bf16"):
    """Pre-activation dense blocks; a block's tensor is allocated at its final
    width and every layer appends its `growth` channels in place."""
    n = Net(name, size, size, classes, dtype)
    t = n.conv(0, 2 * growth, 7, stride=2)
    h, w, c = n.tensors[t]
    ho, wo = n._out(h, 3, 2, 1, 1), n._out(w, 3, 2, 1, 1)
    blk = n.tensor(ho, wo, c + blocks[0] * growth)
    n.maxpool(t, 3, 2, 1, dst=(blk, 0))
    for bi, nl in enumerate(blocks):
        for _ in range(nl):
            u = n.conv(blk, bn_size * growth, 1, pre=True, src_slice=(0, c))
            n.conv(u, growth, 3, bn=False, act=None, bias=False, dst=(blk, c))
            c += growth
        if bi + 1 < len(blocks):
            u = n.conv(blk, c // 2, 1, pre=True, bn=False, act=None, bias=False)
            c //= 2
            h, w, _ = n.tensors[u]
            nxt = n.tensor(h // 2, w // 2, c + blocks[bi + 1] * growth)
            n.avgpool(u, 2, 2, dst=(nxt, 0))
            blk = nxt
    t = n.gap(blk, pre=True)
    n.fc(t, classes)
    return n


def densenet121(**kw):
    return densenet("densenet121", (6, 12, 24, 16), **kw)


def densenet169(**kw):
    return densenet("densenet169", (6, 12, 32, 32), **kw)


def densenet201(**kw):
    return densenet("densenet201", (6, 12, 48, 32), **kw)


def _round8(c):
    return max(8, int(c + 4) // 8 * 8)


_EFF_STAGES = ((1, 3, 1, 16, 1), (6, 3, 2, 24, 2), (6, 5, 2, 40, 2), (6, 3, 2, 80, 3),
               (6, 5, 1, 112, 3), (6, 5, 2, 192, 4), (6, 3, 1, 320, 1))
_EFF_SCALE = {0: (1.0, 1.0), 1: (1.0, 1.1), 2: (1.1, 1.2), 3: (1.2, 1.4), 4: (1.4, 1.8)}


def efficientnet(variant=0, classes=1000, size=224, dtype="bf16"):
    """EfficientNet-B<variant>-shaped member (inverted residuals with depthwise
    convolutions, squeeze-excite at a quarter of the block input width, SiLU)."""
    wm, dm = _EFF_SCALE[variant]
    n = Net("efficientnet_b%d" % variant, size, size, classes, dtype)
    cin = _round8(32 * wm)
    t = n.conv(0, cin, 3, stride=2, act="silu")
    for (e, k, s, c, reps) in _EFF_STAGES:
        cout = _round8(c * wm)
        for i in range(int(math.ceil(reps * dm))):
            stride = s if i == 0 else 1
            x = t
            u = n.conv(x, cin * e, 1, act="silu") if e != 1 else x
            u = n.dwconv(u, k, stride)
            u = n.se(u, max(1, cin // 4))
            skip = x if (stride == 1 and cin == cout) else None
            t = n.conv(u, cout, 1, act=None, res=skip, gamma=RES_ALPHA if skip is not None else 1.0)
            cin = cout
    t = n.conv(t, _round8(1280 * wm), 1, act="silu")
    t = n.gap(t)
    n.fc(t, classes, gain=400.0)     # squeeze-excite gates and SiLU shrink the signal; keep logits O(1)
    return n


def inception_v3(classes=1000, size=299, dtype="bf16"):
    """Inception-v3-shaped member: factorised 1x7/7x1 and 1x3/3x1 branches,
    branch outputs written side by side into the module's output tensor."""
    n = Net("inception_v3", size, size, classes, dtype)
    t = n.conv(0, 32, 3, stride=2, pad="valid")
    t = n.conv(t, 32, 3, pad="valid")
    t = n.conv(t, 64, 3)
    t = n.maxpool(t, 3, 2)
    t = n.conv(t, 80, 1)
    t = n.conv(t, 192, 3, pad="valid")
    t = n.maxpool(t, 3, 2)

    def mod_a(x, pool_c):
        h, w, _ = n.tensors[x]
        o = n.tensor(h, w, 64 + 64 + 96 + pool_c)
        n.conv(x, 64, 1, dst=(o, 0))
        u = n.conv(x, 48, 1)
        n.conv(u, 64, 5, dst=(o, 64))
        u = n.conv(x, 64, 1)
        u = n.conv(u, 96, 3)
        n.conv(u, 96, 3, dst=(o, 128))
        u = n.avgpool(x, 3, 1, 1)
        n.conv(u, pool_c, 1, dst=(o, 224))
        return o

    def mod_b(x):
        h, w, c = n.tensors[x]
        ho, wo = (h - 3) // 2 + 1, (w - 3) // 2 + 1
        o = n.tensor(ho, wo, 384 + 96 + c)
        n.conv(x, 384, 3, stride=2, pad="valid", dst=(o, 0))
        u = n.conv(x, 64, 1)
        u = n.conv(u, 96, 3)
        n.conv(u, 96, 3, stride=2, pad="valid", dst=(o, 384))
        n.maxpool(x, 3, 2, dst=(o, 480))
        return o

    def mod_c(x, c7):
        h, w, _ = n.tensors[x]
        o = n.tensor(h, w, 768)
        n.conv(x, 192, 1, dst=(o, 0))
        u = n.conv(x, c7, 1)
        u = n.conv(u, c7, (1, 7))
        n.conv(u, 192, (7, 1), dst=(o, 192))
        u = n.conv(x, c7, 1)
        u = n.conv(u, c7, (7, 1))
        u = n.conv(u, c7, (1, 7))
        u = n.conv(u, c7, (7, 1))
        n.conv(u, 192, (1, 7), dst=(o, 384))
        u = n.avgpool(x, 3, 1, 1)
        n.conv(u, 192, 1, dst=(o, 576))
        return o

    def mod_d(x):
        h, w, c = n.tensors[x]
        ho, wo = (h - 3) // 2 + 1, (w - 3) // 2 + 1
        o = n.tensor(ho, wo, 320 + 192 + c)
        u = n.conv(x, 192, 1)
        n.conv(u, 320, 3, stride=2, pad="valid", dst=(o, 0))
        u = n.conv(x, 192, 1)
        u = n.conv(u, 192, (1, 7))
        u = n.conv(u, 192, (7, 1))
        n.conv(u, 192, 3, stride=2, pad="valid", dst=(o, 320))
        n.maxpool(x, 3, 2, dst=(o, 512))
        return o

    def mod_e(x):
        h, w, _ = n.tensors[x]
        o = n.tensor(h, w, 2048)
        n.conv(x, 320, 1, dst=(o, 0))
        u = n.conv(x, 384, 1)
        n.conv(u, 384, (1, 3), dst=(o, 320))
        n.conv(u, 384, (3, 1), dst=(o, 704))
        u = n.conv(x, 448, 1)
        u = n.conv(u, 384, 3)
        n.conv(u, 384, (1, 3), dst=(o, 1088))
        n.conv(u, 384, (3, 1), dst=(o, 1472))
        u = n.avgpool(x, 3, 1, 1)
        n.conv(u, 192, 1, dst=(o, 1856))
        return o

    t = mod_a(t, 32)
    t = mod_a(t, 64)
    t = mod_a(t, 64)
    t = mod_b(t)
    for c7 in (128, 160, 160, 192):
        t = mod_c(t, c7)
    t = mod_d(t)
    t = mod_e(t)
    t = mod_e(t)
    t = n.gap(t)
    n.fc(t, classes, gain=0.15)
    return n


# ----------------------------------------------------------------------
# The five workload configurations
# ----------------------------------------------------------------------

_VGG = {16: (2, 2, 3, 3, 3), 19: (2, 2, 4, 4, 4)}


def vgg(depth=16, classes=1000, size=224, dtype="bf16"):
    """VGG-16 / VGG-19-shaped member: 3x3 convolutions with bias and no normalisation, five 2x2 max
    pools, two hidden fully connected layers of 4096.  The first of those is written as a
    convolution over the whole remaining map (7x7 at 224) and the second as a 1x1 convolution, which
    is what a fully connected layer over a flattened map is."""
    n = Net("vgg%d" % depth, size, size, classes, dtype)
    t, widths = 0, (64, 128, 256, 512, 512)
    for w, reps in zip(widths, _VGG[depth]):
        for _ in range(reps):
            t = n.conv(t, w, 3, bn=False)
        t = n.maxpool(t, 2, 2)
    h, w_, _ = n.tensors[t]
    t = n.conv(t, 4096, (h, w_), pad="valid", bn=False)
    t = n.conv(t, 4096, 1, bn=False)
    t = n.gap(t)
    n.fc(t, classes)
    return n


def xception(classes=1000, size=299, dtype="bf16"):
    """Xception-shaped member: depthwise-separable convolutions (3x3 depthwise without norm or
    activation, then 1x1 with norm) in residual blocks; entry flow 128-256-728 with strided max
    pools and 1x1 stride-2 shortcuts, eight middle blocks at 728, exit flow to 2048.  The ReLU
    that the architecture puts in front of a separable convolution sits behind the operation that
    feeds it here (the sum included), which keeps every shape and operation count."""
    n = Net("xception", size, size, classes, dtype)

    def sep(x, cout, act="relu", res=None, gamma=1.0):
        d = n.dwconv(x, 3, 1, bn=False, act=None, gain=1.0)
        return n.conv(d, cout, 1, act=act, res=res, gamma=gamma)

    t = n.conv(0, 32, 3, stride=2, pad="valid")
    t = n.conv(t, 64, 3, pad="valid")
    for c in (128, 256, 728):                                   # entry flow
        u = sep(t, c)
        u = sep(u, c, act=None, gamma=RES_ALPHA)
        u = n.maxpool(u, 3, 2, 1)
        t = n.conv(t, c, 1, stride=2, act="relu", res=u)        # shortcut + pooled branch
    for _ in range(8):                                           # middle flow
        u = sep(t, 728)
        u = sep(u, 728)
        t = sep(u, 728, act="relu", res=t, gamma=RES_ALPHA)
    u = sep(t, 728)                                              # exit flow
    u = sep(u, 1024, act=None, gamma=RES_ALPHA)
    u = n.maxpool(u, 3, 2, 1)
    t = n.conv(t, 1024, 1, stride=2, act=None, res=u)
    t = sep(t, 1536)
    t = sep(t, 2048)
    t = n.gap(t)
    n.fc(t, classes, gain=0.3)
    return n


_MBV2 = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1))


def mobilenet_v2(classes=1000, size=224, dtype="bf16"):
    """MobileNetV2-shaped member: inverted residuals (1x1 expansion, 3x3 depthwise, linear 1x1
    projection), widths 16-320, 1280 features.  ReLU stands where the architecture has ReLU6."""
    n = Net("mobilenet_v2", size, size, classes, dtype)
    cin = 32
    t = n.conv(0, cin, 3, stride=2)
    for (e, c, reps, s) in _MBV2:
        for i in range(reps):
            stride = s if i == 0 else 1
            x = t
            u = n.conv(x, cin * e, 1, gain=1.0) if e != 1 else x      # the block input is a linear projection: unit gain
            u = n.dwconv(u, 3, stride, act="relu")
            skip = x if (stride == 1 and cin == c) else None
            t = n.conv(u, c, 1, act=None, res=skip, gamma=RES_ALPHA if skip is not None else 1.0)
            cin = c
    t = n.conv(t, 1280, 1, gain=1.0)
    t = n.gap(t)
    n.fc(t, classes, gain=4.0)
    return n


def config_members(cfg):
    """Members of workload configuration `cfg` (1-9) as a list of Net."""
    if cfg == 1:
        return [tiny_a(), tiny_b()]
    if cfg == 2:
        return [resnet18(), resnet18(), resnet18()]
    if cfg == 3:
        return [resnet50(), inception_v3(size=299), efficientnet(0), densenet121()]
    if cfg == 4:
        return [resnet50(), resnet101(), resnet152(),
                efficientnet(0), efficientnet(2), efficientnet(4),
                densenet121(), densenet169(), densenet201(),
                inception_v3(size=224), inception_v3(size=224), inception_v3(size=224)]
    if cfg == 5:
        return [resnet50()]
    if cfg == 6:        # further members of the paper's ImageNet ensembles: VGG, ResNeXt, Xception, MobileNetV2 shapes
        return [vgg(16), vgg(19), resnext50(), xception(size=299), mobilenet_v2()]
    # the paper's own ImageNet ensembles (section "Experimental settings"), as shapes with synthetic weights
    if cfg == 7:        # IMN1
        return [resnet152()]
    if cfg == 8:        # IMN4
        return [resnet50(), resnet101(), densenet121(), vgg(19)]
    if cfg == 9:        # IMN12
        return [resnet152(), resnet50(), resnet101(), densenet121(), vgg(19), resnet18(), resnet34(), resnext50(),
                inception_v3(size=299), xception(size=299), vgg(16), mobilenet_v2()]
    raise ValueError("configuration must be 1..9")


BASE_SIZE = {1: 32, 2: 224, 3: 224, 4: 224, 5: 224, 6: 224, 7: 224, 8: 224, 9: 224}
