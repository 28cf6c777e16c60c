"""Workload definitions: the network shapes the benchmark and the tests run on.

Plain data only (layer lists); no arithmetic of the method lives here.  Both the oracle and
the HIP library consume these descriptions through their own code.

A network is a dict:
  name, batch, in_c, in_h, in_w, layers
and each layer is a dict:
  type   : "conv" | "relu" | "maxpool" | "avgpool" | "fc" | "concat" | "softmax_ce"
  inputs : list of producer layer ids (-1 = the network input)
  out    : output channels (conv) / output features (fc)
  k, stride, pad : window geometry (conv, pools)
"""


class _Builder:
    def __init__(self, name, batch, in_c, in_h, in_w):
        self.net = dict(name=name, batch=batch, in_c=in_c, in_h=in_h, in_w=in_w, layers=[])
        self.last = -1

    def add(self, type_, inputs=None, **kw):
        layer = dict(type=type_, inputs=[self.last] if inputs is None else list(inputs), out=0, k=0, stride=1, pad=0)
        layer.update(kw)
        self.net["layers"].append(layer)
        self.last = len(self.net["layers"]) - 1
        return self.last

    def conv(self, out, k, stride=1, pad=0, relu=True, inputs=None):
        i = self.add("conv", inputs, out=out, k=k, stride=stride, pad=pad)
        if relu:
            i = self.add("relu")
        return i

    def fc(self, out, relu=True):
        i = self.add("fc", out=out)
        if relu:
            i = self.add("relu")
        return i

    def maxpool(self, k, stride, pad=0, inputs=None):
        return self.add("maxpool", inputs, k=k, stride=stride, pad=pad)

    def avgpool(self, k, stride, pad=0):
        return self.add("avgpool", k=k, stride=stride, pad=pad)

    def done(self):
        self.add("softmax_ce")
        return self.net


def tiny(batch=8):
    b = _Builder("tiny", batch, 3, 32, 32)
    b.conv(16, 3, pad=1)
    b.maxpool(2, 2)
    b.conv(32, 3, pad=1)
    b.maxpool(2, 2)
    b.fc(10, relu=False)
    return b.done()


def alexnet(batch=128):
    b = _Builder("alexnet", batch, 3, 227, 227)
    b.conv(96, 11, stride=4)
    b.maxpool(3, 2)
    b.conv(256, 5, pad=2)
    b.maxpool(3, 2)
    b.conv(384, 3, pad=1)
    b.conv(384, 3, pad=1)
    b.conv(256, 3, pad=1)
    b.maxpool(3, 2)
    b.fc(4096)
    b.fc(4096)
    b.fc(1000, relu=False)
    return b.done()


def overfeat(batch=128):
    b = _Builder("overfeat", batch, 3, 231, 231)
    b.conv(96, 11, stride=4)
    b.maxpool(2, 2)
    b.conv(256, 5)
    b.maxpool(2, 2)
    b.conv(512, 3, pad=1)
    b.conv(1024, 3, pad=1)
    b.conv(1024, 3, pad=1)
    b.maxpool(2, 2)
    b.fc(3072)
    b.fc(4096)
    b.fc(1000, relu=False)
    return b.done()


# (1x1, 3x3 reduce, 3x3, 5x5 reduce, 5x5, pool projection) per inception module
_INCEPTION = [
    ("3a", 64, 96, 128, 16, 32, 32),
    ("3b", 128, 128, 192, 32, 96, 64),
    ("pool", 0, 0, 0, 0, 0, 0),
    ("4a", 192, 96, 208, 16, 48, 64),
    ("4b", 160, 112, 224, 24, 64, 64),
    ("4c", 128, 128, 256, 24, 64, 64),
    ("4d", 112, 144, 288, 32, 64, 64),
    ("4e", 256, 160, 320, 32, 128, 128),
    ("pool", 0, 0, 0, 0, 0, 0),
    ("5a", 256, 160, 320, 32, 128, 128),
    ("5b", 384, 192, 384, 48, 128, 128),
]


def googlenet(batch=128, in_hw=224, modules=None):
    b = _Builder("googlenet", batch, 3, in_hw, in_hw)
    b.conv(64, 7, stride=2, pad=3)
    b.maxpool(3, 2, pad=1)
    b.conv(64, 1)
    b.conv(192, 3, pad=1)
    src = b.maxpool(3, 2, pad=1)
    for name, c1, r3, c3, r5, c5, pp in (_INCEPTION if modules is None else modules):
        if name == "pool":
            src = b.maxpool(3, 2, pad=1, inputs=[src])
            continue
        a = b.conv(c1, 1, inputs=[src])
        t = b.conv(r3, 1, inputs=[src])
        bb = b.conv(c3, 3, pad=1, inputs=[t])
        t = b.conv(r5, 1, inputs=[src])
        cc = b.conv(c5, 5, pad=2, inputs=[t])
        t = b.maxpool(3, 1, pad=1, inputs=[src])
        dd = b.conv(pp, 1, inputs=[t])
        src = b.add("concat", [a, bb, cc, dd])
    b.avgpool(in_hw // 32, 1)
    b.fc(1000, relu=False)
    return b.done()


def vgg(batch=256, extra_per_group=0, in_hw=224, widths=(64, 128, 256, 512, 512), fc=(4096, 4096, 1000)):
    """VGG-16 for extra_per_group=0; 20 extra convs per group per +100 layers gives the
    very deep VGG-116/216/316/416 variants."""
    base = (2, 2, 3, 3, 3)
    name = "vgg%d" % (16 + 5 * extra_per_group)
    b = _Builder(name, batch, 3, in_hw, in_hw)
    for g, width in enumerate(widths):
        for _ in range(base[g] + extra_per_group):
            b.conv(width, 3, pad=1)
        b.maxpool(2, 2)
    for i, f in enumerate(fc):
        b.fc(f, relu=(i + 1 < len(fc)))
    return b.done()


def vgg16(batch=256):
    return vgg(batch)


def fork_join(batch=4):
    """Small non-linear net (one inception-style module) for graph tests."""
    mods = [("m", 8, 4, 8, 4, 8, 8)]
    b = _Builder("forkjoin", batch, 3, 16, 16)
    src = b.conv(8, 3, pad=1)
    for name, c1, r3, c3, r5, c5, pp in mods:
        a = b.conv(c1, 1, inputs=[src])
        t = b.conv(r3, 1, inputs=[src])
        bb = b.conv(c3, 3, pad=1, inputs=[t])
        t = b.conv(r5, 1, inputs=[src])
        cc = b.conv(c5, 5, pad=2, inputs=[t])
        t = b.maxpool(3, 1, pad=1, inputs=[src])
        dd = b.conv(pp, 1, inputs=[t])
        src = b.add("concat", [a, bb, cc, dd])
    b.avgpool(4, 4)
    b.fc(10, relu=False)
    return b.done()


CONFIGS = {
    "tiny": tiny,
    "alexnet": alexnet,
    "overfeat": overfeat,
    "googlenet": googlenet,
    "vgg16": vgg16,
}


def shapes(net):
    """Per-layer output shapes (N, C, H, W) and weight shapes, from the window geometry.
    Pure shape bookkeeping so that the generators know how many numbers to draw."""
    n = net["batch"]
    out, wshape = [], []
    def shp(i):
        return (n, net["in_c"], net["in_h"], net["in_w"]) if i < 0 else out[i]
    for layer in net["layers"]:
        ins = [shp(i) for i in layer["inputs"]]
        _, c, h, w = ins[0]
        t = layer["type"]
        k, st, pd = layer["k"], layer["stride"], layer["pad"]
        if t == "conv":
            out.append((n, layer["out"], (h + 2 * pd - k) // st + 1, (w + 2 * pd - k) // st + 1))
            wshape.append((layer["out"], c, k, k))
        elif t in ("maxpool", "avgpool"):
            out.append((n, c, (h + 2 * pd - k) // st + 1, (w + 2 * pd - k) // st + 1))
            wshape.append(None)
        elif t == "fc":
            out.append((n, layer["out"], 1, 1))
            wshape.append((layer["out"], c * h * w))
        elif t == "concat":
            out.append((n, sum(s[1] for s in ins), h, w))
            wshape.append(None)
        elif t == "relu":
            out.append(ins[0])
            wshape.append(None)
        elif t == "softmax_ce":
            out.append((1, 1, 1, 1))
            wshape.append(None)
        else:
            raise ValueError(t)
    return out, wshape


def random_net(seed, batch=2, in_hw=20, max_layers=10, wide=False):
    """A random small network for fuzzing the planners and the kernels on irregular graphs: chains of
    conv / pool layers with random geometry, conv layers without a ReLU, forks whose branches are joined
    by a concat (branches of different depth, a feature map read by several layers), FC head.
    wide: channel counts of 128 ... 384 instead of 4 ... 24 (layers wide enough for every convolution algorithm)."""
    import random
    rnd = random.Random(seed)
    cw = 32 if wide else 1   # 4, 8 -> 128, 256; 16 -> 512; 24 -> 768
    b = _Builder("random%d%s" % (seed, "w" if wide else ""), batch, 256 if wide else rnd.choice((1, 3, 4)), in_hw, in_hw + rnd.choice((0, 3)))
    h, w = b.net["in_h"], b.net["in_w"]
    src = -1
    n = 0
    while n < max_layers and min(h, w) >= 4:
        kind = rnd.random()
        if kind < 0.45:      # conv, same-size
            k = rnd.choice((1, 3, 3, 5))
            src = b.conv(rnd.choice((4, 8, 8, 12) if wide else (4, 8, 16, 24)) * cw, k, pad=k // 2, relu=rnd.random() < 0.8, inputs=[src])
        elif kind < 0.6:     # strided or unpadded conv
            k = rnd.choice((2, 3))
            st = rnd.choice((1, 2))
            src = b.conv(rnd.choice((4, 8) if wide else (8, 16)) * cw, k, stride=st, pad=0, inputs=[src])
            h, w = (h - k) // st + 1, (w - k) // st + 1
        elif kind < 0.75:    # pool
            k, st, pd = rnd.choice(((2, 2, 0), (3, 2, 1), (3, 1, 1), (3, 2, 0)))
            if rnd.random() < 0.8:
                src = b.maxpool(k, st, pd, inputs=[src])
            else:
                b.last = src
                src = b.avgpool(k, st, pd)
            h, w = (h + 2 * pd - k) // st + 1, (w + 2 * pd - k) // st + 1
        else:                # fork: 2-3 branches of depth 1-2 over the same source, joined by a concat
            outs = []
            for _ in range(rnd.choice((2, 3))):
                t = src
                for _ in range(rnd.choice((1, 2))):
                    k = rnd.choice((1, 3))
                    t = b.conv(rnd.choice((4, 8)) * cw, k, pad=k // 2, relu=rnd.random() < 0.7, inputs=[t])
                outs.append(t)
            if rnd.random() < 0.5:
                t = b.maxpool(3, 1, 1, inputs=[src])
                outs.append(b.conv(4 * cw, 1, inputs=[t]))
            src = b.add("concat", outs)
        n += 1
    b.last = src
    if rnd.random() < 0.5:
        b.fc(rnd.choice((8, 16)))
    b.fc(rnd.choice((3, 5, 10)), relu=False)
    return b.done()
