"""Operator graphs of the tenant models, written from the architectures' published layer tables.

Every builder returns a ModelSpec whose `ops` list is the serial order the
scheduler sees (paper Sec. III-B, Eq. 1 and its footnote on serialising
multi-branch models).  Residual adds are carried by the last convolution of a
branch (`res=`), channel concatenations by channel-offset writes.

Synthetic BN gain: the last convolution of every residual branch gets gain
0.25 so that activations of deep residual stacks stay inside fp16 range with
random weights.
"""
from .graph import GraphBuilder

RES_GAIN = 0.25


# ---------------------------------------------------------------- tiny nets
def tiny_a(dtype="f32", batch=1):
    g = GraphBuilder("tinyA", dtype, batch, 32, 32, 3)
    t = g.conv(0, 16, 3, pad=1)
    t = g.conv(t, 32, 3, pad=1)
    t = g.maxpool(t, 2, 2)
    t = g.conv(t, 32, 3, pad=1)
    t = g.conv(t, 64, 3, pad=1)
    t = g.maxpool(t, 2, 2)
    t = g.gap(t)
    g.fc(t, 10)
    return g.done()


def tiny_b(dtype="f32", batch=1):
    g = GraphBuilder("tinyB", dtype, batch, 32, 32, 3)
    t = g.conv(0, 32, 5)
    t = g.maxpool(t, 2, 2)
    t = g.conv(t, 64, 5)
    t = g.maxpool(t, 2, 2)
    g.fc(t, 10)
    return g.done()


def tiny_c(dtype="f32", batch=1):
    g = GraphBuilder("tinyC", dtype, batch, 32, 32, 3)
    t = g.conv(0, 16, 3, stride=2, pad=1)
    for ch in (32, 64, 128):
        t = g.dwconv(t, 3, 1, 1, act="relu")
        t = g.conv(t, ch, 1, act="relu")
    t = g.gap(t)
    g.fc(t, 10)
    return g.done()


# ------------------------------------------------------------------ ResNets
def _resnet_stem(g):
    t = g.conv(0, 64, 7, stride=2, pad=3, bn=True)
    return g.maxpool(t, 3, 2, 1)


def _basic_block(g, t, ch, stride):
    h, w, c = g.shapes[t]
    short = t
    if stride != 1 or c != ch:
        short = g.conv(t, ch, 1, stride=stride, act="none", bn=True)
    u = g.conv(t, ch, 3, stride=stride, pad=1, bn=True)
    return g.conv(u, ch, 3, pad=1, bn=True, gain=RES_GAIN, res=short, act="relu")


def _bottleneck(g, t, mid, stride):
    h, w, c = g.shapes[t]
    out = mid * 4
    short = t
    if stride != 1 or c != out:
        short = g.conv(t, out, 1, stride=stride, act="none", bn=True)
    u = g.conv(t, mid, 1, bn=True)
    u = g.conv(u, mid, 3, stride=stride, pad=1, bn=True)     # stride sits on the 3x3
    return g.conv(u, out, 1, bn=True, gain=RES_GAIN, res=short, act="relu")


def _resnet(name, block, layers, dtype, batch, classes=1000):
    g = GraphBuilder(name, dtype, batch, 224, 224, 3)
    t = _resnet_stem(g)
    for i, n in enumerate(layers):
        for j in range(n):
            stride = 2 if (i > 0 and j == 0) else 1
            t = block(g, t, 64 << i, stride)
    t = g.gap(t)
    g.fc(t, classes)
    return g.done()


def resnet18(dtype="f16", batch=1):
    return _resnet("resnet18", _basic_block, (2, 2, 2, 2), dtype, batch)


def resnet34(dtype="f16", batch=1):
    return _resnet("resnet34", _basic_block, (3, 4, 6, 3), dtype, batch)


def resnet50(dtype="f16", batch=1):
    return _resnet("resnet50", _bottleneck, (3, 4, 6, 3), dtype, batch)


def resnet101(dtype="f16", batch=1):
    return _resnet("resnet101", _bottleneck, (3, 4, 23, 3), dtype, batch)


# -------------------------------------------------------------------- VGG-16
def vgg16(dtype="f16", batch=1):
    g = GraphBuilder("vgg16", dtype, batch, 224, 224, 3)
    t = 0
    for ch, n in ((64, 2), (128, 2), (256, 3), (512, 3), (512, 3)):
        for _ in range(n):
            t = g.conv(t, ch, 3, pad=1)
        t = g.maxpool(t, 2, 2)
    t = g.fc(t, 4096, act="relu")
    t = g.fc(t, 4096, act="relu")
    g.fc(t, 1000)
    return g.done()


# ------------------------------------------------------------------- AlexNet
def alexnet(dtype="bf16", batch=1):
    """Original layer widths at 227x227, one group, no LRN / dropout / softmax."""
    g = GraphBuilder("alexnet", dtype, batch, 227, 227, 3)
    t = g.conv(0, 96, 11, stride=4)
    t = g.maxpool(t, 3, 2)
    t = g.conv(t, 256, 5, pad=2)
    t = g.maxpool(t, 3, 2)
    t = g.conv(t, 384, 3, pad=1)
    t = g.conv(t, 384, 3, pad=1)
    t = g.conv(t, 256, 3, pad=1)
    t = g.maxpool(t, 3, 2)
    t = g.fc(t, 4096, act="relu")
    t = g.fc(t, 4096, act="relu")
    g.fc(t, 1000)
    return g.done()


def alexnet_published(dtype="bf16", batch=1):
    """AlexNet as its paper prints it: two filter groups in conv2, conv4 and conv5, local response
    normalisation (5 channels, k = 2, alpha = 1e-4, beta = 0.75) after conv1 and conv2; no dropout / softmax."""
    g = GraphBuilder("alexnet_published", dtype, batch, 227, 227, 3)
    t = g.conv(0, 96, 11, stride=4)
    t = g.lrn(t)
    t = g.maxpool(t, 3, 2)
    t = g.conv(t, 256, 5, pad=2, groups=2)
    t = g.lrn(t)
    t = g.maxpool(t, 3, 2)
    t = g.conv(t, 384, 3, pad=1)
    t = g.conv(t, 384, 3, pad=1, groups=2)
    t = g.conv(t, 256, 3, pad=1, groups=2)
    t = g.maxpool(t, 3, 2)
    t = g.fc(t, 4096, act="relu")
    t = g.fc(t, 4096, act="relu")
    g.fc(t, 1000)
    return g.done()


def tiny_d(dtype="f32", batch=1):
    """A small residual net whose shortcut sum is an operator of its own (not fused into a convolution),
    with a grouped convolution and a local response normalisation."""
    g = GraphBuilder("tinyD", dtype, batch, 24, 24, 8)
    t = g.conv(0, 32, 3, pad=1)
    u = g.conv(t, 32, 3, pad=1, groups=4)
    u = g.conv(u, 32, 1, act="none")
    t = g.add(u, t, act="relu")
    t = g.lrn(t, size=3, alpha=2e-2, beta=0.75, k=1.0)
    t = g.maxpool(t, 2, 2)
    t = g.gap(t)
    g.fc(t, 10)
    return g.done()


# --------------------------------------------------------------- MobileNetV2
def mobilenet_v2(dtype="f16", batch=1):
    g = GraphBuilder("mobilenetv2", dtype, batch, 224, 224, 3)
    t = g.conv(0, 32, 3, stride=2, pad=1, act="relu6", bn=True)
    table = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
             (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1))
    for expand, ch, n, s in table:
        for j in range(n):
            stride = s if j == 0 else 1
            h, w, c = g.shapes[t]
            u = t
            if expand != 1:
                u = g.conv(u, c * expand, 1, act="relu6", bn=True)
            u = g.dwconv(u, 3, stride, 1, act="relu6", bn=True)
            if stride == 1 and c == ch:
                t = g.conv(u, ch, 1, act="none", bn=True, gain=RES_GAIN, res=t)
            else:
                t = g.conv(u, ch, 1, act="none", bn=True)
    t = g.conv(t, 1280, 1, act="relu6", bn=True)
    t = g.gap(t)
    g.fc(t, 1000)
    return g.done()


# -------------------------------------------------------------- Inception-v3
def inception_v3(dtype="bf16", batch=1):
    """299x299 inference graph, no auxiliary head.  Branches are serialised in
    the order 1x1, 5x5 / 7x7, double 3x3 / double 7x7, pool; each branch's last
    operator writes into the concatenated tensor at its channel offset."""
    g = GraphBuilder("inceptionv3", dtype, batch, 299, 299, 3)

    def c(src, ch, k, stride=1, pad=0, **kw):
        return g.conv(src, ch, k, stride=stride, pad=pad, bn=True, **kw)

    t = c(0, 32, 3, stride=2)
    t = c(t, 32, 3)
    t = c(t, 64, 3, pad=1)
    t = g.maxpool(t, 3, 2)
    t = c(t, 80, 1)
    t = c(t, 192, 3)
    t = g.maxpool(t, 3, 2)

    def block_a(t, pool_ch):
        tot = 64 + 64 + 96 + pool_ch
        d = g.new_tensor()
        c(t, 64, 1, dst=d, c_off=0, c_tot=tot)
        u = c(t, 48, 1)
        c(u, 64, 5, pad=2, dst=d, c_off=64, c_tot=tot)
        u = c(t, 64, 1)
        u = c(u, 96, 3, pad=1)
        c(u, 96, 3, pad=1, dst=d, c_off=128, c_tot=tot)
        u = g.avgpool(t, 3, 1, 1)
        c(u, pool_ch, 1, dst=d, c_off=224, c_tot=tot)
        return d

    def block_b(t):
        h, w, cin = g.shapes[t]
        tot = 384 + 96 + cin
        d = g.new_tensor()
        c(t, 384, 3, stride=2, dst=d, c_off=0, c_tot=tot)
        u = c(t, 64, 1)
        u = c(u, 96, 3, pad=1)
        c(u, 96, 3, stride=2, dst=d, c_off=384, c_tot=tot)
        g.maxpool(t, 3, 2, dst=d, c_off=480, c_tot=tot)
        return d

    def block_c(t, c7):
        tot = 768
        d = g.new_tensor()
        c(t, 192, 1, dst=d, c_off=0, c_tot=tot)
        u = c(t, c7, 1)
        u = c(u, c7, (1, 7), pad=(0, 3))
        c(u, 192, (7, 1), pad=(3, 0), dst=d, c_off=192, c_tot=tot)
        u = c(t, c7, 1)
        u = c(u, c7, (7, 1), pad=(3, 0))
        u = c(u, c7, (1, 7), pad=(0, 3))
        u = c(u, c7, (7, 1), pad=(3, 0))
        c(u, 192, (1, 7), pad=(0, 3), dst=d, c_off=384, c_tot=tot)
        u = g.avgpool(t, 3, 1, 1)
        c(u, 192, 1, dst=d, c_off=576, c_tot=tot)
        return d

    def block_d(t):
        h, w, cin = g.shapes[t]
        tot = 320 + 192 + cin
        d = g.new_tensor()
        u = c(t, 192, 1)
        c(u, 320, 3, stride=2, dst=d, c_off=0, c_tot=tot)
        u = c(t, 192, 1)
        u = c(u, 192, (1, 7), pad=(0, 3))
        u = c(u, 192, (7, 1), pad=(3, 0))
        c(u, 192, 3, stride=2, dst=d, c_off=320, c_tot=tot)
        g.maxpool(t, 3, 2, dst=d, c_off=512, c_tot=tot)
        return d

    def block_e(t):
        tot = 2048
        d = g.new_tensor()
        c(t, 320, 1, dst=d, c_off=0, c_tot=tot)
        u = c(t, 384, 1)
        c(u, 384, (1, 3), pad=(0, 1), dst=d, c_off=320, c_tot=tot)
        c(u, 384, (3, 1), pad=(1, 0), dst=d, c_off=704, c_tot=tot)
        u = c(t, 448, 1)
        u = c(u, 384, 3, pad=1)
        c(u, 384, (1, 3), pad=(0, 1), dst=d, c_off=1088, c_tot=tot)
        c(u, 384, (3, 1), pad=(1, 0), dst=d, c_off=1472, c_tot=tot)
        u = g.avgpool(t, 3, 1, 1)
        c(u, 192, 1, dst=d, c_off=1856, c_tot=tot)
        return d

    t = block_a(t, 32)
    t = block_a(t, 64)
    t = block_a(t, 64)
    t = block_b(t)
    for c7 in (128, 160, 160, 192):
        t = block_c(t, c7)
    t = block_d(t)
    t = block_e(t)
    t = block_e(t)
    t = g.gap(t)
    g.fc(t, 1000)
    return g.done()


BUILDERS = {
    "tinyA": tiny_a, "tinyB": tiny_b, "tinyC": tiny_c,
    "resnet18": resnet18, "resnet34": resnet34, "resnet50": resnet50, "resnet101": resnet101,
    "vgg16": vgg16, "alexnet": alexnet, "mobilenetv2": mobilenet_v2, "inceptionv3": inception_v3,
    "alexnet_published": alexnet_published, "tinyD": tiny_d,
}
