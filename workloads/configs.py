"""Layer lists of the benchmark workloads, as plain dicts, and their seeded tensors.

A layer dict has the keys
  kind      'conv' | 'fc' | 'maxpool2' | 'gap' | 'softmax_ce' | 'attn'
  cin, cout, kh, kw, stride, pad, h_in, w_in
  d_in, kd, pad_d       volumetric convolutions only (defaults 1, 1, 0): input depth, filter depth, depth padding
  relu, bias, scale     booleans (scale = frozen per-channel multiplier, i.e. a folded BatchNorm)
  src       index of the layer whose output is this layer's input (-1 = network input)
  add_src   index of the layer whose output is added before the ReLU, or None
  cut_after whether a partition boundary may follow this layer
Logical tensor layouts: activations [N][C][H][W], weights [Cout][Cin][Kh][Kw]; an
'fc' layer sees its input flattened in (C,H,W) order, i.e. it is a conv whose kernel
covers the whole input.  All five workloads are synthetic stand-ins for the image
classification runs of the paper's evaluation (CIFAR-shaped and ImageNet-shaped
tensors); no dataset item is used.
"""
import numpy as np
from . import rng

BASE_SEED = 20220711


def _layer(kind, cin, cout, k, stride, pad, h, w, relu=False, bias=False, scale=False,
           src=None, add_src=None, d=1, kd=1, pad_d=0):
    return dict(kind=kind, cin=cin, cout=cout, kh=k[0], kw=k[1], stride=stride, pad=pad, h_in=h, w_in=w,
                relu=relu, bias=bias, scale=scale, src=src, add_src=add_src, cut_after=False, d_in=d, kd=kd, pad_d=pad_d)


def out_dhw(l):
    """(D, H, W) of a layer's output for one sample (D = 1 for everything that is not a volumetric convolution)."""
    k = l["kind"]
    if k == "conv":
        s = l["stride"]
        return ((l.get("d_in", 1) + 2 * l.get("pad_d", 0) - l.get("kd", 1)) // s + 1,
                (l["h_in"] + 2 * l["pad"] - l["kh"]) // s + 1, (l["w_in"] + 2 * l["pad"] - l["kw"]) // s + 1)
    if k == "maxpool2":
        return (1, l["h_in"] // 2, l["w_in"] // 2)
    if k == "attn":
        return (1, l["h_in"], l["w_in"])
    return (1, 1, 1)


def out_shape(l):
    """(C, H, W) of a layer's output for one image; the depth of a volume is folded into H (tensor [C][D*H][W])."""
    k = l["kind"]
    if k == "conv":
        do, ho, wo = out_dhw(l)
        return (l["cout"], do * ho, wo)
    if k == "attn":
        return (l["cout"], l["h_in"], l["w_in"])
    if k == "fc":
        return (l["cout"], 1, 1)
    if k == "maxpool2":
        return (l["cin"], l["h_in"] // 2, l["w_in"] // 2)
    if k == "gap":
        return (l["cin"], 1, 1)
    if k == "softmax_ce":
        return (l["cin"], 1, 1)
    raise ValueError(k)


def in_shape(l):
    return (l["cin"], (l.get("d_in", 1) if l["kind"] in ("conv", "fc") else 1) * l["h_in"], l["w_in"])


class _Builder:
    def __init__(self, c, h, w, d=1):
        self.layers = []
        self.c, self.h, self.w, self.d = c, h, w, d          # h, w, d: true extents (a tensor is stored [C][D*H][W])

    @property
    def last(self):
        return len(self.layers) - 1

    def _push(self, l, src):
        l["src"] = self.last if src is None else src
        self.layers.append(l)
        self.c = out_shape(l)[0]
        self.d, self.h, self.w = out_dhw(l)
        return self.last

    def conv(self, cout, k, stride=1, pad=0, relu=True, bias=True, scale=False, src=None, add_src=None,
             in_chw=None):
        c, h, w = in_chw if in_chw else (self.c, self.h, self.w)
        return self._push(_layer("conv", c, cout, (k, k), stride, pad, h, w, relu, bias, scale, None, add_src), src)

    def conv3d(self, cout, k, stride=1, pad=0, relu=True, bias=True, scale=False, src=None, add_src=None, in_cdhw=None,
               w_gain=1.0):
        """k x k x k filter over the volume [C][D][H][W].  w_gain: factor on the He-normal standard deviation of its weights."""
        c, d, h, w = in_cdhw if in_cdhw else (self.c, self.d, self.h, self.w)
        l = _layer("conv", c, cout, (k, k), stride, pad, h, w, relu, bias, scale, None, add_src, d=d, kd=k, pad_d=pad)
        if w_gain != 1.0:
            l["w_gain"] = w_gain
        return self._push(l, src)

    def fc(self, cout, relu=True, bias=True):
        l = _layer("fc", self.c, cout, (self.h, self.w), 1, 0, self.h, self.w, relu, bias, d=self.d, kd=self.d)
        return self._push(l, None)

    def pool(self):
        assert self.d == 1
        return self._push(_layer("maxpool2", self.c, self.c, (2, 2), 2, 0, self.h, self.w), None)

    def gap(self):
        h = self.d * self.h
        return self._push(_layer("gap", self.c, self.c, (h, self.w), 1, 0, h, self.w), None)

    def attn(self, src=None):
        """Self-attention over all positions of the current tensor, whose 3*C channels are queries | keys | values."""
        assert self.c % 3 == 0
        d, h, w = self.d, self.h, self.w
        i = self._push(_layer("attn", self.c, self.c // 3, (1, 1), 1, 0, d * h, w), src)
        self.d, self.h, self.w = d, h, w          # the layer keeps the volume's extents (it sees them folded)
        return i

    def loss(self):
        return self._push(_layer("softmax_ce", self.c, self.c, (1, 1), 1, 0, 1, 1), None)

    def finish(self):
        """A cut may follow layer l when the only tensor crossing it is l's own output, the next
        layer is not a pooling layer (a pool stays with its conv) and not the loss."""
        L = self.layers
        for i, l in enumerate(L[:-1]):
            ok = L[i + 1]["kind"] not in ("maxpool2", "softmax_ce", "gap", "attn")
            for j in range(i + 1, len(L)):
                for ref in (L[j]["src"], L[j]["add_src"]):
                    if ref is not None and ref < i:
                        ok = False
            l["cut_after"] = ok
        return L


def lenet():
    b = _Builder(1, 28, 28)
    b.conv(6, 5); b.pool(); b.conv(16, 5); b.pool()
    b.fc(120); b.fc(84); b.fc(10, relu=False); b.loss()
    return b.finish()


def _vgg(c, hw, widths, fcs, n_classes):
    b = _Builder(c, hw, hw)
    for wd in widths:
        if wd == "M":
            b.pool()
        else:
            b.conv(wd, 3, pad=1)
    for f in fcs:
        b.fc(f)
    b.fc(n_classes, relu=False)
    b.loss()
    return b.finish()


_VGG16 = [64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M", 512, 512, 512, "M"]


def vgg16_cifar():
    return _vgg(3, 32, _VGG16, [512], 10)


def vgg16_224():
    return _vgg(3, 224, _VGG16, [4096, 4096], 1000)


def _basic_block(b, cout, stride):
    """conv3x3-ReLU-conv3x3, + shortcut, ReLU; a strided block has a 1x1 projection shortcut."""
    x = b.last                       # -1 when the block input is the network input
    chw = (b.c, b.h, b.w)
    a = b.conv(cout, 3, stride=stride, pad=1, relu=True, scale=True, src=x)
    if stride != 1 or chw[0] != cout:
        sc = b.conv(cout, 1, stride=stride, pad=0, relu=False, scale=True, src=x, in_chw=chw)
        b.c, b.h, b.w = out_shape(b.layers[a])
    else:
        sc = x
    b.conv(cout, 3, pad=1, relu=True, scale=True, src=a, add_src=sc,
           in_chw=out_shape(b.layers[a]))


def resnet18_cifar(widths=(64, 128, 256, 512), blocks=2, hw=32, n_classes=10):
    """blocks: basic blocks per stage, one number for all stages or one per stage."""
    b = _Builder(3, hw, hw)
    b.conv(widths[0], 3, pad=1, scale=True)
    per_stage = [blocks] * len(widths) if isinstance(blocks, int) else list(blocks)
    for i, wd in enumerate(widths):
        for j in range(per_stage[i]):
            _basic_block(b, wd, 2 if (i > 0 and j == 0) else 1)
    b.gap()
    b.fc(n_classes, relu=False)
    b.loss()
    return b.finish()


def resnet34_cifar():
    """The deeper basic-block network of the paper's second use case: 3, 4, 6, 3 blocks per stage."""
    return resnet18_cifar(blocks=(3, 4, 6, 3))


def _bottleneck(b, mid, cout, stride, project):
    x = b.last
    chw = (b.c, b.h, b.w)
    a = b.conv(mid, 1, relu=True, scale=True, src=x)
    c = b.conv(mid, 3, stride=stride, pad=1, relu=True, scale=True, src=a)
    if project:
        sc = b.conv(cout, 1, stride=stride, pad=0, relu=False, scale=True, src=x, in_chw=chw)
        b.c, b.h, b.w = out_shape(b.layers[c])
    else:
        sc = x
    b.conv(cout, 1, relu=True, scale=True, src=c, add_src=sc, in_chw=out_shape(b.layers[c]))


def r50_conv4x(cin=512, hw=28, mid=256, cout=1024, blocks=6):
    """One partition: the conv4_x stage of a ResNet-50 (stride 2 on the 3x3 of the first block)."""
    b = _Builder(cin, hw, hw)
    for j in range(blocks):
        _bottleneck(b, mid, cout, 2 if j == 0 else 1, j == 0)
    return b.finish()


def _basic_block3d(b, cout, stride):
    """The residual network layer of the volumetric use case: two 3x3x3 convolutions with folded normalisation and ReLU,
    plus the shortcut (a 1x1x1 projection when the block down-samples)."""
    x = b.last
    cdhw = (b.c, b.d, b.h, b.w)
    a = b.conv3d(cout, 3, stride=stride, pad=1, relu=True, scale=True, src=x)
    after = (b.c, b.d, b.h, b.w)
    if stride != 1 or cdhw[0] != cout:
        sc = b.conv3d(cout, 1, stride=stride, pad=0, relu=False, scale=True, src=x, in_cdhw=cdhw)
    else:
        sc = x
    # (the branch's last layer starts small, as a normalisation layer's zero-initialised gain would make it: without batch
    #  statistics the activations of a He-initialised residual stack otherwise double in variance per block)
    b.conv3d(cout, 3, pad=1, relu=True, scale=True, src=a, add_src=sc, in_cdhw=after, w_gain=0.25)


def _attention_block(b):
    """Residual self-attention: a 1x1x1 convolution makes queries | keys | values, the attention layer mixes the positions,
    a 1x1x1 convolution projects back and the block input is added before the ReLU."""
    x, c = b.last, b.c
    b.conv3d(3 * c, 1, relu=False, src=x, w_gain=0.5)          # scores of order one on unit-variance activations
    b.attn()
    b.conv3d(c, 1, relu=True, src=b.last, add_src=x, w_gain=0.25)


def resattnet18_3d(widths=(32, 64, 128, 256), blocks=2, vol=32, n_classes=2, attention_from=2):
    """A 3D-ResAttNet18-shaped network on synthetic one-channel volumes (stand-in for the structural-MRI scans of the
    paper's first use case; two classes as in its AD-vs-NC task): 3x3x3 stem, four stages of `blocks` residual blocks
    (stride 2 from the second stage on), a residual self-attention block after every stage from `attention_from` on
    (where the volume is small enough for all-pairs attention), global average pooling, classifier."""
    b = _Builder(1, vol, vol, vol)
    b.conv3d(widths[0], 3, pad=1, scale=True)
    for i, wd in enumerate(widths):
        for j in range(blocks):
            _basic_block3d(b, wd, 2 if (i > 0 and j == 0) else 1)
        if i >= attention_from:
            _attention_block(b)
    b.gap()
    b.fc(n_classes, relu=False)
    b.loss()
    return b.finish()


def tiny_conv3d():
    """Small volumetric network: 3x3x3 stem on 2 channels, one residual block, one strided block, attention, head."""
    b = _Builder(2, 8, 8, 4)          # 2 channels, 4 slices of 8 x 8 (a sample is a whole number of 256-byte lines)
    b.conv3d(8, 3, pad=1, scale=True)
    _basic_block3d(b, 8, 1)
    _basic_block3d(b, 16, 2)
    _attention_block(b)
    b.gap(); b.fc(5, relu=False); b.loss()
    return b.finish()


def tiny_conv3d_mfma():
    """The same shape with 32 / 64 channels, so that the matrix-core kernels take the volumetric layers."""
    b = _Builder(2, 8, 8, 4)          # 2 channels, 4 slices of 8 x 8 (a sample is a whole number of 256-byte lines)
    b.conv3d(32, 3, pad=1, scale=True)
    _basic_block3d(b, 32, 1)
    _basic_block3d(b, 64, 2)
    _attention_block(b)
    b.gap(); b.fc(5, relu=False); b.loss()
    return b.finish()


def tiny_lenet():
    """2-conv, 2-FC net on 1x8x8 inputs for finite-difference checks."""
    b = _Builder(1, 8, 8)
    b.conv(3, 3); b.pool(); b.conv(4, 2, pad=1); b.pool()
    b.fc(7); b.fc(5, relu=False); b.loss()
    return b.finish()


def tiny_linear():
    """Two convolutions without ReLU, global average pooling and an FC head: the only non-linearity is the loss,
    so no result hinges on a sign or a maximum taken on rounded values (bf16 runs of several dependent steps)."""
    b = _Builder(3, 8, 8)
    b.conv(32, 3, pad=1, relu=False); b.conv(32, 3, pad=1, relu=False); b.gap(); b.fc(5, relu=False); b.loss()
    return b.finish()


def tiny_fc():
    """One convolution, then a fully connected layer of 512 x 64 weights and a 10-class head: large enough for the
    kernels that stream a weight matrix at a few samples per micro-batch."""
    b = _Builder(3, 8, 8)
    b.conv(8, 3, pad=1); b.fc(64); b.fc(10, relu=False); b.loss()
    return b.finish()


def tiny_wide():
    """64-channel 3x3 convolutions over 4x4 and 2x2 images: gradient matrices far larger than the activations."""
    b = _Builder(3, 8, 8)
    b.conv(64, 3, pad=1); b.pool(); b.conv(64, 3, pad=1); b.pool(); b.conv(64, 3, pad=1); b.gap()
    b.fc(5, relu=False); b.loss()
    return b.finish()


def tiny_deep_pool():
    """A 512 -> 72 channel 3x3 convolution over 4x4 images followed by a pooling: a long reduction (split over blocks)
    into a channel count that is not a multiple of the 64-channel tile, then the pooling its second kernel performs."""
    b = _Builder(3, 4, 4)
    b.conv(512, 3, pad=1); b.conv(72, 3, pad=1); b.pool(); b.conv(40, 3, pad=1); b.gap()
    b.fc(5, relu=False); b.loss()
    return b.finish()


def tiny_resnet(hw=8, widths=(4, 6), n_classes=5):
    """Stem + one identity block + one strided projection block + GAP + FC."""
    return resnet18_cifar(widths=widths, blocks=1, hw=hw, n_classes=n_classes)


def tiny_vgg(hw=8, n_classes=10):
    return _vgg(3, hw, [8, 8, "M", 16, "M", 16, 16, "M"], [24], n_classes)


# name -> (builder, batch, n_microbatch, Z, dtype, fixed plan (list of stage starts) or None)
CONFIGS = {
    "lenet":          (lenet, 32, 4, 2, "f32", None),
    "vgg16_cifar":    (vgg16_cifar, 128, 8, 4, "bf16", None),
    "resnet18_cifar": (resnet18_cifar, 256, 8, 4, "bf16", [0, 5, 10, 15, 23]),      # cuts at the stage boundaries
    "resnet34_cifar": (resnet34_cifar, 256, 8, 4, "bf16", [0, 7, 16, 29, 39]),      # (not one of the five benchmark configurations: the same shapes, more depth)
    "r50_conv4x":     (r50_conv4x, 64, 4, 1, "bf16", None),
    "vgg16_224":      (vgg16_224, 32, 8, 4, "bf16", None),
}
# the volumetric use case (not one of the five benchmark configurations): batch of six volumes as in the paper's runs,
# three micro-batches of two, four partitions by the cost model
EXTRA_CONFIGS = {
    "resattnet18_3d": (resattnet18_3d, 6, 3, 4, "bf16", None),
}


def tensor_shapes(layers):
    """[(C,H,W)] for tensor -1 (network input) followed by every layer's output."""
    return [in_shape(layers[0])] + [out_shape(l) for l in layers]


def param_shapes(l):
    """{'W': shape, 'b': shape, 's': shape} of a layer's parameters (only the ones it has)."""
    if l["kind"] not in ("conv", "fc"):
        return {}
    p = {"W": (l["cout"], l["cin"], l.get("kd", 1) * l["kh"], l["kw"])}          # [Cout][Cin][Kd*Kh][Kw]
    if l["bias"]:
        p["b"] = (l["cout"],)
    if l["scale"]:
        p["s"] = (l["cout"],)
    return p


_WHICH = {"W": 0, "b": 1, "s": 2, "vW": 3, "vb": 4}


def make_params(layers, seed=BASE_SEED, bf16=False, bias_std=0.0, momentum_std=0.0):
    """He-normal weights N(0, 2/fan_in) (standard deviation times the layer's w_gain where it has one), bias N(0, bias_std) (zeros when 0), frozen scale U[0.5,1.5),
    initial momentum N(0, momentum_std) (zeros when 0).  float64, logical layouts.
    With bf16=True weights are rounded to bf16 so that both sides start from representable values."""
    params, momentum = {}, {}
    for i, l in enumerate(layers):
        sh = param_shapes(l)
        if not sh:
            continue
        fan_in = l["cin"] * l.get("kd", 1) * l["kh"] * l["kw"]
        p = {"W": rng.normal(seed, i * 8 + 0, sh["W"], 0.0, l.get("w_gain", 1.0) * np.sqrt(2.0 / fan_in))}
        if bf16:
            p["W"] = rng.round_to_bf16(p["W"])
        if "b" in sh:
            p["b"] = rng.normal(seed, i * 8 + 1, sh["b"], 0.0, bias_std) if bias_std else np.zeros(sh["b"])
        if "s" in sh:
            p["s"] = rng.uniform(seed, i * 8 + 2, sh["s"], 0.5, 1.5)
        params[i] = p
        v = {}
        for k in ("W", "b"):
            if k in sh:
                v[k] = (rng.normal(seed, i * 8 + _WHICH["v" + k], sh[k], 0.0, momentum_std)
                        if momentum_std else np.zeros(sh[k]))
        momentum[i] = v
    return params, momentum


def make_batch(layers, batch, seed=BASE_SEED, bf16=False, grad_std=1e-3):
    """Network input ~N(0,1) [batch,C,H,W]; labels uniform over the classes when the list ends in a
    loss layer, otherwise an upstream gradient ~N(0, grad_std) of the output shape."""
    x = rng.normal(seed, 1 << 20, (batch,) + in_shape(layers[0]))
    if bf16:
        x = rng.round_to_bf16(x)
    if layers[-1]["kind"] == "softmax_ce":
        return x, rng.integers(seed, (1 << 20) + 1, (batch,), layers[-1]["cin"]), None
    g = rng.normal(seed, (1 << 20) + 2, (batch,) + out_shape(layers[-1]), 0.0, grad_std)
    if bf16:
        g = rng.round_to_bf16(g)
    return x, None, g
