"""Workload shapes and the chain order of trainable tensors.

The tensor order is the execution order of the trainable tensors in the
forward pass (Section 5: the list of trainable tensors sorted by execution
order); index 0 is the input-most tensor, index N-1 the output-most one.
"""
from dataclasses import dataclass, field
from typing import List, Tuple


@dataclass(frozen=True)
class MLPConfig:
    """ReLU multi-layer perceptron without biases: dims[0] -> ... -> dims[-1]."""
    name: str
    dims: Tuple[int, ...]
    batch: int
    dtype: str = "f32"
    kind: str = "mlp"

    @property
    def classes(self) -> int:
        return self.dims[-1]


@dataclass(frozen=True)
class ViTConfig:
    """Pre-LN vision-transformer encoder fed with flattened patches."""
    name: str
    batch: int
    tokens: int        # patches + 1 CLS token
    patch_dim: int     # flattened patch length (16*16*3 = 768)
    width: int         # D
    heads: int         # H, head size = D / H
    mlp: int           # F
    blocks: int        # L
    classes: int       # C
    dtype: str = "bf16"
    kind: str = "vit"
    ln_eps: float = 1e-6

    @property
    def head_dim(self) -> int:
        return self.width // self.heads

    @property
    def rows(self) -> int:
        return self.batch * self.tokens


@dataclass(frozen=True)
class ResNetConfig:
    """Bottleneck ResNet on NHWC images; BatchNorm folded into a per-channel affine (gain, shift).

    Stem: 7x7/2 convolution, affine, ReLU, 3x3/2 max pooling.  Stage i has blocks[i] bottleneck
    blocks of planes[i] -> 4*planes[i] channels (1x1, 3x3, 1x1 convolutions, each followed by an
    affine; ReLU after the first two and after the residual sum); the 3x3 convolution of the first
    block of stages 1.. has stride 2 and that block has a 1x1 projection shortcut (so has the
    first block of stage 0, stride 1).  Global average pooling and a linear head follow.
    Convolutions carry no bias.  Weights are stored [out, kh, kw, in]."""
    name: str
    batch: int
    image: int
    in_ch: int
    stem: int
    blocks: Tuple[int, ...]
    planes: Tuple[int, ...]
    classes: int
    dtype: str = "bf16"
    kind: str = "resnet"


@dataclass(frozen=True)
class VGGConfig:
    """Plain convolution stack on NHWC images (VGG family): stage i has convs[i] 3x3 convolutions (stride 1,
    padding 1, with bias, ReLU) to widths[i] channels followed by 2x2 / stride 2 max pooling; then the
    flattened (h, w, c) features go through linear layers of fc[j] units with bias and ReLU and a linear
    head.  Convolution weights are stored [out, kh, kw, in], linear ones [out, in]."""
    name: str
    batch: int
    image: int
    in_ch: int
    widths: Tuple[int, ...]
    convs: Tuple[int, ...]
    fc: Tuple[int, ...]
    classes: int
    dtype: str = "bf16"
    kind: str = "vgg"


@dataclass(frozen=True)
class MobileNetConfig:
    """Inverted-residual network on NHWC images (MobileNetV2 family); BatchNorm folded into a per-channel
    affine.  Stem: 3x3 / stride 2 convolution to `stem` channels, affine, ReLU6.  Each entry (t, c, n, s) of
    `settings` is n blocks to c channels with expansion factor t, the first of stride s: a 1x1 expansion to
    t * c_in channels (affine, ReLU6; absent when t = 1), a 3x3 depthwise convolution (stride s or 1, affine,
    ReLU6), a 1x1 projection to c channels (affine, no activation); a block of stride 1 whose input has c
    channels adds its input to its output.  Then a 1x1 convolution to `last` channels (affine, ReLU6), global
    average pooling and a linear head.  Convolution weights are stored [out, kh, kw, in], the depthwise ones
    [channels, 3, 3, 1]; convolutions carry no bias."""
    name: str
    batch: int
    image: int
    in_ch: int
    stem: int
    settings: Tuple[Tuple[int, int, int, int], ...]
    last: int
    classes: int
    dtype: str = "bf16"
    kind: str = "mobilenet"


def mobilenet_blocks(cfg):
    """[(c_in, hidden, c_out, stride, has_expansion, has_shortcut)] in forward order."""
    out, cin = [], cfg.stem
    for (t, c, n, s) in cfg.settings:
        for i in range(n):
            stride = s if i == 0 else 1
            out.append((cin, cin * t, c, stride, t != 1, stride == 1 and cin == c))
            cin = c
    return out


CONFIGS = {
    # BASELINE configs[0]: 4-layer ReLU MLP, fp32, batch 32
    "mlp": MLPConfig("mlp", (256, 256, 256, 256, 10), 32),
    # BASELINE configs[1]/[2]: ViT-B/16 shape, batch 64
    "vit_b": ViTConfig("vit_b", 64, 197, 768, 768, 12, 3072, 12, 200),
    # BASELINE configs[3]: ViT-L/16 shape, batch 32
    "vit_l": ViTConfig("vit_l", 32, 197, 768, 1024, 16, 4096, 24, 200),
    # BASELINE configs[4]: ResNet-50 shape, batch 32
    "resnet50": ResNetConfig("resnet50", 32, 224, 3, 64, (3, 4, 6, 3), (64, 128, 256, 512), 200),
    "resnet_tiny": ResNetConfig("resnet_tiny", 2, 16, 3, 8, (1, 1), (8, 8), 8),
    "resnet_small": ResNetConfig("resnet_small", 3, 64, 3, 16, (2, 1, 2, 1), (8, 16, 24, 32), 24),
    # bottleneck width 64: the 3x3 convolutions that run as implicit GEMMs (stride 1) next to a strided one
    "resnet_c64": ResNetConfig("resnet_c64", 2, 32, 3, 64, (2, 1), (64, 128), 16),
    # odd image sizes and output-pixel counts that are not multiples of 64: the convolutions whose weight gradient (and,
    # for the stem, forward product) falls back to an explicit column matrix
    "resnet_odd": ResNetConfig("resnet_odd", 1, 18, 3, 8, (1, 1), (8, 8), 8),
    "resnet_c64_odd": ResNetConfig("resnet_c64_odd", 1, 36, 3, 64, (1, 1), (64, 128), 16),
    # second CNN family of the paper's evaluation (Section 8): VGG16 shape, 200 classes
    "vgg16": VGGConfig("vgg16", 32, 224, 3, (64, 128, 256, 512, 512), (2, 2, 3, 3, 3), (4096, 4096), 200),
    "vgg_tiny": VGGConfig("vgg_tiny", 2, 8, 3, (8, 8), (1, 2), (16,), 8),
    "vgg_small": VGGConfig("vgg_small", 3, 32, 3, (8, 16, 24), (2, 1, 2), (40, 24), 24),
    # channel counts in multiples of 64, as in VGG16: the convolutions that run as implicit GEMMs
    "vgg_c64": VGGConfig("vgg_c64", 2, 16, 3, (64, 128), (2, 2), (64,), 16),
    # third CNN family of the paper's evaluation (Section 8): MobileNetV2 shape (width 1.0), 200 classes
    "mobilenetv2": MobileNetConfig("mobilenetv2", 32, 224, 3, 32, ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                                                                  (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)), 1280, 200),
    "mobilenet_tiny": MobileNetConfig("mobilenet_tiny", 2, 16, 3, 8, ((1, 8, 1, 1), (2, 8, 2, 2)), 16, 8),
    "mobilenet_small": MobileNetConfig("mobilenet_small", 3, 32, 3, 8, ((1, 8, 1, 1), (6, 16, 2, 2), (6, 24, 2, 2), (4, 24, 1, 1)), 64, 24),
    # small cases the oracle finishes in well under a second
    "mlp_tiny": MLPConfig("mlp_tiny", (8, 8, 8, 4), 4),
    "mlp5": MLPConfig("mlp5", (6, 6, 6, 6, 6, 3), 4),
    "vit_tiny": ViTConfig("vit_tiny", 2, 5, 12, 16, 2, 32, 2, 7),
    # spans several GEMM tiles with ragged tails in every dimension
    "vit_small": ViTConfig("vit_small", 3, 197, 200, 192, 3, 320, 2, 56),
    "vit_mid": ViTConfig("vit_mid", 5, 197, 768, 384, 6, 1536, 3, 200),
    # more tokens than the fused attention kernels take: exercises the unfused attention path
    "vit_t230": ViTConfig("vit_t230", 2, 230, 64, 128, 2, 256, 1, 16),
    # fewer tokens: one and two key tiles in the fused attention kernels
    "vit_t40": ViTConfig("vit_t40", 3, 40, 64, 128, 2, 256, 2, 16),
    # widths that are multiples of 256 (rows the LayerNorm kernels keep in registers): one block each, few tokens
    "vit_w256": ViTConfig("vit_w256", 2, 9, 64, 256, 4, 256, 1, 16),
    "vit_w512": ViTConfig("vit_w512", 2, 9, 64, 512, 8, 256, 1, 16),
    "vit_w1280": ViTConfig("vit_w1280", 1, 7, 64, 1280, 20, 256, 1, 16),
    "vit_w1536": ViTConfig("vit_w1536", 1, 7, 64, 1536, 24, 256, 1, 16),
    "vit_w2048": ViTConfig("vit_w2048", 1, 7, 64, 2048, 32, 256, 1, 16),
}


def tensor_specs(cfg) -> List[Tuple[str, Tuple[int, ...]]]:
    """(name, shape) of every trainable tensor in chain order."""
    if cfg.kind == "mlp":
        return [(f"fc{i}.W", (cfg.dims[i + 1], cfg.dims[i])) for i in range(len(cfg.dims) - 1)]
    if cfg.kind == "vit":
        D, F = cfg.width, cfg.mlp
        out = [("patch.W", (D, cfg.patch_dim)), ("patch.b", (D,)), ("cls", (D,)), ("pos", (cfg.tokens, D))]
        for l in range(cfg.blocks):
            p = f"blk{l}."
            out += [(p + "ln1.g", (D,)), (p + "ln1.b", (D,)),
                    (p + "qkv.W", (3 * D, D)), (p + "qkv.b", (3 * D,)),
                    (p + "proj.W", (D, D)), (p + "proj.b", (D,)),
                    (p + "ln2.g", (D,)), (p + "ln2.b", (D,)),
                    (p + "fc1.W", (F, D)), (p + "fc1.b", (F,)),
                    (p + "fc2.W", (D, F)), (p + "fc2.b", (D,))]
        out += [("lnf.g", (D,)), ("lnf.b", (D,)), ("head.W", (cfg.classes, D)), ("head.b", (cfg.classes,))]
        return out
    if cfg.kind == "resnet":
        out = [("stem.W", (cfg.stem, 7, 7, cfg.in_ch)), ("stem.g", (cfg.stem,)), ("stem.b", (cfg.stem,))]
        cin = cfg.stem
        for si, (nb, p) in enumerate(zip(cfg.blocks, cfg.planes)):
            for bi in range(nb):
                n = "s%db%d." % (si, bi)
                out += [(n + "c1.W", (p, 1, 1, cin)), (n + "c1.g", (p,)), (n + "c1.b", (p,)),
                        (n + "c2.W", (p, 3, 3, p)), (n + "c2.g", (p,)), (n + "c2.b", (p,)),
                        (n + "c3.W", (4 * p, 1, 1, p)), (n + "c3.g", (4 * p,)), (n + "c3.b", (4 * p,))]
                if bi == 0:      # projection shortcut; in chain order it follows the main branch
                    out += [(n + "sc.W", (4 * p, 1, 1, cin)), (n + "sc.g", (4 * p,)), (n + "sc.b", (4 * p,))]
                cin = 4 * p
        out += [("head.W", (cfg.classes, cin)), ("head.b", (cfg.classes,))]
        return out
    if cfg.kind == "mobilenet":
        out = [("stem.W", (cfg.stem, 3, 3, cfg.in_ch)), ("stem.g", (cfg.stem,)), ("stem.b", (cfg.stem,))]
        for i, (cin, hid, cout, stride, expand, shortcut) in enumerate(mobilenet_blocks(cfg)):
            n = "b%d." % i
            if expand:
                out += [(n + "exp.W", (hid, 1, 1, cin)), (n + "exp.g", (hid,)), (n + "exp.b", (hid,))]
            out += [(n + "dw.W", (hid, 3, 3, 1)), (n + "dw.g", (hid,)), (n + "dw.b", (hid,)),
                    (n + "proj.W", (cout, 1, 1, hid)), (n + "proj.g", (cout,)), (n + "proj.b", (cout,))]
        c_last = mobilenet_blocks(cfg)[-1][2]
        out += [("last.W", (cfg.last, 1, 1, c_last)), ("last.g", (cfg.last,)), ("last.b", (cfg.last,)),
                ("head.W", (cfg.classes, cfg.last)), ("head.b", (cfg.classes,))]
        return out
    if cfg.kind == "vgg":
        out, cin, i = [], cfg.in_ch, 0
        for w, n in zip(cfg.widths, cfg.convs):
            for _ in range(n):
                out += [("conv%d.W" % i, (w, 3, 3, cin)), ("conv%d.b" % i, (w,))]
                cin, i = w, i + 1
        side = cfg.image >> len(cfg.widths)
        fin = side * side * cin
        for j, f in enumerate(tuple(cfg.fc) + (cfg.classes,)):
            out += [("fc%d.W" % j, (f, fin)), ("fc%d.b" % j, (f,))]
            fin = f
        return out
    raise ValueError(cfg.kind)
