"""Seeded synthetic tensor sets with the shapes of the paper's evaluation models.

The paper measures on ImageNet-pretrained ResNet18v1 / ResNet50v1 / MobileNetv2 /
VGG (Sec. 7, experimental setup) with activations from calibration images
(Sec. 5, calibration stage).  Neither the weights nor the images are available
here, so these generators stand in for them: real layer shapes, random values
with the stated distributions.

This module only produces inputs.  It holds none of the method's arithmetic (no
quantizer, no metric) so that the CPU oracle and the HIP path can both be fed
from it without sharing anything else.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

WEIGHT = 0
ACTIVATION = 1

# scheme ids (same numbering as the C ABI's qv2_scheme)
ASYM_TENSOR = 0
SYM_TENSOR = 1
SYM_CHANNEL = 2


@dataclass
class TensorSpec:
    name: str
    shape: Tuple[int, ...]
    kind: int                  # WEIGHT or ACTIVATION
    layer: int                 # index of the layer this tensor belongs to
    scheme: int
    seed: int
    dist: str                  # "normal" | "relu_normal" | "relu6_normal" | "laplace_outlier"
    sigma: float = 1.0
    fold_seed: Optional[int] = None   # per-output-channel BN-fold factor ~ U(0.5, 1.5)
    has_pair: bool = False     # activation tensors carry a quantized-run partner

    @property
    def numel(self) -> int:
        return math.prod(self.shape)

    @property
    def channels(self) -> int:
        return self.shape[0] if self.scheme == SYM_CHANNEL else 1


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def materialize(spec: TensorSpec, device="cpu") -> torch.Tensor:
    """Draw the tensor a spec describes (fp32, contiguous, on `device`)."""
    g = _gen(spec.seed, device)
    n = spec.numel
    if spec.dist == "normal":
        x = torch.randn(n, generator=g, device=device, dtype=torch.float32).mul_(spec.sigma)
    elif spec.dist in ("relu_normal", "relu6_normal"):
        x = torch.randn(n, generator=g, device=device, dtype=torch.float32).mul_(spec.sigma)
        x.clamp_(min=0.0)
        if spec.dist == "relu6_normal":
            x.clamp_(max=6.0)
    elif spec.dist == "laplace_outlier":
        u = torch.rand(n, generator=g, device=device, dtype=torch.float32).sub_(0.5)
        # Laplace(0, b) by inverse CDF; |u| is kept below 1/2 so the draw stays finite
        mag = torch.log1p(-2.0 * u.abs().clamp_(max=0.49999997)).mul_(-spec.sigma)
        x = torch.sign(u).mul_(mag)
        hit = torch.rand(n, generator=g, device=device, dtype=torch.float32) < 0.01
        x = torch.where(hit, x * 20.0, x)
    else:
        raise ValueError(spec.dist)
    x = x.view(spec.shape)
    if spec.fold_seed is not None:
        gf = _gen(spec.fold_seed, device)
        f = torch.rand(spec.shape[0], generator=gf, device=device, dtype=torch.float32).add_(0.5)
        x = x * f.view(-1, *([1] * (len(spec.shape) - 1)))
    return x.contiguous()


def unit_noise(spec: TensorSpec, device="cpu") -> torch.Tensor:
    """N(0,1) tensor of the spec's shape; the harness scales it into the
    perturbation added to the quantized-run copy of an activation."""
    g = _gen(spec.seed + 500_000, device)
    return torch.randn(spec.numel, generator=g, device=device, dtype=torch.float32).view(spec.shape)


# ----------------------------------------------------------------------------
# architecture shape tables: (name, weight shape, output shape without batch)
# ----------------------------------------------------------------------------
def _conv_out(h: int, k: int, s: int, p: int) -> int:
    return (h + 2 * p - k) // s + 1


def resnet18_layers():
    L = []
    h = _conv_out(224, 7, 2, 3)                       # 112
    L.append(("conv1", (64, 3, 7, 7), (64, h, h)))
    h = _conv_out(h, 3, 2, 1)                         # maxpool -> 56
    cin = 64
    for si, c in enumerate((64, 128, 256, 512)):
        for b in range(2):
            s = 2 if (si > 0 and b == 0) else 1
            ho = _conv_out(h, 3, s, 1)
            L.append((f"s{si + 1}b{b}.conv1", (c, cin, 3, 3), (c, ho, ho)))
            L.append((f"s{si + 1}b{b}.conv2", (c, c, 3, 3), (c, ho, ho)))
            if s == 2:
                L.append((f"s{si + 1}b{b}.down", (c, cin, 1, 1), (c, ho, ho)))
            h, cin = ho, c
    L.append(("fc", (1000, 512), (1000,)))
    return L


def resnet50_layers():
    """ResNet-50 v1: the stride of a down-sampling bottleneck sits on its first 1x1."""
    L = []
    h = _conv_out(224, 7, 2, 3)
    L.append(("conv1", (64, 3, 7, 7), (64, h, h)))
    h = _conv_out(h, 3, 2, 1)
    cin = 64
    for si, (c, nb) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for b in range(nb):
            s = 2 if (si > 0 and b == 0) else 1
            ho = _conv_out(h, 1, s, 0)
            L.append((f"s{si + 1}b{b}.conv1", (c, cin, 1, 1), (c, ho, ho)))
            L.append((f"s{si + 1}b{b}.conv2", (c, c, 3, 3), (c, ho, ho)))
            L.append((f"s{si + 1}b{b}.conv3", (4 * c, c, 1, 1), (4 * c, ho, ho)))
            if b == 0:
                L.append((f"s{si + 1}b{b}.down", (4 * c, cin, 1, 1), (4 * c, ho, ho)))
            h, cin = ho, 4 * c
    L.append(("fc", (1000, 2048), (1000,)))
    return L


def mobilenetv2_layers():
    """Returns (name, weight shape, out shape, relu6?) rows."""
    L = []
    h = _conv_out(224, 3, 2, 1)
    L.append(("stem", (32, 3, 3, 3), (32, h, h), True))
    cin = 32
    cfg = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
           (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1))
    bi = 0
    for t, c, n, s in cfg:
        for i in range(n):
            stride = s if i == 0 else 1
            hid = cin * t
            if t != 1:
                L.append((f"b{bi}.expand", (hid, cin, 1, 1), (hid, h, h), True))
            ho = _conv_out(h, 3, stride, 1)
            L.append((f"b{bi}.dw", (hid, 1, 3, 3), (hid, ho, ho), True))
            L.append((f"b{bi}.project", (c, hid, 1, 1), (c, ho, ho), False))
            h, cin = ho, c
            bi += 1
    L.append(("head", (1280, cin, 1, 1), (1280, h, h), True))
    L.append(("fc", (1000, 1280), (1000,), False))
    return L


def vgg16_layers():
    L = []
    h, cin, i = 224, 3, 0
    for block in ((64, 64), (128, 128), (256, 256, 256), (512, 512, 512), (512, 512, 512)):
        for c in block:
            L.append((f"conv{i}", (c, cin, 3, 3), (c, h, h)))
            cin = c
            i += 1
        h //= 2
    L.append(("fc6", (4096, 512 * 7 * 7), (4096,)))
    L.append(("fc7", (4096, 4096), (4096,)))
    L.append(("fc8", (1000, 4096), (1000,)))
    return L


def layer_macs(layers) -> List[int]:
    """Multiply-accumulates per image of each row of a shape table:
    output elements x (input channels per group x kernel area)."""
    return [math.prod(row[2]) * math.prod(row[1][1:]) for row in layers]


def _fan_in(wshape) -> int:
    return math.prod(wshape[1:])


def _sigmas(n: int, seed: int) -> List[float]:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return (torch.rand(n, generator=g, dtype=torch.float64) * 1.5 + 0.5).tolist()


# ----------------------------------------------------------------------------
# the five tensor sets
# ----------------------------------------------------------------------------
def config_tiny() -> List[TensorSpec]:
    """Three tensors, per-tensor asymmetric; the activation carries a pair."""
    return [
        TensorSpec("conv.w", (64, 3, 7, 7), WEIGHT, 0, ASYM_TENSOR, 1000, "normal", 0.05),
        TensorSpec("conv.out", (1, 64, 56, 56), ACTIVATION, 0, ASYM_TENSOR, 1001, "relu_normal", 1.0,
                   has_pair=True),
        TensorSpec("fc.w", (10, 64), WEIGHT, 1, ASYM_TENSOR, 1002, "normal", 0.1),
    ]


def _he_set(layers, batch, seed0, w_scheme, a_scheme, fold=False) -> List[TensorSpec]:
    sig = _sigmas(len(layers), seed0 + 999)
    out = []
    for i, row in enumerate(layers):
        name, w, o = row[0], row[1], row[2]
        out.append(TensorSpec(name + ".w", tuple(w), WEIGHT, i, w_scheme, seed0 + i, "normal",
                              math.sqrt(2.0 / _fan_in(w)),
                              fold_seed=(seed0 + 999 + 7 * (i + 1)) if fold else None))
    for i, row in enumerate(layers):
        name, w, o = row[0], row[1], row[2]
        out.append(TensorSpec(name + ".out", (batch,) + tuple(o), ACTIVATION, i, a_scheme,
                              seed0 + 100 + i, "relu_normal", sig[i], has_pair=True))
    return out


def config_resnet18(batch: int = 32) -> List[TensorSpec]:
    return _he_set(resnet18_layers(), batch, 2000, ASYM_TENSOR, ASYM_TENSOR)


def config_mobilenetv2(batch: int = 64) -> List[TensorSpec]:
    layers = mobilenetv2_layers()
    sig = _sigmas(len(layers), 3999)
    out = []
    for i, (name, w, o, r6) in enumerate(layers):
        out.append(TensorSpec(name + ".w", tuple(w), WEIGHT, i, SYM_CHANNEL, 3000 + i,
                              "laplace_outlier", 0.05))
    for i, (name, w, o, r6) in enumerate(layers):
        out.append(TensorSpec(name + ".out", (batch,) + tuple(o), ACTIVATION, i, ASYM_TENSOR,
                              3100 + i, "relu6_normal" if r6 else "relu_normal", 2.0 * sig[i],
                              has_pair=True))
    return out


def config_vgg16(batch: int = 16, per_channel: bool = False) -> List[TensorSpec]:
    return _he_set(vgg16_layers(), batch, 4000,
                   SYM_CHANNEL if per_channel else ASYM_TENSOR, ASYM_TENSOR)


def config_resnet50(batch: int = 256, fused: bool = False) -> List[TensorSpec]:
    """fused=True: conv+BN folded weights (Sec. 6.3 Eq. 12), each output channel
    of a conv weight multiplied by a factor ~ U(0.5, 1.5)."""
    specs = _he_set(resnet50_layers(), batch, 5000, SYM_CHANNEL, ASYM_TENSOR, fold=fused)
    if fused:
        for s in specs:
            if s.kind == WEIGHT and len(s.shape) == 2:   # the fc layer has no BN to fold
                s.fold_seed = None
    return specs


CONFIGS = {
    "tiny": config_tiny,
    "resnet18": config_resnet18,
    "mobilenetv2": config_mobilenetv2,
    "vgg16": config_vgg16,
    "resnet50": config_resnet50,
}
