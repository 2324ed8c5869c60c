"""Parameter-tensor layouts (trainable parameters only, no BatchNorm running
statistics: the paper does not shuffle those, Sec. 4 "Training methods").

Each layout is the list of tensors in definition order; a population row is
their concatenation with no padding, so tensor starts are in general not
16-byte aligned.  kind is one of "conv", "linear", "norm_w", "norm_b", "bias",
"embed" and drives the init rule in generate.py.
"""
from dataclasses import dataclass
from math import prod
from typing import List, Sequence, Tuple


@dataclass(frozen=True)
class Tensor:
    name: str
    shape: Tuple[int, ...]
    kind: str

    @property
    def numel(self) -> int:
        return prod(self.shape)


def _bn(name: str, c: int) -> List[Tensor]:
    return [Tensor(name + ".weight", (c,), "norm_w"), Tensor(name + ".bias", (c,), "norm_b")]


def _conv(name: str, cout: int, cin: int, k: int) -> Tensor:
    return Tensor(name + ".weight", (cout, cin, k, k), "conv")


def resnet18_cifar(num_classes: int = 10) -> List[Tensor]:
    """ResNet-18, CIFAR variant (3x3 stem, no max-pool): 62 tensors, 11,173,962 parameters."""
    t = [_conv("conv1", 64, 3, 3)] + _bn("bn1", 64)
    cin = 64
    for stage, (c, stride) in enumerate([(64, 1), (128, 2), (256, 2), (512, 2)], start=1):
        for b in range(2):
            s = stride if b == 0 else 1
            pre = f"layer{stage}.{b}"
            t += [_conv(pre + ".conv1", c, cin, 3)] + _bn(pre + ".bn1", c)
            t += [_conv(pre + ".conv2", c, c, 3)] + _bn(pre + ".bn2", c)
            if s != 1 or cin != c:
                t += [_conv(pre + ".shortcut.0", c, cin, 1)] + _bn(pre + ".shortcut.1", c)
            cin = c
    t += [Tensor("fc.weight", (num_classes, 512), "linear"), Tensor("fc.bias", (num_classes,), "bias")]
    return t


def resnet50_imagenet(num_classes: int = 1000) -> List[Tensor]:
    """ResNet-50, ImageNet: 161 tensors, 25,557,032 parameters."""
    t = [_conv("conv1", 64, 3, 7)] + _bn("bn1", 64)
    cin = 64
    for stage, (planes, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], start=1):
        for b in range(blocks):
            pre = f"layer{stage}.{b}"
            t += [_conv(pre + ".conv1", planes, cin, 1)] + _bn(pre + ".bn1", planes)
            t += [_conv(pre + ".conv2", planes, planes, 3)] + _bn(pre + ".bn2", planes)
            t += [_conv(pre + ".conv3", 4 * planes, planes, 1)] + _bn(pre + ".bn3", 4 * planes)
            if b == 0:
                t += [_conv(pre + ".downsample.0", 4 * planes, cin, 1)] + _bn(pre + ".downsample.1", 4 * planes)
            cin = 4 * planes
    t += [Tensor("fc.weight", (num_classes, 2048), "linear"), Tensor("fc.bias", (num_classes,), "bias")]
    return t


def vit_b16(num_classes: int = 1000) -> List[Tensor]:
    """ViT-B/16 at 224x224: 152 tensors, 86,567,656 parameters."""
    d, mlp = 768, 3072
    t = [Tensor("cls_token", (1, 1, d), "embed"), Tensor("pos_embed", (1, 197, d), "embed"),
         Tensor("patch_embed.proj.weight", (d, 3, 16, 16), "linear"),
         Tensor("patch_embed.proj.bias", (d,), "bias")]
    for b in range(12):
        pre = f"blocks.{b}"
        t += [Tensor(pre + ".norm1.weight", (d,), "norm_w"), Tensor(pre + ".norm1.bias", (d,), "norm_b"),
              Tensor(pre + ".attn.qkv.weight", (3 * d, d), "linear"), Tensor(pre + ".attn.qkv.bias", (3 * d,), "bias"),
              Tensor(pre + ".attn.proj.weight", (d, d), "linear"), Tensor(pre + ".attn.proj.bias", (d,), "bias"),
              Tensor(pre + ".norm2.weight", (d,), "norm_w"), Tensor(pre + ".norm2.bias", (d,), "norm_b"),
              Tensor(pre + ".mlp.fc1.weight", (mlp, d), "linear"), Tensor(pre + ".mlp.fc1.bias", (mlp,), "bias"),
              Tensor(pre + ".mlp.fc2.weight", (d, mlp), "linear"), Tensor(pre + ".mlp.fc2.bias", (d,), "bias")]
    t += [Tensor("norm.weight", (d,), "norm_w"), Tensor("norm.bias", (d,), "norm_b"),
          Tensor("head.weight", (num_classes, d), "linear"), Tensor("head.bias", (num_classes,), "bias")]
    return t


def flat(P: int, parts: int = 1) -> List[Tensor]:
    """P coordinates cut into `parts` segments of (almost) equal length."""
    edges = [P * k // parts for k in range(parts + 1)]
    return [Tensor(f"seg{k}", (edges[k + 1] - edges[k],), "flat") for k in range(parts)]


def segments_of(tensors: Sequence[Tensor], probs: Sequence[float]) -> List[Tuple[int, int, float]]:
    """(offset, length, p) triples for a layout and one probability per tensor."""
    assert len(tensors) == len(probs)
    out, off = [], 0
    for t, p in zip(tensors, probs):
        out.append((off, t.numel, float(p)))
        off += t.numel
    return out
