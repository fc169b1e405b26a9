"""Layer shapes of the five benchmark configurations.

The shapes follow the network families the paper evaluates (MobileNet v1/v2, ResNet-50);
only the shapes are taken -- the ImageNet data and trained weights are replaced by seeded
synthetic tensors (see synth.py).  Each layer gets its own synthetic input, so pooling and
other glue between layers is not part of the path.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Tuple


@dataclass(frozen=True)
class Layer:
    name: str
    kind: str  # "conv", "dw", "qadd", "conv_add" (a convolution with the residual add fused behind it)
    H: int
    W: int
    Cin: int
    Cout: int
    k: int = 1
    stride: int = 1
    pad: int = 0
    act: str = "relu6"  # "relu6", "relu", "none"
    weight_bits: int = 8
    count: int = 1  # how many times this exact shape occurs in the network

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.k) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.k) // self.stride + 1

    @property
    def K(self) -> int:
        return self.k * self.k * (1 if self.kind == "dw" else self.Cin)

    def macs(self, batch: int) -> int:
        if self.kind == "qadd":
            return 0
        return batch * self.Ho * self.Wo * self.Cout * self.K

    def bytes(self, batch: int) -> int:
        """Algorithmic traffic: every input and output byte once, weights once, 12 B of
        per-channel parameters."""
        if self.kind == "qadd":
            return 3 * batch * self.H * self.W * self.Cout
        w_bytes = self.K * self.Cout * self.weight_bits // 8
        residual = batch * self.Ho * self.Wo * self.Cout if self.kind == "conv_add" else 0
        return batch * (self.H * self.W * self.Cin + self.Ho * self.Wo * self.Cout) + residual + w_bytes + 12 * self.Cout


def single_conv() -> List[Layer]:
    """Configuration 1: one 3x3 convolution, 28x28x32 -> 32 channels, ReLU6."""
    return [Layer("conv3x3_28x28x32", "conv", 28, 28, 32, 32, k=3, stride=1, pad=1, act="relu6")]


def gemm_sweep() -> Tuple[List[Tuple[int, int, int]], List[Tuple[int, int, int]]]:
    """Configuration 2: (square-ish, skinny) lists of (M, N, K)."""
    dims = [256, 1024, 4096, 8192]
    full = [(m, n, k) for m in dims for n in dims for k in dims]
    skinny = [(m, 4096, 4096) for m in (1, 2, 4, 8, 16, 32, 64)]
    return full, skinny


def mobilenet_v1() -> List[Layer]:
    """Configuration 3: 3x3 stride-2 stem, then 13 x (depthwise 3x3 + pointwise 1x1)."""
    layers = [Layer("stem", "conv", 224, 224, 3, 32, k=3, stride=2, pad=1)]
    spec = [(32, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1), (256, 512, 2), (512, 512, 1),
            (512, 512, 1), (512, 512, 1), (512, 512, 1), (512, 512, 1), (512, 1024, 2), (1024, 1024, 1)]
    h = 112
    for i, (cin, cout, s) in enumerate(spec, 1):
        layers.append(Layer(f"dw{i}", "dw", h, h, cin, cin, k=3, stride=s, pad=1))
        h = (h + 2 - 3) // s + 1
        layers.append(Layer(f"pw{i}", "conv", h, h, cin, cout, k=1))
    return layers


def resnet50() -> List[Layer]:
    """Configuration 4: 7x7 stem, bottleneck stages [3,4,6,3] (stride 2 on the 3x3 of the first
    block of stages 2-4, 1x1 projection shortcuts), and the rescaling residual adds."""
    layers = [Layer("stem7x7", "conv", 224, 224, 3, 64, k=7, stride=2, pad=3, act="relu")]
    h, cin = 56, 64
    for stage, (width, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], 1):
        cout = width * 4
        for b in range(blocks):
            s = 2 if (b == 0 and stage > 1) else 1
            tag = f"s{stage}b{b}"
            layers.append(Layer(f"{tag}_1x1a", "conv", h, h, cin, width, k=1, act="relu"))
            layers.append(Layer(f"{tag}_3x3", "conv", h, h, width, width, k=3, stride=s, pad=1, act="relu"))
            ho = (h + 2 - 3) // s + 1
            layers.append(Layer(f"{tag}_1x1b", "conv", ho, ho, width, cout, k=1, act="none"))
            if b == 0:
                layers.append(Layer(f"{tag}_proj", "conv", h, h, cin, cout, k=1, stride=s, act="none"))
            layers.append(Layer(f"{tag}_add", "qadd", ho, ho, cout, cout, act="relu"))
            h, cin = ho, cout
    return layers


def mobilenet_v2(weight_bits: int = 4) -> List[Layer]:
    """Configuration 5: inverted-residual blocks (expansion 6, widths 16-24-32-64-96-160-320),
    1x1 / stem weights stored with `weight_bits` bits, depthwise weights int8."""
    wb = weight_bits
    # the stem has Cin = 3 (odd), which nibble packing along Cin cannot hold: it stays int8
    layers = [Layer("stem", "conv", 224, 224, 3, 32, k=3, stride=2, pad=1, weight_bits=8)]
    h, cin = 112, 32
    layers.append(Layer("b0_dw", "dw", h, h, 32, 32, k=3, stride=1, pad=1))
    layers.append(Layer("b0_project", "conv", h, h, 32, 16, k=1, act="none", weight_bits=wb))
    cin = 16
    idx = 1
    for t, c, n, s in [(6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]:
        for i in range(n):
            stride = s if i == 0 else 1
            mid = cin * t
            layers.append(Layer(f"b{idx}_expand", "conv", h, h, cin, mid, k=1, weight_bits=wb))
            layers.append(Layer(f"b{idx}_dw", "dw", h, h, mid, mid, k=3, stride=stride, pad=1))
            ho = (h + 2 - 3) // stride + 1
            layers.append(Layer(f"b{idx}_project", "conv", ho, ho, mid, c, k=1, act="none", weight_bits=wb))
            if stride == 1 and cin == c:
                layers.append(Layer(f"b{idx}_add", "qadd", ho, ho, c, c, act="none"))
            h, cin = ho, c
            idx += 1
    layers.append(Layer("head", "conv", h, h, 320, 1280, k=1, weight_bits=wb))
    return layers


def fuse_adds(layers: List[Layer]) -> List[Layer]:
    """The same network with every residual add folded into the convolution that produces its
    first operand (the last 1x1 of the block): that layer becomes a "conv_add" carrying the
    add's activation, and the separate "qadd" entry disappears."""
    out: List[Layer] = []
    for l in layers:
        if l.kind == "qadd":
            for back in (1, 2):  # the producing 1x1 is the previous layer, or the one before a projection shortcut
                if back > len(out):
                    continue  # not enough layers before the add to look this far back
                p = out[-back]
                if p.kind == "conv" and p.act == "none" and (p.Ho, p.Wo, p.Cout) == (l.H, l.W, l.Cout) and \
                        not p.name.endswith("_proj"):
                    out[-back] = replace(p, kind="conv_add", act=l.act, name=p.name + "+add")
                    break
            else:
                out.append(l)
            continue
        out.append(l)
    return out


def unique_shapes(layers: List[Layer]) -> List[Layer]:
    """Collapse layers that differ only by name into one entry with a count."""
    seen = {}
    for l in layers:
        key = replace(l, name="", count=1)
        if key in seen:
            seen[key] = replace(seen[key], count=seen[key].count + 1)
        else:
            seen[key] = l
    return list(seen.values())
