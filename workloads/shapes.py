"""Parameter-tensor shapes of the five synthetic parameter sets.

Each function returns a list of ``(name, shape)`` in the order a framework
would enumerate the model's parameters.  Only shapes are produced here.
"""

from __future__ import annotations

from typing import List, Tuple

Shape = Tuple[int, ...]
Named = List[Tuple[str, Shape]]


def tiny_mlp_shapes() -> Named:
    """784-128-10 multilayer perceptron: 101,770 parameters in 4 tensors."""
    return [
        ("fc1.weight", (784, 128)),
        ("fc1.bias", (128,)),
        ("fc2.weight", (128, 10)),
        ("fc2.bias", (10,)),
    ]


def resnet18_cifar_shapes(num_classes: int = 10) -> Named:
    """ResNet-18 with the CIFAR stem (3x3 first convolution, no max-pool).

    Architecture named in the paper's Sec. 4 ("Setup").  62 tensors,
    11,173,962 parameters for a 10-class head.
    """
    out: Named = [("conv1.weight", (64, 3, 3, 3)), ("bn1.weight", (64,)), ("bn1.bias", (64,))]
    in_ch = 64
    for stage, ch in enumerate((64, 128, 256, 512), start=1):
        for block in range(2):
            pre = f"layer{stage}.{block}"
            downsample = block == 0 and ch != in_ch
            out.append((f"{pre}.conv1.weight", (ch, in_ch, 3, 3)))
            out.append((f"{pre}.bn1.weight", (ch,)))
            out.append((f"{pre}.bn1.bias", (ch,)))
            out.append((f"{pre}.conv2.weight", (ch, ch, 3, 3)))
            out.append((f"{pre}.bn2.weight", (ch,)))
            out.append((f"{pre}.bn2.bias", (ch,)))
            if downsample:
                out.append((f"{pre}.downsample.0.weight", (ch, in_ch, 1, 1)))
                out.append((f"{pre}.downsample.1.weight", (ch,)))
                out.append((f"{pre}.downsample.1.bias", (ch,)))
            in_ch = ch
    out.append(("fc.weight", (num_classes, 512)))
    out.append(("fc.bias", (num_classes,)))
    return out


def efficientnet_b0_shapes(num_classes: int = 10) -> Named:
    """EfficientNet-B0 (width 1.0, depth 1.0), squeeze-excite convolutions with bias.

    Architecture named in the paper's Sec. 4 ("Setup").  213 tensors,
    4,020,358 parameters for a 10-class head.
    """
    out: Named = [
        ("features.0.0.weight", (32, 3, 3, 3)),
        ("features.0.1.weight", (32,)),
        ("features.0.1.bias", (32,)),
    ]
    # (expand ratio, kernel, input channels, output channels, repeats)
    stages = [
        (1, 3, 32, 16, 1),
        (6, 3, 16, 24, 2),
        (6, 5, 24, 40, 2),
        (6, 3, 40, 80, 3),
        (6, 5, 80, 112, 3),
        (6, 5, 112, 192, 4),
        (6, 3, 192, 320, 1),
    ]
    for si, (expand, k, cin, cout, reps) in enumerate(stages, start=1):
        for r in range(reps):
            pre = f"features.{si}.{r}.block"
            c_in = cin if r == 0 else cout
            c_exp = c_in * expand
            c_sq = max(1, c_in // 4)
            j = 0
            if expand != 1:
                out.append((f"{pre}.{j}.0.weight", (c_exp, c_in, 1, 1)))
                out.append((f"{pre}.{j}.1.weight", (c_exp,)))
                out.append((f"{pre}.{j}.1.bias", (c_exp,)))
                j += 1
            out.append((f"{pre}.{j}.0.weight", (c_exp, 1, k, k)))  # depthwise
            out.append((f"{pre}.{j}.1.weight", (c_exp,)))
            out.append((f"{pre}.{j}.1.bias", (c_exp,)))
            j += 1
            out.append((f"{pre}.{j}.fc1.weight", (c_sq, c_exp, 1, 1)))
            out.append((f"{pre}.{j}.fc1.bias", (c_sq,)))
            out.append((f"{pre}.{j}.fc2.weight", (c_exp, c_sq, 1, 1)))
            out.append((f"{pre}.{j}.fc2.bias", (c_exp,)))
            j += 1
            out.append((f"{pre}.{j}.0.weight", (cout, c_exp, 1, 1)))
            out.append((f"{pre}.{j}.1.weight", (cout,)))
            out.append((f"{pre}.{j}.1.bias", (cout,)))
    out.append(("features.8.0.weight", (1280, 320, 1, 1)))
    out.append(("features.8.1.weight", (1280,)))
    out.append(("features.8.1.bias", (1280,)))
    out.append(("classifier.1.weight", (num_classes, 1280)))
    out.append(("classifier.1.bias", (num_classes,)))
    return out


def large_streaming_shapes(n_tensors: int = 64, side: int = 4096) -> Named:
    """``n_tensors`` square matrices; 64 x 4096^2 = 1,073,741,824 parameters."""
    return [(f"w{i}", (side, side)) for i in range(n_tensors)]


def mixed_state_shapes(n_square: int = 16, n_wide: int = 80, rows: int = 1024) -> Named:
    """16 x [1024x1024] + 80 x [1024x4096] = 352,321,536 parameters in 96 tensors.

    The two kinds are interleaved (one square after every five wide) so that a
    prefix of the list has the same mix as the whole.
    """
    out: Named = []
    total = n_square + n_wide
    sq_left, wide_left = n_square, n_wide
    for i in range(total):
        take_square = sq_left > 0 and (i % (total // max(n_square, 1))) == 0
        if take_square or wide_left == 0:
            out.append((f"p{i}", (rows, rows)))
            sq_left -= 1
        else:
            out.append((f"p{i}", (rows, 4 * rows)))
            wide_left -= 1
    return out


def numel(shape: Shape) -> int:
    n = 1
    for d in shape:
        n *= int(d)
    return n
