"""Tensor-shape recipes for the synthetic gradient workloads.

Each recipe returns a list of (name, numel) pairs: the per-layer tensors of a model family, packed back to
back with no padding into one flat n-element gradient.  Nothing in this module touches the method's
arithmetic; it only fixes how many elements there are and where each tensor starts.

The families stand in for the models the paper trains (Table 1: FNN-3, VGG-16, ResNet-20, LSTM-PTB); the
LSTM recipe reproduces Table 1's LSTM-PTB parameter count exactly (66,034,000).
"""
from __future__ import annotations

from typing import List, Tuple

Tensors = List[Tuple[str, int]]


def flat(n: int) -> Tensors:
    return [("flat", int(n))]


def resnet50(width: int = 64, num_classes: int = 1000) -> Tensors:
    """ResNet-50: 7x7 stem, bottleneck stages [3, 4, 6, 3], a BN weight and bias after every conv, FC + bias.

    width=64, num_classes=1000 gives 25,557,032 elements in 161 tensors.
    """
    t: Tensors = []

    def conv_bn(name: str, cin: int, cout: int, k: int) -> None:
        t.append((f"{name}.weight", cout * cin * k * k))
        t.append((f"{name}.bn.weight", cout))
        t.append((f"{name}.bn.bias", cout))

    conv_bn("stem", 3, width, 7)
    cin = width
    for s, blocks in enumerate([3, 4, 6, 3]):
        mid = width * (2 ** s)
        out = 4 * mid
        for b in range(blocks):
            pre = f"stage{s + 1}.block{b}"
            conv_bn(f"{pre}.conv1", cin, mid, 1)
            conv_bn(f"{pre}.conv2", mid, mid, 3)
            conv_bn(f"{pre}.conv3", mid, out, 1)
            if b == 0:
                conv_bn(f"{pre}.downsample", cin, out, 1)
            cin = out
    t.append(("fc.weight", cin * num_classes))
    t.append(("fc.bias", num_classes))
    return t


def lstm_lm(vocab: int = 10000, hidden: int = 1500, layers: int = 2) -> Tensors:
    """2-layer LSTM language model: encoder, per layer one (4*hidden) x (2*hidden) gate matrix and two
    (4*hidden) biases, decoder of the encoder's shape plus a bias.

    vocab=10000, hidden=1500 gives 66,034,000 elements in 9 tensors (Table 1's LSTM-PTB count).
    """
    t: Tensors = [("encoder.weight", vocab * hidden)]
    for l in range(layers):
        t.append((f"lstm{l}.gates", 4 * hidden * 2 * hidden))
        t.append((f"lstm{l}.bias_ih", 4 * hidden))
        t.append((f"lstm{l}.bias_hh", 4 * hidden))
    t.append(("decoder.weight", vocab * hidden))
    t.append(("decoder.bias", vocab))
    return t


def vgg16(width: int = 64, fc: int = 4096, spatial: int = 7, num_classes: int = 1000) -> Tensors:
    """VGG-16 (ImageNet shape): 13 conv 3x3 with biases, then three FC layers with biases.

    Defaults give 138,357,544 elements in 32 tensors.
    """
    mult = [1, 1, 2, 2, 4, 4, 4, 8, 8, 8, 8, 8, 8]
    t: Tensors = []
    cin = 3
    for i, m in enumerate(mult):
        cout = width * m
        t.append((f"conv{i}.weight", cout * cin * 9))
        t.append((f"conv{i}.bias", cout))
        cin = cout
    t.append(("fc0.weight", cin * spatial * spatial * fc))
    t.append(("fc0.bias", fc))
    t.append(("fc1.weight", fc * fc))
    t.append(("fc1.bias", fc))
    t.append(("fc2.weight", fc * num_classes))
    t.append(("fc2.bias", num_classes))
    return t


def transformer(layers: int = 48, d_model: int = 1600, d_ff: int = 6400, vocab: int = 50257,
                positions: int = 1024, truncate_to: int | None = 1_500_000_000) -> Tensors:
    """Decoder-only transformer: token + position embeddings, per layer two LayerNorms, QKV, projection
    and a two-matrix MLP (all with biases), final LayerNorm.

    Defaults give 1,557,611,200 elements; the tensor list is cut at exactly `truncate_to` elements (the
    last kept tensor is shortened) so the flat gradient has n = 1.5e9.
    """
    t: Tensors = [("wte", vocab * d_model), ("wpe", positions * d_model)]
    for l in range(layers):
        pre = f"h{l}"
        t += [(f"{pre}.ln1.weight", d_model), (f"{pre}.ln1.bias", d_model),
              (f"{pre}.attn.qkv.weight", d_model * 3 * d_model), (f"{pre}.attn.qkv.bias", 3 * d_model),
              (f"{pre}.attn.proj.weight", d_model * d_model), (f"{pre}.attn.proj.bias", d_model),
              (f"{pre}.ln2.weight", d_model), (f"{pre}.ln2.bias", d_model),
              (f"{pre}.mlp.fc.weight", d_model * d_ff), (f"{pre}.mlp.fc.bias", d_ff),
              (f"{pre}.mlp.proj.weight", d_ff * d_model), (f"{pre}.mlp.proj.bias", d_model)]
    t += [("ln_f.weight", d_model), ("ln_f.bias", d_model)]
    if truncate_to is not None:
        out: Tensors = []
        left = int(truncate_to)
        for name, numel in t:
            if left <= 0:
                break
            take = min(numel, left)
            out.append((name, take))
            left -= take
        t = out
    return t


def fnn3() -> Tensors:
    """Table 1's FNN-3 on MNIST: 784-200-200-10 with biases, 199,210 elements in 6 tensors."""
    t: Tensors = []
    for i, (cin, cout) in enumerate([(784, 200), (200, 200), (200, 10)]):
        t.append((f"fc{i}.weight", cin * cout))
        t.append((f"fc{i}.bias", cout))
    return t


def resnet20(num_classes: int = 10) -> Tensors:
    """Table 1's ResNet-20 on CIFAR10: 3x3 stem, three stages of three basic blocks with 16/32/64 channels,
    parameter-free shortcuts, a BN weight and bias after every conv, FC + bias: 269,722 elements in 59 tensors."""
    t: Tensors = []

    def conv_bn(name: str, cin: int, cout: int) -> None:
        t.append((f"{name}.weight", cout * cin * 9))
        t.append((f"{name}.bn.weight", cout))
        t.append((f"{name}.bn.bias", cout))

    conv_bn("stem", 3, 16)
    cin = 16
    for s, ch in enumerate([16, 32, 64]):
        for b in range(3):
            conv_bn(f"stage{s + 1}.block{b}.conv1", cin, ch)
            conv_bn(f"stage{s + 1}.block{b}.conv2", ch, ch)
            cin = ch
    t.append(("fc.weight", cin * num_classes))
    t.append(("fc.bias", num_classes))
    return t


def vgg16_cifar(num_classes: int = 10) -> Tensors:
    """Table 1's VGG-16 on CIFAR10: 13 conv 3x3 with biases, each followed by a BN weight and bias, and one
    512 x 10 classifier: 14,728,266 elements in 54 tensors."""
    t: Tensors = []
    cin = 3
    for i, cout in enumerate([64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512]):
        t.append((f"conv{i}.weight", cout * cin * 9))
        t.append((f"conv{i}.bias", cout))
        t.append((f"bn{i}.weight", cout))
        t.append((f"bn{i}.bias", cout))
        cin = cout
    t.append(("classifier.weight", cin * num_classes))
    t.append(("classifier.bias", num_classes))
    return t


def total(tensors: Tensors) -> int:
    return sum(numel for _, numel in tensors)


def offsets(tensors: Tensors) -> List[int]:
    """Start offset of each tensor in the flat gradient."""
    off, acc = [], 0
    for _, numel in tensors:
        off.append(acc)
        acc += numel
    return off
