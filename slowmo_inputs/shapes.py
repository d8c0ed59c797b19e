"""Tensor-shape lists of the workloads.

Only shapes and sizes are taken from the paper's experiments (Section 4 and
Appendix A: ResNet-18 on CIFAR-10, ResNet-50 on ImageNet, the "big"
Transformer with 6+6 blocks on WMT'16 En-De).  The lists are generated from
the architectures' published layer recipes; no dataset or weight is involved.

Each function returns a list of (name, shape) with shape a tuple of ints.
This module holds no optimizer arithmetic.
"""
from __future__ import annotations

from math import prod
from typing import List, Tuple

Shape = Tuple[int, ...]
NamedShape = Tuple[str, Shape]


def _bn(name: str, c: int) -> List[NamedShape]:
    return [(name + ".weight", (c,)), (name + ".bias", (c,))]


def tiny_flat(d: int = 65536) -> List[NamedShape]:
    """One flat fp32 tensor (the tiny configuration)."""
    return [("flat", (d,))]


def stress_flat(d: int = 1_000_000_000) -> List[NamedShape]:
    """One flat tensor of 1e9 elements: offsets exceed 32 bits in bytes."""
    return [("flat", (d,))]


def resnet18() -> List[NamedShape]:
    """ResNet-18 with a 1000-way head: 62 tensors, 11 689 512 elements."""
    out: List[NamedShape] = [("conv1.weight", (64, 3, 7, 7))] + _bn("bn1", 64)
    cin = 64
    for s, (w, nblk) in enumerate(zip((64, 128, 256, 512), (2, 2, 2, 2)), 1):
        for b in range(nblk):
            p = f"layer{s}.{b}"
            out.append((p + ".conv1.weight", (w, cin, 3, 3)))
            out += _bn(p + ".bn1", w)
            out.append((p + ".conv2.weight", (w, w, 3, 3)))
            out += _bn(p + ".bn2", w)
            if b == 0 and s > 1:
                out.append((p + ".downsample.0.weight", (w, cin, 1, 1)))
                out += _bn(p + ".downsample.1", w)
            cin = w
    out += [("fc.weight", (1000, 512)), ("fc.bias", (1000,))]
    return out


def resnet50() -> List[NamedShape]:
    """ResNet-50 (bottleneck, expansion 4): 161 tensors, 25 557 032 elements."""
    out: List[NamedShape] = [("conv1.weight", (64, 3, 7, 7))] + _bn("bn1", 64)
    cin = 64
    for s, (w, nblk) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3)), 1):
        for b in range(nblk):
            p = f"layer{s}.{b}"
            out.append((p + ".conv1.weight", (w, cin, 1, 1)))
            out += _bn(p + ".bn1", w)
            out.append((p + ".conv2.weight", (w, w, 3, 3)))
            out += _bn(p + ".bn2", w)
            out.append((p + ".conv3.weight", (4 * w, w, 1, 1)))
            out += _bn(p + ".bn3", 4 * w)
            if b == 0:
                out.append((p + ".downsample.0.weight", (4 * w, cin, 1, 1)))
                out += _bn(p + ".downsample.1", 4 * w)
            cin = 4 * w
    out += [("fc.weight", (1000, 2048)), ("fc.bias", (1000,))]
    return out


def transformer_big(d_model: int = 1024, ffn: int = 4096, layers: int = 6,
                    vocab: int = 32768) -> List[NamedShape]:
    """Transformer "big", 6+6 blocks, one shared embedding:
    253 tensors, 209 911 808 elements."""
    def lin(name: str, o: int, i: int) -> List[NamedShape]:
        return [(name + ".weight", (o, i)), (name + ".bias", (o,))]

    def attn(name: str) -> List[NamedShape]:
        r: List[NamedShape] = []
        for proj in ("q_proj", "k_proj", "v_proj", "out_proj"):
            r += lin(f"{name}.{proj}", d_model, d_model)
        return r

    def ln(name: str) -> List[NamedShape]:
        return [(name + ".weight", (d_model,)), (name + ".bias", (d_model,))]

    out: List[NamedShape] = [("embed_tokens.weight", (vocab, d_model))]
    for l in range(layers):
        p = f"encoder.layers.{l}"
        out += attn(p + ".self_attn") + ln(p + ".self_attn_layer_norm")
        out += lin(p + ".fc1", ffn, d_model) + lin(p + ".fc2", d_model, ffn)
        out += ln(p + ".final_layer_norm")
    for l in range(layers):
        p = f"decoder.layers.{l}"
        out += attn(p + ".self_attn") + ln(p + ".self_attn_layer_norm")
        out += attn(p + ".encoder_attn") + ln(p + ".encoder_attn_layer_norm")
        out += lin(p + ".fc1", ffn, d_model) + lin(p + ".fc2", d_model, ffn)
        out += ln(p + ".final_layer_norm")
    return out


def ragged_mini() -> List[NamedShape]:
    """A small list made to exercise every edge of a multi-tensor kernel:
    lengths that are not multiples of 4, single elements, an empty tensor,
    lengths around tile sizes, and one tensor spanning several tiles."""
    sizes = [1, 2, 3, 5, 0, 63, 64, 65, 255, 257, 1000, 1023, 1025, 4095, 4097,
             7, 8191, 8193, 16384, 16385, 33, 70001, 4, 12, 131077, 9]
    return [(f"t{i}", (n,)) for i, n in enumerate(sizes)]


def numels(shapes: List[NamedShape]) -> List[int]:
    return [int(prod(s)) for _, s in shapes]


def total(shapes: List[NamedShape]) -> int:
    return sum(numels(shapes))
