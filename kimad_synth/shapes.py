"""Per-tensor shape lists of the public architectures the synthetic gradient sets imitate.

One entry per parameter tensor (weights and biases separate), in the order a
framework would list them.  A "layer" of the compression method is one such
tensor: the paper compresses per layer (Section 4.2, "Setting").
"""
from __future__ import annotations

from typing import List, Tuple

Shape = Tuple[int, ...]


def numel(shape: Shape) -> int:
    n = 1
    for s in shape:
        n *= int(s)
    return n


def mlp_shapes() -> List[Shape]:
    """784-256-128-10 perceptron: 6 tensors, 235,146 elements."""
    return [(784, 256), (256,), (256, 128), (128,), (128, 10), (10,)]


def _bn(c: int) -> List[Shape]:
    return [(c,), (c,)]


def resnet18_shapes(num_classes: int = 1000) -> List[Shape]:
    """ResNet-18 with an ImageNet head: 62 tensors, 11,689,512 elements."""
    out: List[Shape] = [(64, 3, 7, 7)] + _bn(64)
    inplanes = 64
    for stage, planes in enumerate((64, 128, 256, 512)):
        for block in range(2):
            out += [(planes, inplanes, 3, 3)] + _bn(planes)
            out += [(planes, planes, 3, 3)] + _bn(planes)
            if block == 0 and stage > 0:
                out += [(planes, inplanes, 1, 1)] + _bn(planes)
            inplanes = planes
    out += [(num_classes, 512), (num_classes,)]
    return out


def resnet50_shapes(num_classes: int = 1000) -> List[Shape]:
    """ResNet-50 (bottleneck blocks 3/4/6/3): 161 tensors, 25,557,032 elements."""
    out: List[Shape] = [(64, 3, 7, 7)] + _bn(64)
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for block in range(blocks):
            out += [(planes, inplanes, 1, 1)] + _bn(planes)
            out += [(planes, planes, 3, 3)] + _bn(planes)
            out += [(planes * 4, planes, 1, 1)] + _bn(planes * 4)
            if block == 0:
                out += [(planes * 4, inplanes, 1, 1)] + _bn(planes * 4)
            inplanes = planes * 4
    out += [(num_classes, 2048), (num_classes,)]
    return out


def gpt2_small_shapes(n_layer: int = 12, n_embd: int = 768, vocab: int = 50257,
                      n_ctx: int = 1024) -> List[Shape]:
    """GPT-2 small: 148 tensors, 124,439,808 elements at the defaults."""
    out: List[Shape] = [(vocab, n_embd), (n_ctx, n_embd)]
    for _ in range(n_layer):
        out += [(n_embd,), (n_embd,)]                          # ln_1
        out += [(n_embd, 3 * n_embd), (3 * n_embd,)]            # attention qkv
        out += [(n_embd, n_embd), (n_embd,)]                    # attention out-proj
        out += [(n_embd,), (n_embd,)]                          # ln_2
        out += [(n_embd, 4 * n_embd), (4 * n_embd,)]            # mlp fc
        out += [(4 * n_embd, n_embd), (n_embd,)]                # mlp proj
    out += [(n_embd,), (n_embd,)]                              # ln_f
    return out


def llama_shapes(n_layer: int = 24, hidden: int = 2048, ffn: int = 5632,
                 vocab: int = 32000) -> List[Shape]:
    """Llama-style decoder with a tied head: 218 tensors, 1,298,761,728 elements at the defaults."""
    out: List[Shape] = [(vocab, hidden)]
    for _ in range(n_layer):
        out += [(hidden,)]                                     # input rmsnorm
        out += [(hidden, hidden)] * 4                          # q, k, v, o
        out += [(hidden,)]                                     # post-attention rmsnorm
        out += [(ffn, hidden), (ffn, hidden), (hidden, ffn)]   # gate, up, down
    out += [(hidden,)]
    return out
