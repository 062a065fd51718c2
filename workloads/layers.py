"""Parameter-tensor sizes of the three architectures whose gradient shapes the
synthetic workloads imitate (the paper trains ResNets on CIFAR / Tiny ImageNet;
VGG-16 is the large-d stress shape).  Sizes are derived here by arithmetic from
the published layer definitions (ImageNet heads, 1000 classes); no weights and
no third-party code are involved.  Used only to give the synthetic gradients a
per-layer scale structure.
"""
from __future__ import annotations

from typing import List


def _conv(c_in: int, c_out: int, k: int) -> int:
    return c_out * c_in * k * k


def _bn(c: int) -> List[int]:
    return [c, c]  # scale and shift


def resnet18_layers() -> List[int]:
    sizes: List[int] = [_conv(3, 64, 7)] + _bn(64)
    c_in = 64
    for stage, c in enumerate((64, 128, 256, 512)):
        for block in range(2):
            first = block == 0
            sizes += [_conv(c_in if first else c, c, 3)] + _bn(c)
            sizes += [_conv(c, c, 3)] + _bn(c)
            if first and stage > 0:
                sizes += [_conv(c_in, c, 1)] + _bn(c)
        c_in = c
    sizes += [512 * 1000, 1000]
    assert len(sizes) == 62 and sum(sizes) == 11_689_512, (len(sizes), sum(sizes))
    return sizes


def resnet50_layers() -> List[int]:
    sizes: List[int] = [_conv(3, 64, 7)] + _bn(64)
    c_in = 64
    for c, blocks in zip((64, 128, 256, 512), (3, 4, 6, 3)):
        for block in range(blocks):
            first = block == 0
            sizes += [_conv(c_in if first else 4 * c, c, 1)] + _bn(c)
            sizes += [_conv(c, c, 3)] + _bn(c)
            sizes += [_conv(c, 4 * c, 1)] + _bn(4 * c)
            if first:
                sizes += [_conv(c_in, 4 * c, 1)] + _bn(4 * c)
        c_in = 4 * c
    sizes += [2048 * 1000, 1000]
    assert len(sizes) == 161 and sum(sizes) == 25_557_032, (len(sizes), sum(sizes))
    return sizes


def vgg16_layers() -> List[int]:
    sizes: List[int] = []
    c_in = 3
    for c in (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512):
        sizes += [_conv(c_in, c, 3), c]
        c_in = c
    for n_in, n_out in ((25088, 4096), (4096, 4096), (4096, 1000)):
        sizes += [n_in * n_out, n_out]
    assert len(sizes) == 32 and sum(sizes) == 138_357_544, (len(sizes), sum(sizes))
    return sizes


def equal_layers(d: int, n: int) -> List[int]:
    assert d % n == 0
    return [d // n] * n
