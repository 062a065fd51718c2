"""Seeded synthetic gradients shaped like the paper's DNN workloads.

The paper measures on gradients of ResNets trained on CIFAR-10/100 and Tiny
ImageNet; neither the datasets nor trained weights exist here, so per-layer
Gaussian gradients (optionally with heavy-tailed outliers) stand in for them.
This module only draws random inputs: it holds none of the method's arithmetic
and is the one module both the HIP path's tests and the CPU oracle's tests use,
so that both consume exactly the same fp32 arrays.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import torch

from . import layers as _layers


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    d: int
    worker_comp: str          # "sign" | "topk" | "identity"
    server_comp: str
    worker_k: int
    server_k: int
    lr: float
    steps: int
    layer_sizes: List[int] = field(repr=False)
    log10_sigma_lo: float     # sigma_l log-uniform in [10**lo, 10**hi]; lo == hi == 0 -> sigma = 1
    log10_sigma_hi: float
    outlier_prob: float       # fraction of elements replaced by a Student-t(nu=2) variate
    blocks: Optional[List[int]] = field(default=None, repr=False)   # block offsets for the blockwise operator

    @property
    def alg_bytes_per_step(self) -> int:
        """Bytes the step must move: grads twice (once when the workers' operator does not look at them:
        random-k, identity), x in and out, e read twice and written."""
        reads_of_g = 1 if self.worker_comp in ("randk", "identity") else 2
        return (8 + 4 * reads_of_g) * self.N * self.d + 12 * self.d


def _mk(name, N, d, wc, sc, wk, sk, lr, steps, sizes, lo, hi, out) -> Workload:
    assert sum(sizes) == d
    return Workload(name, N, d, wc, sc, wk, sk, lr, steps, sizes, lo, hi, out)


def workloads() -> Dict[str, Workload]:
    r18, r50, vgg = _layers.resnet18_layers(), _layers.resnet50_layers(), _layers.vgg16_layers()
    d2, d3, d4, d5 = 1_048_576, sum(r18), sum(r50), sum(vgg)
    w = [
        _mk("c1_tiny_sign", 4, 65_536, "sign", "sign", 0, 0, 0.1, 20, [65_536], 0.0, 0.0, 0.0),
        _mk("c2_topk_mid", 8, d2, "topk", "topk", d2 // 100, d2 // 100, 0.05, 50,
            _layers.equal_layers(d2, 16), -3.0, 0.0, 0.0),
        _mk("c3_resnet18_sign", 16, d3, "sign", "sign", 0, 0, 0.1, 100, r18, -4.0, -1.0, 1e-3),
        _mk("c4_resnet50_topk", 32, d4, "topk", "topk", d4 // 1000, d4 // 1000, 0.1, 100, r50,
            -4.0, -1.0, 1e-3),
        _mk("c5_vgg16_mixed", 16, d5, "topk", "sign", d5 // 200, 0, 0.01, 50, vgg, -5.0, -2.0, 0.0),
        # same shape and inputs as c5 with the scaled-sign operator in both directions
        _mk("c5_vgg16_sign", 16, d5, "sign", "sign", 0, 0, 0.01, 50, vgg, -5.0, -2.0, 0.0),
    ]
    import dataclasses
    # the operator of the paper's experiments: Blockwise-SignSGD with 10 blocks for ResNet-18; the
    # paper does not say where the blocks are cut, so the 62 parameter tensors are grouped in order
    w.append(dataclasses.replace(w[2], name="c3_resnet18_blocksign", worker_comp="blocksign",
                                 server_comp="blocksign", blocks=layer_blocks(r18, 10)))
    # the ResNet-50 shape with random-k (Definition 3) in place of top-k, same k
    w.append(dataclasses.replace(w[3], name="c4_resnet50_randk", worker_comp="randk", server_comp="randk"))
    return {x.name: x for x in w}


def layer_blocks(sizes: List[int], nblocks: int) -> List[int]:
    """Offsets of `nblocks` consecutive groups of whole layers, as even in layer count as possible."""
    n = len(sizes)
    assert 1 <= nblocks <= n
    cuts = [round(i * n / nblocks) for i in range(nblocks + 1)]
    pre = [0]
    for sz in sizes:
        pre.append(pre[-1] + sz)
    return [pre[c] for c in cuts]


def scaled(w: Workload, N: Optional[int] = None, d: Optional[int] = None, **kw) -> Workload:
    """A smaller workload with the same recipe (layer sizes rescaled to sum to d)."""
    import dataclasses

    N = w.N if N is None else N
    d = w.d if d is None else d
    sizes = [max(1, s * d // w.d) for s in w.layer_sizes]
    while sum(sizes) > d:
        sizes[sizes.index(max(sizes))] -= 1
    sizes[sizes.index(max(sizes))] += d - sum(sizes)
    frac_w = w.worker_k / w.d
    frac_s = w.server_k / w.d
    blocks = None
    if w.blocks is not None:       # keep the number of blocks, cut at the rescaled positions
        cuts = sorted({max(1, min(d - 1, o * d // w.d)) for o in w.blocks[1:-1]})
        blocks = [0] + cuts + [d]
    upd = dict(N=N, d=d, layer_sizes=sizes, blocks=blocks,
               worker_k=max(1, int(frac_w * d)) if w.worker_comp == "topk" else 0,
               server_k=max(1, int(frac_s * d)) if w.server_comp == "topk" else 0)
    upd.update(kw)
    return dataclasses.replace(w, **upd)


class GradientSource:
    """grads(t) -> [N, d] fp32 tensor on `device`, a pure function of (seed, t).

    sigma_l is drawn once per layer from a generator seeded `seed` (fixed over
    steps and workers); step t draws its variates from a generator seeded
    `seed + 1 + t`.  Elements are i.i.d. sigma_l * z with z ~ N(0,1); with
    probability `outlier_prob` z is replaced by a Student-t(nu=2) variate
    z' / sqrt(-ln u), u ~ U(0,1).
    """

    def __init__(self, w: Workload, seed: int = 0, device: str = "cpu"):
        self.w, self.seed, self.device = w, int(seed), torch.device(device)
        g = torch.Generator(device="cpu")
        g.manual_seed(self.seed)
        u = torch.rand(len(w.layer_sizes), generator=g, dtype=torch.float64)
        log_sigma = w.log10_sigma_lo + (w.log10_sigma_hi - w.log10_sigma_lo) * u
        self.layer_sigma = (10.0 ** log_sigma).to(torch.float32)
        self._sigma = None

    def _sigma_vec(self) -> torch.Tensor:
        if self._sigma is None:
            sizes = torch.tensor(self.w.layer_sizes, dtype=torch.int64)
            self._sigma = torch.repeat_interleave(self.layer_sigma, sizes).to(self.device)
        return self._sigma

    def grads(self, t: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        w = self.w
        gen = torch.Generator(device=self.device)
        gen.manual_seed(self.seed + 1 + int(t))
        if out is None:
            out = torch.empty((w.N, w.d), dtype=torch.float32, device=self.device)
        assert out.shape == (w.N, w.d) and out.dtype == torch.float32
        flat_sigma = w.log10_sigma_lo == 0.0 and w.log10_sigma_hi == 0.0
        for i in range(w.N):  # row at a time bounds the temporaries to a few d
            row = out[i]
            row.normal_(generator=gen)
            if w.outlier_prob > 0.0:
                pick = torch.rand(w.d, generator=gen, device=self.device) < w.outlier_prob
                z2 = torch.randn(w.d, generator=gen, device=self.device)
                u = torch.rand(w.d, generator=gen, device=self.device).clamp_(min=1e-30)
                heavy = z2 / torch.sqrt(-torch.log(u))
                row.copy_(torch.where(pick, heavy, row))
                del pick, z2, u, heavy
            if not flat_sigma:
                row.mul_(self._sigma_vec())
        return out


def inject_ties(g: torch.Tensor, seed: int, frac_zero: float = 0.05, frac_dup: float = 0.05) -> torch.Tensor:
    """Edge-case structure for top-k tests: exact zeros, negative zeros and
    duplicated magnitudes (with both signs), placed by a seeded generator."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    flat = g.view(-1)
    n = flat.numel()
    nz = int(n * frac_zero)
    idx = torch.randperm(n, generator=gen)[:nz].to(g.device)
    flat[idx] = 0.0
    flat[idx[: nz // 2]] = -0.0
    nd = int(n * frac_dup)
    if nd >= 2:
        idx = torch.randperm(n, generator=gen)[:nd].to(g.device)
        vals = flat[idx[: max(1, nd // 8)]].abs()
        rep = vals[torch.randint(0, vals.numel(), (nd,), generator=gen).to(g.device)]
        sgn = (torch.randint(0, 2, (nd,), generator=gen).to(g.device).float() * 2 - 1)
        flat[idx] = rep * sgn
    return g

