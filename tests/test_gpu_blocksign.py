"""Blockwise-SignSGD (Definition 5) on the GPU against the oracle.
"""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))
import _harness as H  # noqa: E402
from _gpu import DEV, GPU_MARKS, PAIRS, SMALL_SHAPES, WL, check_descriptors, ctx_for, run_chain, say  # noqa: E402,F401

import workloads  # noqa: E402

pytestmark = GPU_MARKS


# ---- Blockwise-SignSGD (Definition 5) --------------------------------------------------------------
BLOCK_TABLES = {
    "one": lambda d: [0, d],
    "aligned": lambda d: [0, d // 4 // 4 * 4, d // 2 // 4 * 4, d],
    "ragged": lambda d: sorted({0, 1, 7, d // 3, d // 3 + 1, 2 * d // 3 + 5, d - 1, d}),
    "many": lambda d: list(range(0, d, max(1, d // 37))) + [d] if d % max(1, d // 37) else list(range(0, d + 1, max(1, d // 37))),
}


@pytest.mark.parametrize("table", list(BLOCK_TABLES))
@pytest.mark.parametrize("wc,sc", [("blocksign", "blocksign"), ("blocksign", "sign"), ("topk", "blocksign"),
                                   ("blocksign", "topk"), ("identity", "blocksign")])
@pytest.mark.parametrize("N,d", [(3, 5000), (4, 70_001), (2, 12_288)])
def test_blockwise_sign(N, d, wc, sc, table):
    say(f"case blocksign N={N} d={d} {wc}/{sc} table={table}")
    import oracle
    from paper_2402_11857_amd import LiecContext

    off = BLOCK_TABLES[table](d)
    assert off[0] == 0 and off[-1] == d and all(a < b for a, b in zip(off, off[1:]))
    k = max(1, d // 50)
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp=wc, server_comp=sc,
                         worker_k=k if wc == "topk" else 0, server_k=k if sc == "topk" else 0, lr=0.05)
    src = workloads.GradientSource(w, seed=d + N, device=DEV)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    with LiecContext(N, d, wc, sc, w.worker_k, w.server_k, w.lr) as ctx:
        ctx.set_blocks(off)
        for t in range(3):
            g = src.grads(t)
            ctx.step(g, x, e)
            tr = oracle.step_blocks(g.cpu().numpy(), xo, eo, wc, sc, w.lr, off, w.worker_k, w.server_k)
            ws, ss = ctx.block_scales()
            if wc == "blocksign":
                assert np.array_equal(np.array(ws, dtype=np.float32), tr.worker_scales), f"step {t}: worker block scales"
            if sc == "blocksign":
                assert np.array_equal(np.array(ss, dtype=np.float32), tr.server_scales), f"step {t}: server block scales"
            assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo), f"step {t}"
        assert ctx.info().nonfinite == 0


def test_blockwise_sign_needs_a_block_table_and_validates_it():
    say("case blocksign errors")
    from paper_2402_11857_amd import LiecContext, LiecError

    N, d = 2, 4096
    g = torch.randn((N, d), device=DEV)
    x = torch.zeros((N, d), device=DEV)
    e = torch.zeros(d, device=DEV)
    with LiecContext(N, d, "blocksign", "blocksign", 0, 0, 0.1) as ctx:
        with pytest.raises(LiecError):
            ctx.step(g, x, e)                       # no table yet
        for bad in ([0, 100, 100, d], [1, d], [0, d - 1], [0, 3000, 2000, d]):
            with pytest.raises(LiecError):
                ctx.set_blocks(bad)
        ctx.set_blocks([0, 1000, d])
        ctx.step(g, x, e)
        ctx.set_blocks([0, d])                      # a new table replaces the old one
        ctx.step(g, x, e)
        torch.cuda.synchronize()


def test_full_size_c3_resnet18_blocksign():
    import oracle
    w = WL["c3_resnet18_blocksign"]
    say(f"case full size {w.name} blocks={len(w.blocks) - 1}")
    src = workloads.GradientSource(w, seed=0, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    with ctx_for(w) as ctx:
        ctx.set_blocks(w.blocks)
        for t in range(2):
            g = src.grads(t)
            ctx.step(g, x, e)
            tr = oracle.step_blocks(g.cpu().numpy(), xo, eo, "blocksign", "blocksign", w.lr, w.blocks)
            ws, ss = ctx.block_scales()
            assert np.array_equal(np.array(ws, dtype=np.float32), tr.worker_scales)
            assert np.array_equal(np.array(ss, dtype=np.float32), tr.server_scales)
            assert H.bit_equal(e.cpu().numpy(), eo)
            for i in range(w.N):
                assert H.bit_equal(x[i].cpu().numpy(), xo[i]), f"step {t} row {i}"
