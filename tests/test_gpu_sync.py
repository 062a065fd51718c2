"""The averaging iteration of Algorithm 1 on the GPU against the oracle.
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


# ---- averaging iteration of Algorithm 1 ------------------------------------------------------------
@pytest.mark.parametrize("N,d", [(1, 1), (3, 1023), (4, 4096), (5, 50_003), (16, 70_000)])
def test_sync_iteration_small_shapes(N, d):
    say(f"case sync N={N} d={d}")
    from paper_2402_11857_amd import LiecContext

    import oracle
    rng = np.random.default_rng(N * 7 + d)
    g = rng.standard_normal((N, d)).astype(np.float32)
    x = rng.standard_normal((N, d)).astype(np.float32)
    e = (0.1 * rng.standard_normal(d)).astype(np.float32)
    gd, xd, ed = (torch.from_numpy(a).to(DEV) for a in (g, x, e))
    with LiecContext(N, d, "sign", "sign", 0, 0, 0.05) as ctx:
        ctx.step_sync(gd, xd, ed)
        torch.cuda.synchronize()
    oracle.step_sync(g, x, e, 0.05)
    assert H.bit_equal(xd.cpu().numpy(), x) and H.bit_equal(ed.cpu().numpy(), e)
    assert not e.any()


@pytest.mark.parametrize("wc,sc", [("sign", "sign"), ("topk", "topk"), ("topk", "sign")])
def test_mixed_chain_with_averaging_period(wc, sc):
    """Algorithm 1 in full: compressed iterations, an averaging iteration every 4th step."""
    say(f"case period chain {wc}/{sc}")
    import oracle
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=120_000, worker_comp=wc, server_comp=sc,
                         worker_k=1200 if wc == "topk" else 0, server_k=1200 if sc == "topk" else 0)
    src = workloads.GradientSource(w, seed=11, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    with ctx_for(w) as ctx:
        for t in range(13):
            g = src.grads(t)
            gh = g.cpu().numpy()
            ctx.iteration(t, 4, g, x, e)               # Algorithm 1 as a whole: the library picks the branch
            if (t + 1) % 4 == 0:
                oracle.step_sync(gh, xo, eo, w.lr)
            else:
                H.oracle_step_rows(gh, xo, eo, wc, sc, w.lr, w.worker_k, w.server_k)
            assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo), f"step {t}"


def test_full_size_c3_sync_iteration():
    import oracle
    w = WL["c3_resnet18_sign"]
    say(f"case full size sync {w.name}")
    src = workloads.GradientSource(w, seed=2, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    with ctx_for(w) as ctx:
        g = src.grads(0)
        ctx.step(g, x, e)                      # make the local models differ first
        H.oracle_step_rows(g.cpu().numpy(), xo, eo, "sign", "sign", w.lr)
        g = src.grads(1)
        ctx.step_sync(g, x, e)
        oracle.step_sync(g.cpu().numpy(), xo, eo, w.lr)
    assert H.bit_equal(e.cpu().numpy(), eo)
    for i in range(w.N):
        assert H.bit_equal(x[i].cpu().numpy(), xo[i]), f"row {i}"
