"""The compressed step under HIP graph capture.
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


# ---- the step under HIP graph capture ----------------------------------------------------------------
@pytest.mark.parametrize("wc,sc", [("sign", "sign"), ("topk", "topk"), ("topk", "sign"), ("randk", "randk")])
def test_step_captured_in_a_hip_graph_replays_like_eager_steps(wc, sc):
    """liec_step neither allocates, synchronises nor copies, and every decision of the threshold
    search is taken on the device, so a caller may capture it once and replay it; each replay is
    compared with the oracle, with eager work and synchronisation between the replays."""
    say(f"case graph capture {wc}/{sc}")
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=200_003 if wc == "sign" else 200_000, worker_comp=wc, server_comp=sc,
                         worker_k=2000 if wc != "sign" else 0, server_k=6000 if sc != "sign" else 0)
    src = workloads.GradientSource(w, seed=13, device=DEV)
    gs = [src.grads(t) for t in range(6)]
    g_static = torch.empty_like(gs[0])
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with ctx_for(w, stream=s) as ctx, torch.cuda.stream(s):
        ctx.set_random(31, 0)
        g_static.copy_(gs[0])
        ctx.step(g_static, x, e)                                  # one eager step first
        H.oracle_step_rows(gs[0].cpu().numpy(), xo, eo, wc, sc, w.lr, w.worker_k, w.server_k, rng=(31, 0))
        s.synchronize()
        graph = torch.cuda.CUDAGraph()
        graph.capture_begin()
        ctx.step(g_static, x, e)                                  # recorded, not run
        graph.capture_end()
        s.synchronize()
        assert H.bit_equal(x.cpu().numpy(), xo), "capturing must not run the step"
        for t in range(1, 5):
            g_static.copy_(gs[t])
            graph.replay()
            H.oracle_step_rows(gs[t].cpu().numpy(), xo, eo, wc, sc, w.lr, w.worker_k, w.server_k, rng=(31, t))
            s.synchronize()
            assert ctx.info().nonfinite == 0                      # eager work between the replays
            assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo), f"replay {t}"
        g_static.copy_(gs[5])
        ctx.step(g_static, x, e)                                  # and an eager step after the replays
        H.oracle_step_rows(gs[5].cpu().numpy(), xo, eo, wc, sc, w.lr, w.worker_k, w.server_k, rng=(31, 5))
        s.synchronize()
        assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo)
        if "randk" in (wc, sc):
            assert ctx.get_random() == (31, 6)
        del graph
