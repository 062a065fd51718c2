"""Shared pieces of the GPU parity tests: the context helper, the chained-step comparison against the
oracle, and the small shapes every operator pair is run on.

Integer-valued results (top-k index sets, sign bits, thresholds, cut-offs) must be bit-exact;
fp32 state (x, server error, scales) must agree within 1e-5 relative after one step and 1e-4
after a chain.  With the conventions both sides follow the expected outcome is bit identity.
"""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))
import _harness as H  # noqa: E402
from _say import say  # noqa: E402,F401

import workloads  # noqa: E402

GPU_MARKS = [pytest.mark.gpu, pytest.mark.skipif(not torch.cuda.is_available(), reason="needs an MI355X")]

DEV = "cuda:0"
WL = workloads.workloads()


def ctx_for(w, **kw):
    from paper_2402_11857_amd import LiecContext

    return LiecContext(w.N, w.d, w.worker_comp, w.server_comp, w.worker_k, w.server_k, w.lr, **kw)


def check_descriptors(ctx, w, wdesc, sdesc, g_host, v_host, label):
    """Scales, thresholds and cut-offs of the last step against the oracle's."""
    got = ctx.worker_desc()
    info = ctx.info()
    if w.worker_comp == "sign":
        for i in range(w.N):
            assert got["scale"][i] == np.float32(wdesc[i].scale), f"{label}: worker {i} scale"
            assert abs(got["l1"][i] - wdesc[i].l1) <= 1e-12 * wdesc[i].l1
    if w.worker_comp in ("topk", "randk"):
        for i in range(w.N):
            assert got["tau_key"][i] == wdesc[i].tau_key, f"{label}: worker {i} threshold key"
            assert got["cutoff"][i] == wdesc[i].cutoff, f"{label}: worker {i} tie cut-off"
    if w.server_comp == "sign":
        assert info.server_scale == np.float32(sdesc.scale), f"{label}: server scale"
    if w.server_comp in ("topk", "randk"):
        assert info.server_tau_key == sdesc.tau_key, f"{label}: server threshold key"
        assert info.server_cutoff == sdesc.cutoff, f"{label}: server tie cut-off"
    assert info.nonfinite == 0


def run_chain(w, steps, seed=0, teacher_forced=False, mutate=None, check_descs=True, tol_end=H.TOL_CHAIN,
               rk_seed=0, force_mode=None, stats=None):
    """Runs `steps` chained steps on both sides and compares after every step.  rk_seed seeds the
    random-k draws (draw t in step t); force_mode[t], when given, is the search mode forced before step t;
    stats, when given, receives the context's band_misses count at the end of the chain."""
    src = workloads.GradientSource(w, seed=seed, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo = np.zeros((w.N, w.d), dtype=np.float32)
    eo = np.zeros(w.d, dtype=np.float32)
    exact = True
    with ctx_for(w) as ctx:
        ctx.set_random(rk_seed, 0)
        for t in range(steps):
            g = src.grads(t)
            if mutate is not None:
                g = mutate(g, t)
            gh = g.cpu().numpy()
            if teacher_forced and t > 0:
                x.copy_(torch.from_numpy(xo))
                e.copy_(torch.from_numpy(eo))
            if force_mode is not None and force_mode[t] is not None:
                ctx.force_search_mode(force_mode[t])
            ctx.step(g, x, e)
            wdesc, sdesc, v, p, P = H.oracle_step_rows(gh, xo, eo, w.worker_comp, w.server_comp, w.lr,
                                                       w.worker_k, w.server_k, rng=(rk_seed, t))
            xg, eg = x.cpu().numpy(), e.cpu().numpy()
            label = f"{w.name} N={w.N} d={w.d} step {t}"
            if check_descs:
                check_descriptors(ctx, w, wdesc, sdesc, gh, v, label)
            tol = H.TOL_STEP if (t == 0 or teacher_forced) else tol_end
            assert H.rel_err(eg, eo) <= tol, f"{label}: server error"
            assert H.rel_err(xg, xo) <= tol, f"{label}: models"
            # integer-valued parts of the state: the sign pattern / support of the new error
            if w.server_comp in ("topk", "randk"):
                assert np.array_equal(eg == 0, eo == 0), f"{label}: server index set"
            exact = exact and H.bit_equal(xg, xo) and H.bit_equal(eg, eo)
        if stats is not None:
            stats["band_misses"] = ctx.info().band_misses
    return exact


SMALL_SHAPES = [(1, 1), (2, 3), (3, 255), (4, 1024), (2, 1025), (5, 4100), (3, 50_003), (8, 70_000)]
PAIRS = [("sign", "sign"), ("topk", "topk"), ("topk", "sign"), ("sign", "topk"), ("identity", "identity"),
         ("identity", "sign"), ("topk", "identity"), ("sign", "identity"), ("identity", "topk")]
