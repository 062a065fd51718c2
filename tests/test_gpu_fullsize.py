"""The large configurations at full size, in the launch configuration the bench times: every element
of the new state compared with the oracle.
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


# ---- full-size configurations, in the launch configuration the bench times -------------------
def _full_size_steps(name, steps, seed=0, mantissa_bits=23, expect_slow_rows=None):
    w = WL[name]
    say(f"case full size {name} N={w.N} d={w.d} steps={steps} mantissa bits={mantissa_bits}")
    src = workloads.GradientSource(w, seed=seed, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo = np.zeros((w.N, w.d), dtype=np.float32)
    eo = np.zeros(w.d, dtype=np.float32)
    with ctx_for(w) as ctx:
        ctx.set_random(seed + 1000, 0)
        for t in range(steps):
            g = src.grads(t)
            if mantissa_bits < 23:                   # gradients as a low-precision backward pass leaves them
                g = (g.view(torch.int32) & -(1 << (23 - mantissa_bits))).view(torch.float32).contiguous()
            ctx.step(g, x, e)
            gh = g.cpu().numpy()
            del g
            wdesc, sdesc, v, p, P = H.oracle_step_rows(gh, xo, eo, w.worker_comp, w.server_comp, w.lr,
                                                       w.worker_k, w.server_k, rng=(seed + 1000, t))
            say(f"  oracle step {t} done")
            check_descriptors(ctx, w, wdesc, sdesc, gh, v, f"{name} step {t}")
            if expect_slow_rows is not None:
                assert ctx.info().slow_rows == expect_slow_rows, f"{name} step {t}: rows in the general search"
            del P, gh
            eg = e.cpu().numpy()
            assert H.rel_err(eg, eo) <= (H.TOL_STEP if t == 0 else H.TOL_CHAIN)
            assert H.bit_equal(eg, eo), f"{name} step {t}: server error not bit-identical"
            for i in range(w.N):     # row at a time keeps the host copies small
                xi = x[i].cpu().numpy()
                assert H.rel_err(xi, xo[i]) <= (H.TOL_STEP if t == 0 else H.TOL_CHAIN), f"{name} step {t} row {i}"
                assert H.bit_equal(xi, xo[i]), f"{name} step {t} row {i}: model not bit-identical"


def test_full_size_c3_resnet18_sign():
    _full_size_steps("c3_resnet18_sign", steps=5)


def test_full_size_c4_resnet50_topk():
    _full_size_steps("c4_resnet50_topk", steps=3)       # cold, predicted band, band extrapolated from two thresholds


def test_full_size_c5_vgg16_mixed():
    _full_size_steps("c5_vgg16_mixed", steps=3)       # cold, predicted band, band extrapolated from two thresholds


def test_full_size_c5_vgg16_sign():
    _full_size_steps("c5_vgg16_sign", steps=2)


def test_full_size_c4_resnet50_randk():
    _full_size_steps("c4_resnet50_randk", steps=2)


def test_full_size_c4_resnet50_topk_on_bf16_like_gradients():
    """7 mantissa bits: tens of thousands of entries of a row share the threshold; no row may need the
    general search."""
    _full_size_steps("c4_resnet50_topk", steps=2, mantissa_bits=7, expect_slow_rows=0)
