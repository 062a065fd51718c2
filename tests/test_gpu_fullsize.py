"""The large configurations in the launch configuration the bench times, every element of the new state
compared with the oracle: each of them at full size for a few steps, and their whole chains (the step
counts the configurations name: 100, 100, 50) at full size where the oracle keeps up (the ResNet-18
shape) or with the row length cut to a sixteenth at full N (the ResNet-50 and VGG-16 shapes).
"""
import os
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))
import _harness as H  # noqa: E402
from _gpu import DEV, GPU_MARKS, PAIRS, SMALL_SHAPES, WL, check_descriptors, ctx_for, run_chain, say  # noqa: E402,F401

import workloads  # noqa: E402

pytestmark = GPU_MARKS

_ORACLE_THREAD = ThreadPoolExecutor(max_workers=1)       # the oracle's step runs beside the GPU's


def _assert_same(got, want, tol, what):
    """Bit identity is the expected outcome; the relative error is only worked out to word the failure."""
    if H.bit_equal(got, want):
        return
    err = H.rel_err(got, want)
    assert err <= tol, f"{what}: relative error {err:.3e} above {tol:.0e}"
    raise AssertionError(f"{what}: within {tol:.0e} (relative error {err:.3e}) but not bit-identical")


def _chain(w, steps, label, seed=0, mantissa_bits=23, expect_slow_rows=None, progress_every=1):
    """`steps` chained steps on both sides; after every step the descriptors, the server error and every
    model row are compared.  The oracle works on step t while the GPU side copies its results of step t
    back and draws the gradients of step t + 1."""
    say(f"case {label} N={w.N} d={w.d} {w.worker_comp}/{w.server_comp} k={w.worker_k}/{w.server_k} steps={steps} "
        f"mantissa bits={mantissa_bits}")
    src = workloads.GradientSource(w, seed=seed, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo = np.zeros((w.N, w.d), dtype=np.float32)
    eo = np.zeros(w.d, dtype=np.float32)

    def draw(t):
        g = src.grads(t)
        if mantissa_bits < 23:                   # gradients as a low-precision backward pass leaves them
            g = (g.view(torch.int32) & -(1 << (23 - mantissa_bits))).view(torch.float32).contiguous()
        return g, g.cpu().numpy()

    with ctx_for(w) as ctx:
        ctx.set_random(seed + 1000, 0)
        g, gh = draw(0)
        for t in range(steps):
            fut = _ORACLE_THREAD.submit(H.oracle_step_rows, gh, xo, eo, w.worker_comp, w.server_comp, w.lr,
                                        w.worker_k, w.server_k, (seed + 1000, t))
            ctx.step(g, x, e)
            info = ctx.info()                                    # synchronises the step
            eg = e.cpu().numpy()
            nxt = draw(t + 1) if t + 1 < steps else (None, None)
            wdesc, sdesc, v, p, P = fut.result()
            del P, p
            what = f"{label} step {t}"
            check_descriptors(ctx, w, wdesc, sdesc, gh, v, what)
            del v
            if expect_slow_rows is not None:
                assert info.slow_rows == expect_slow_rows, f"{what}: rows in the general search"
            tol = H.TOL_STEP if t == 0 else H.TOL_CHAIN
            _assert_same(eg, eo, tol, f"{what}: server error")
            for i in range(w.N):                 # row at a time keeps the host copies small
                _assert_same(x[i].cpu().numpy(), xo[i], tol, f"{what}: model of worker {i}")
            if (t + 1) % progress_every == 0 or t + 1 == steps:
                say(f"  step {t} compared (row-steps whose predicted band failed so far: {info.band_misses})")
            g, gh = nxt


def _full_size_steps(name, steps, **kw):
    _chain(WL[name], steps, f"full size {name}", **kw)


def _sixteenth(name):
    """Same recipe, operators, N, learning rate and k / d with the row length cut to a sixteenth (a multiple
    of 4, so that the 128-bit path the bench times is the one that runs)."""
    w = WL[name]
    return workloads.scaled(w, d=(w.d // 16) // 4 * 4)


# ---- whole chains: the configurations' own step counts -------------------------------------------
def test_whole_chain_c3_resnet18_sign_full_size():
    w = WL["c3_resnet18_sign"]
    _chain(w, w.steps, "whole chain, full size c3_resnet18_sign", progress_every=10)


def test_whole_chain_c4_resnet50_topk_full_workers_sixteenth_of_the_columns():
    """100 steps at N = 32: the server error at its stationary size, the threshold predicted from the
    trajectory of the last thresholds at every step after the second."""
    w = _sixteenth("c4_resnet50_topk")
    _chain(w, WL["c4_resnet50_topk"].steps, "whole chain, d/16 c4_resnet50_topk", progress_every=10, expect_slow_rows=0)


def test_whole_chain_c5_vgg16_mixed_full_workers_sixteenth_of_the_columns():
    w = _sixteenth("c5_vgg16_mixed")
    _chain(w, WL["c5_vgg16_mixed"].steps, "whole chain, d/16 c5_vgg16_mixed", progress_every=10, expect_slow_rows=0)


# ---- full-size configurations, a few steps each ----------------------------------------------------
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
