"""Pins for the oracle's averaging iteration (Algorithm 1, the branches taken every
floor(1/delta)-th iteration): hand-worked example, the closed form printed after the algorithm,
models unified and error cleared, Lemma 3 across chains that mix both kinds of iteration."""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "liec_step_worked_examples.json")


def _grads(rng, N, d):
    sigma = 10.0 ** rng.uniform(-3, 0, size=8)
    s = np.repeat(sigma, -(-d // 8))[:d]
    return (rng.standard_normal((N, d)) * s).astype(np.float32)


def test_hand_worked_averaging_iteration(oracle):
    with open(GOLDEN) as f:
        cases = json.load(f)["sync_cases"]
    for c in cases:
        g = np.array(c["g"], dtype=np.float32)
        x = np.array(c["x0"], dtype=np.float32)
        e = np.array(c["e0"], dtype=np.float32)
        v = oracle.step_sync(g, x, e, c["lr"], want_v=True)
        assert np.array_equal(v, np.array(c["v"], dtype=np.float32))
        assert np.array_equal(e, np.array(c["e1"], dtype=np.float32))
        assert np.array_equal(x, np.array(c["x1"], dtype=np.float32))


@pytest.mark.parametrize("N", [1, 3, 8])
def test_models_are_unified_error_cleared_and_closed_form_holds(oracle, N):
    # x_{t+1}^i = mean_i x_t^i - eta (mean_i g_i + e_t) for every i; e_{t+1} = 0
    rng = np.random.default_rng(N)
    d, lr = 3001, 0.05
    g = _grads(rng, N, d)
    x = rng.standard_normal((N, d)).astype(np.float32)
    e = (0.1 * rng.standard_normal(d)).astype(np.float32)
    expect = x.astype(np.float64).mean(axis=0) - np.float64(np.float32(lr)) * (g.astype(np.float64).mean(axis=0) + e)
    oracle.step_sync(g, x, e, lr)
    assert not e.any()
    assert all(np.array_equal(x[0], x[i]) for i in range(N))
    assert np.abs(x[0] - expect).max() <= 4 * 2.0 ** -23 * max(1.0, np.abs(expect).max())


def test_single_worker_averaging_iteration_is_sgd_on_the_compensated_gradient(oracle):
    rng = np.random.default_rng(4)
    d, lr = 100, np.float32(0.25)
    g = rng.integers(-8, 9, size=(1, d)).astype(np.float32) / np.float32(8)
    x = rng.integers(-8, 9, size=(1, d)).astype(np.float32)
    e = rng.integers(-8, 9, size=d).astype(np.float32) / np.float32(16)
    expect = x[0] - lr * (g[0] + e)            # exact in fp32 for these dyadic values
    oracle.step_sync(g, x, e, float(lr))
    assert np.array_equal(x[0], expect)


@pytest.mark.parametrize("wc,sc", [("sign", "sign"), ("topk", "topk"), ("topk", "sign")])
@pytest.mark.parametrize("period", [2, 5])
def test_lemma3_and_drift_reset_across_mixed_chains(oracle, wc, sc, period):
    # Lemma 3 holds at every t; right after an averaging iteration e = 0, so mean x equals the virtual
    # sequence and every local model equals the mean.
    rng = np.random.default_rng(period)
    N, d, lr, T = 4, 1500, 0.1, 12
    x0 = rng.standard_normal(d).astype(np.float32)
    x = np.tile(x0, (N, 1))
    e = np.zeros(d, dtype=np.float32)
    virt = x0.astype(np.float64)
    eta = np.float64(np.float32(lr))
    for t in range(T):
        g = _grads(rng, N, d)
        if (t + 1) % period == 0:
            oracle.step_sync(g, x, e, lr)
            assert not e.any()
            assert all(np.array_equal(x[0], x[i]) for i in range(N))
        else:
            oracle.step(g, x, e, wc, sc, lr, worker_k=30, server_k=45)
        virt = virt - eta * g.astype(np.float64).mean(axis=0)
        lhs = x.astype(np.float64).mean(axis=0) - virt
        scale = max(np.abs(x).max(), np.abs(e).max(), 1.0)
        assert np.abs(lhs - eta * e).max() <= (t + 1) * 4 * 2.0 ** -23 * scale


def test_averaging_iteration_rounds_once_per_fused_operation(oracle):
    # same numbers as the compressed iteration's pins: 3 * fl32(1/3) - 1 = 2^-25 only if the multiply
    # and the add of the global error round once ...
    g = np.ones((3, 1), dtype=np.float32)
    x = np.zeros((3, 1), dtype=np.float32)
    e = np.array([-1.0], dtype=np.float32)
    oracle.step_sync(g, x, e, 1.0)
    assert np.all(x == np.float32(-(2.0 ** -25))) and e[0] == 0.0
    # ... and fl32(0.3) - fl32(0.1) * 3 = 2^-27 only if the update does
    g = np.array([[3.0]], dtype=np.float32)
    x = np.array([[0.3]], dtype=np.float32)
    e = np.zeros(1, dtype=np.float32)
    oracle.step_sync(g, x, e, float(np.float32(0.1)))
    assert x[0, 0] == np.float32(2.0 ** -27)
