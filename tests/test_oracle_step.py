"""Pins for the oracle's whole step (Algorithm 1, compressed iteration).

Checks are invariants and special cases the paper fixes: the hand-worked
examples under tests/golden/, identity compressor == P-SGD, Lemma 3 (mean model
minus virtual sequence equals eta times the global error), the per-worker drift
identity from the proof of Lemma 6, and the two one-sided ablations.
"""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "liec_step_worked_examples.json")

COMBOS = [("sign", "sign"), ("topk", "topk"), ("topk", "sign"), ("sign", "topk"),
          ("identity", "sign"), ("topk", "identity"), ("identity", "identity"),
          ("randk", "randk"), ("randk", "sign"), ("topk", "randk")]


def _grads(rng, N, d):
    sigma = 10.0 ** rng.uniform(-3, 0, size=8)
    s = np.repeat(sigma, -(-d // 8))[:d]
    return (rng.standard_normal((N, d)) * s).astype(np.float32)


# -- independent statements of the operators, used only to re-derive delta_i = g_i - C(g_i) --
def _np_sign(v):
    s = np.float32(np.sum(np.abs(v.astype(np.float64))) / v.size)
    return np.where(v < 0, -s, s).astype(np.float32)


def _np_topk(v, k):
    order = np.lexsort((np.arange(v.size), -np.abs(v.astype(np.float64))))
    out = np.zeros_like(v)
    out[order[:k]] = v[order[:k]]
    return out


def _np_compress(comp, v, k):
    return {"sign": _np_sign, "identity": lambda a: a.copy(), "topk": lambda a: _np_topk(a, k)}[comp](v)


def test_hand_worked_examples(oracle):
    with open(GOLDEN) as f:
        cases = json.load(f)["cases"]
    assert len(cases) >= 2
    for c in cases:
        g = np.array(c["g"], dtype=np.float32)
        x = np.array(c["x0"], dtype=np.float32)
        e = np.array(c["e0"], dtype=np.float32)
        tr = oracle.step(g, x, e, c["worker_comp"], c["server_comp"], c["lr"],
                         c["worker_k"], c["server_k"], trace=True)
        assert np.array_equal(tr.v, np.array(c["v"], dtype=np.float32)), c["name"]
        assert np.array_equal(tr.p, np.array(c["p"], dtype=np.float32)), c["name"]
        assert np.array_equal(e, np.array(c["e1"], dtype=np.float32)), c["name"]
        assert np.array_equal(x, np.array(c["x1"], dtype=np.float32)), c["name"]
        if "worker_scales" in c:
            assert [w.scale for w in tr.worker] == c["worker_scales"]
            assert tr.server.scale == c["server_scale"]
        if "worker_kept" in c:
            for i, kept in enumerate(c["worker_kept"]):
                assert sorted(np.nonzero(tr.P[i])[0].tolist()) == kept
            assert sorted(np.nonzero(tr.p)[0].tolist()) == c["server_kept"]


@pytest.mark.parametrize("N", [1, 3, 8])
def test_identity_compressor_is_parallel_sgd(oracle, N):
    # P-SGD: every worker applies the average gradient; no error is ever produced.
    rng = np.random.default_rng(N)
    d, lr, T = 501, np.float32(0.05), 6
    x = np.tile(rng.standard_normal(d).astype(np.float32), (N, 1))
    e = np.zeros(d, dtype=np.float32)
    ref = x[0].astype(np.float64)
    for _ in range(T):
        g = _grads(rng, N, d)
        oracle.step(g, x, e, "identity", "identity", float(lr))
        ref = ref - float(lr) * np.mean(g.astype(np.float64), axis=0)
        assert not e.any()
        assert all(np.array_equal(x[0], x[i]) for i in range(N))
    assert np.allclose(x[0], ref, rtol=0, atol=1e-6 * (1 + np.abs(ref).max()))


def test_identity_compressor_single_step_is_bit_exact_psgd(oracle):
    # with N a power of two the fp32 average is exact up to the sequential fp32 sum
    rng = np.random.default_rng(0)
    N, d, lr = 4, 300, np.float32(0.25)
    g = rng.integers(-8, 9, size=(N, d)).astype(np.float32) / np.float32(16)   # sums are exact
    x0 = rng.integers(-8, 9, size=d).astype(np.float32)
    x = np.tile(x0, (N, 1))
    e = np.zeros(d, dtype=np.float32)
    oracle.step(g, x, e, "identity", "identity", float(lr))
    expect = x0 - lr * g.mean(axis=0, dtype=np.float64).astype(np.float32)
    assert all(np.array_equal(x[i], expect) for i in range(N))


@pytest.mark.parametrize("wc,sc", COMBOS)
def test_lemma3_mean_model_minus_virtual_sequence_is_eta_times_error(oracle, wc, sc):
    rng = np.random.default_rng(COMBOS.index((wc, sc)))
    N, d, lr, T = 5, 2000, 0.1, 25
    x0 = rng.standard_normal(d).astype(np.float32)
    x = np.tile(x0, (N, 1))
    e = np.zeros(d, dtype=np.float32)
    virt = x0.astype(np.float64)
    for t in range(T):
        g = _grads(rng, N, d)
        oracle.step(g, x, e, wc, sc, lr, worker_k=40, server_k=60, rng=(17, t))
        virt = virt - np.float64(np.float32(lr)) * g.astype(np.float64).mean(axis=0)
        lhs = x.astype(np.float64).mean(axis=0) - virt
        rhs = np.float64(np.float32(lr)) * e.astype(np.float64)
        scale = max(np.abs(x).max(), np.abs(e).max(), 1.0)
        assert np.abs(lhs - rhs).max() <= (t + 1) * 4 * 2.0 ** -23 * scale


@pytest.mark.parametrize("wc", ["sign", "topk"])
def test_lemma6_worker_drift_identity(oracle, wc):
    # mean_i x_t^i - x_t^i = eta * sum_tau [ (g_i - C(g_i)) - mean_j (g_j - C(g_j)) ]
    rng = np.random.default_rng(21)
    N, d, lr, T, k = 4, 1500, 0.2, 12, 30
    x = np.zeros((N, d), dtype=np.float32)
    e = np.zeros(d, dtype=np.float32)
    acc = np.zeros((N, d), dtype=np.float64)
    for _ in range(T):
        g = _grads(rng, N, d)
        oracle.step(g, x, e, wc, "sign", lr, worker_k=k)
        delta = np.stack([g[i].astype(np.float64) - _np_compress(wc, g[i], k) for i in range(N)])
        acc += delta - delta.mean(axis=0, keepdims=True)
    x64 = x.astype(np.float64)
    lhs = x64.mean(axis=0, keepdims=True) - x64
    rhs = np.float64(np.float32(lr)) * acc
    assert np.abs(lhs - rhs).max() <= T * 8 * 2.0 ** -23 * max(1.0, np.abs(x).max())


def test_server_identity_keeps_error_zero_and_worker_identity_keeps_models_equal(oracle):
    rng = np.random.default_rng(33)
    N, d, lr = 4, 1000, 0.1
    x = np.zeros((N, d), dtype=np.float32)
    e = np.zeros(d, dtype=np.float32)
    for _ in range(5):
        oracle.step(_grads(rng, N, d), x, e, "topk", "identity", lr, worker_k=25)
        assert not e.any()
    assert not np.array_equal(x[0], x[1])     # local models do diverge under worker compression
    x[:] = 0
    for _ in range(5):
        oracle.step(_grads(rng, N, d), x, e, "identity", "sign", lr)
        assert all(np.array_equal(x[0], x[i]) for i in range(1, N))
    assert e.any()


def test_lemma6_worker_drift_identity_random_k(oracle):
    # the same identity with Definition 3's operator; the kept set of (seed, draw, worker) is re-derived
    # from the priorities alone
    rng = np.random.default_rng(22)
    N, d, lr, T, k, seed = 4, 900, 0.2, 10, 45, 5
    x = np.zeros((N, d), dtype=np.float32)
    e = np.zeros(d, dtype=np.float32)
    acc = np.zeros((N, d), dtype=np.float64)
    for t in range(T):
        g = _grads(rng, N, d)
        oracle.step(g, x, e, "randk", "randk", lr, worker_k=k, server_k=2 * k, rng=(seed, t))
        delta = np.empty((N, d))
        for i in range(N):
            pr = oracle.randk_priorities(d, (seed, t, i))
            keep = np.lexsort((np.arange(d), -pr.astype(np.int64)))[:k]
            delta[i] = g[i].astype(np.float64)
            delta[i, keep] = 0.0
        acc += delta - delta.mean(axis=0, keepdims=True)
    x64 = x.astype(np.float64)
    lhs = x64.mean(axis=0, keepdims=True) - x64
    rhs = np.float64(np.float32(lr)) * acc
    assert np.abs(lhs - rhs).max() <= T * 8 * 2.0 ** -23 * max(1.0, np.abs(x).max())


def test_random_k_step_composes_with_worker_rows_and_server_row_N(oracle):
    rng = np.random.default_rng(4)
    N, d, lr, k, seed, draw = 3, 500, 0.3, 25, 99, 12
    g = _grads(rng, N, d)
    x = rng.standard_normal((N, d)).astype(np.float32)
    e = (0.01 * rng.standard_normal(d)).astype(np.float32)
    x2, e2 = x.copy(), e.copy()
    tr = oracle.step(g, x, e, "randk", "randk", lr, worker_k=k, server_k=3 * k, trace=True, rng=(seed, draw))
    P = np.stack([oracle.compress("randk", g[i], k, rng=(seed, draw, i))[0] for i in range(N)])
    v = oracle.server_average(P, e2)
    p, _ = oracle.compress("randk", v, 3 * k, rng=(seed, draw, N))
    e2 = oracle.error_update(v, p)
    for i in range(N):
        oracle.worker_update(g[i], P[i], p, lr, x2[i])
    assert np.array_equal(tr.P, P) and np.array_equal(tr.v, v) and np.array_equal(tr.p, p)
    assert np.array_equal(e, e2) and np.array_equal(x, x2)
    assert len({tuple(np.flatnonzero(P[i])) for i in range(N)}) == N   # the workers draw different sets


def test_step_pieces_compose_to_the_whole_step(oracle):
    # the phase functions exposed for sampled full-size checks are the ones the step uses
    rng = np.random.default_rng(2)
    N, d, lr, k = 3, 700, 0.3, 20
    g = _grads(rng, N, d)
    x = rng.standard_normal((N, d)).astype(np.float32)
    e = (0.01 * rng.standard_normal(d)).astype(np.float32)
    x2, e2 = x.copy(), e.copy()
    tr = oracle.step(g, x, e, "topk", "sign", lr, worker_k=k, trace=True)
    P = np.stack([oracle.compress("topk", g[i], k)[0] for i in range(N)])
    v = oracle.server_average(P, e2)
    p, sd = oracle.compress("sign", v)
    e2 = oracle.error_update(v, p)
    for i in range(N):
        oracle.worker_update(g[i], P[i], p, lr, x2[i])
    assert np.array_equal(tr.v, v) and np.array_equal(tr.p, p) and sd.scale == tr.server.scale
    assert np.array_equal(e, e2) and np.array_equal(x, x2)


def test_server_average_adds_in_worker_order_then_one_fma(oracle):
    # (a + b) + c differs from a + (b + c) in fp32 for these values; worker order is the reading taken
    P = np.array([[1.0], [2.0 ** -24], [2.0 ** -24]], dtype=np.float32)
    e = np.zeros(1, dtype=np.float32)
    v = oracle.server_average(P, e)
    assert v[0] == np.float32(np.float32(1.0) * np.float32(1.0 / 3.0))
    P = P[::-1].copy()
    v = oracle.server_average(P, e)
    assert v[0] == np.float32(np.float32(1.0 + 2.0 ** -23) * np.float32(1.0 / 3.0))


def test_server_average_multiplies_and_adds_the_global_error_with_one_rounding(oracle):
    # acc = 3, 1/N = fl32(1/3) = 11184811 * 2^-25: the exact product is 1 + 2^-25, which a separate
    # multiply would round to 1 before the error is added; one fused operation keeps it
    P = np.ones((3, 1), dtype=np.float32)
    v = oracle.server_average(P, np.array([-1.0], dtype=np.float32))
    assert v[0] == np.float32(2.0 ** -25)
    # and the same through a whole step with the identity operator on both sides: x = -lr * v
    g = np.ones((3, 1), dtype=np.float32)
    x = np.zeros((3, 1), dtype=np.float32)
    e = np.array([-1.0], dtype=np.float32)
    oracle.step(g, x, e, "identity", "identity", 1.0)
    assert np.all(x == np.float32(-(2.0 ** -25))) and e[0] == 0.0


def test_worker_update_is_one_fused_multiply_add(oracle):
    # lr = fl32(0.1) = 13421773 * 2^-27 and u = 3: the exact product 40265319 * 2^-27 is not an fp32
    # number (a separate multiply would round it to fl32(0.3) = 40265320 * 2^-27); subtracting it from
    # x = fl32(0.3) with a single rounding leaves exactly 2^-27
    lr = np.float32(0.1)
    x = np.array([0.3], dtype=np.float32)
    zero = np.zeros(1, dtype=np.float32)
    oracle.worker_update(zero, zero, np.array([3.0], dtype=np.float32), float(lr), x)
    assert x[0] == np.float32(2.0 ** -27)


@pytest.mark.parametrize("wc,sc", [("sign", "sign"), ("topk", "topk"), ("topk", "sign"), ("randk", "randk"),
                                   ("identity", "identity")])
def test_the_all_cores_build_of_the_oracle_gives_the_same_bits(oracle, wc, sc):
    """The -fopenmp build (workers of a step on several threads; timed by the bench as the "all host cores"
    figure) must leave exactly the state the plain build leaves."""
    rng = np.random.default_rng(17)
    N, d, k = 7, 5003, 211
    x1 = rng.standard_normal((N, d)).astype(np.float32)
    e1 = (rng.standard_normal(d) * 0.1).astype(np.float32)
    x2, e2 = x1.copy(), e1.copy()
    for t in range(3):
        g = rng.standard_normal((N, d)).astype(np.float32)
        oracle.step(g, x1, e1, wc, sc, 0.05, k, k, rng=(9, t))
        threads = oracle.step_all_cores(g, x2, e2, wc, sc, 0.05, k, k, rng=(9, t))
        assert threads >= 1
        assert np.array_equal(x1.view(np.uint32), x2.view(np.uint32))
        assert np.array_equal(e1.view(np.uint32), e2.view(np.uint32))
