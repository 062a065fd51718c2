"""Pins for the oracle's Blockwise-SignSGD operator (Definition 5) and the step that uses it."""
import math

import numpy as np
import pytest


def _blocks(rng, d, B):
    cuts = np.sort(rng.choice(np.arange(1, d), size=B - 1, replace=False)) if B > 1 else np.array([], dtype=np.int64)
    return np.concatenate([[0], cuts, [d]]).astype(np.int64)


def test_hand_example(oracle):
    # blocks [3,-1,0,-1] | [2,-2] | [0.5]: scales 5/4, 4/2, 0.5/1; zero counts as positive
    v = np.array([3, -1, 0, -1, 2, -2, 0.5], dtype=np.float32)
    p, scales = oracle.compress_blocksign(v, [0, 4, 6, 7])
    assert scales.tolist() == [1.25, 2.0, 0.5]
    assert p.tolist() == [1.25, -1.25, 1.25, -1.25, 2.0, -2.0, 0.5]


def test_one_block_reduces_to_scaled_sign(oracle):
    # the paper: Blockwise-SignSGD reduces to SignSGD when the number of blocks equals 1
    rng = np.random.default_rng(0)
    v = rng.standard_normal(5000).astype(np.float32)
    p, scales = oracle.compress_blocksign(v, [0, v.size])
    q, desc = oracle.compress("sign", v)
    assert np.array_equal(p, q) and scales[0] == np.float32(desc.scale)


def test_blocks_of_one_element_keep_the_vector(oracle):
    rng = np.random.default_rng(1)
    v = rng.standard_normal(64).astype(np.float32)
    v[5] = 0.0
    p, scales = oracle.compress_blocksign(v, np.arange(65))
    assert np.array_equal(p, v) and np.array_equal(scales, np.abs(v))


@pytest.mark.parametrize("seed", range(6))
def test_each_block_is_definition_4_on_its_own_slice(oracle, seed):
    rng = np.random.default_rng(seed)
    d = int(rng.integers(200, 20000))
    B = int(rng.integers(2, 20))
    off = _blocks(rng, d, B)
    v = (rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 1, size=d)).astype(np.float32)
    p, scales = oracle.compress_blocksign(v, off)
    v64 = v.astype(np.float64)
    for b in range(B):
        lo, hi = off[b], off[b + 1]
        l1 = math.fsum(np.abs(v64[lo:hi]))
        assert scales[b] == np.float32(l1 / (hi - lo))                  # exact mean magnitude of the block
        assert np.all(np.abs(p[lo:hi]) == scales[b])                     # block L1 norm preserved: d_b * s_b
        assert np.array_equal(p[lo:hi] < 0, v[lo:hi] < 0)
        err = math.fsum((v64[lo:hi] - p[lo:hi].astype(np.float64)) ** 2)
        closed = math.fsum(v64[lo:hi] ** 2) - l1 * l1 / (hi - lo)        # ||v_b||^2 - ||v_b||_1^2 / d_b
        assert err == pytest.approx(closed, rel=1e-5, abs=1e-12)
    # finer blocks never increase the compression error (each block's scale is its own least-squares fit)
    q, _ = oracle.compress("sign", v)
    assert np.sum((v64 - p) ** 2) <= np.sum((v64 - q) ** 2) * (1 + 1e-9)


def test_bad_block_tables_are_rejected(oracle):
    v = np.ones(10, dtype=np.float32)
    for off in ([0, 5, 5, 10], [1, 10], [0, 9], [0, 7, 3, 10]):
        with pytest.raises(ValueError):
            oracle.compress_blocksign(v, off)


def test_step_with_blockwise_operator_both_sides(oracle):
    # the step composes the operator exactly as it composes Definition 4; with one block it IS that step
    rng = np.random.default_rng(5)
    N, d, lr = 3, 900, 0.2
    g = rng.standard_normal((N, d)).astype(np.float32)
    x = rng.standard_normal((N, d)).astype(np.float32)
    e = (0.1 * rng.standard_normal(d)).astype(np.float32)
    x1, e1 = x.copy(), e.copy()
    oracle.step(g, x1, e1, "sign", "sign", lr)
    x2, e2 = x.copy(), e.copy()
    oracle.step_blocks(g, x2, e2, "blocksign", "blocksign", lr, [0, d])
    assert np.array_equal(x1, x2) and np.array_equal(e1, e2)
    # several blocks: re-assemble the step from the operator and the phase functions
    off = [0, 100, 450, 451, 900]
    x3, e3 = x.copy(), e.copy()
    tr = oracle.step_blocks(g, x3, e3, "blocksign", "blocksign", lr, off)
    P = np.stack([oracle.compress_blocksign(g[i], off)[0] for i in range(N)])
    v = oracle.server_average(P, e)
    p, ss = oracle.compress_blocksign(v, off)
    e4 = oracle.error_update(v, p)
    x4 = x.copy()
    for i in range(N):
        oracle.worker_update(g[i], P[i], p, lr, x4[i])
    assert np.array_equal(x3, x4) and np.array_equal(e3, e4) and np.array_equal(tr.server_scales, ss)


@pytest.mark.parametrize("wc,sc", [("blocksign", "blocksign"), ("blocksign", "sign"), ("topk", "blocksign")])
def test_lemma3_with_blockwise_operator(oracle, wc, sc):
    rng = np.random.default_rng(8)
    N, d, lr, T = 4, 1200, 0.1, 15
    off = [0, 64, 300, 301, 1000, 1200]
    x0 = rng.standard_normal(d).astype(np.float32)
    x = np.tile(x0, (N, 1))
    e = np.zeros(d, dtype=np.float32)
    virt = x0.astype(np.float64)
    eta = np.float64(np.float32(lr))
    for t in range(T):
        g = (rng.standard_normal((N, d)) * 10.0 ** rng.uniform(-2, 0)).astype(np.float32)
        oracle.step_blocks(g, x, e, wc, sc, lr, off, worker_k=25, server_k=40)
        virt = virt - eta * g.astype(np.float64).mean(axis=0)
        lhs = x.astype(np.float64).mean(axis=0) - virt
        scale = max(np.abs(x).max(), np.abs(e).max(), 1.0)
        assert np.abs(lhs - eta * e).max() <= (t + 1) * 4 * 2.0 ** -23 * scale
