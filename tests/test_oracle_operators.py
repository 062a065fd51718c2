"""Pins for the oracle's compression operators (Definitions 1, 2 and 4).

None of these re-types the oracle's own formula: each check is a brute force
on tiny inputs, a closed form, an invariant the definition implies, or a
special case with a textbook answer.
"""
import math

import numpy as np
import pytest


def _tricky(rng, d):
    """Small vectors with ties, zeros, negative zeros and mixed signs."""
    v = rng.choice(np.array([0.0, -0.0, 0.5, -0.5, 1.0, -1.0, 2.0, 3.25, -3.25], dtype=np.float32), size=d)
    m = rng.random(d) < 0.4
    v[m] = rng.standard_normal(m.sum()).astype(np.float32)
    return v.astype(np.float32)


def _brute_topk(v, k):
    """Definition 2 with ties to the lower index: a stable sort on |v|."""
    order = sorted(range(len(v)), key=lambda j: (-abs(float(v[j])), j))
    return sorted(order[:k])


@pytest.mark.parametrize("seed", range(40))
def test_topk_matches_brute_force_on_tiny_inputs(oracle, seed):
    rng = np.random.default_rng(seed)
    d = int(rng.integers(1, 65))
    k = int(rng.integers(1, d + 1))
    v = _tricky(rng, d)
    p, desc = oracle.compress("topk", v, k)
    kept = _brute_topk(v, k)
    expect = np.zeros(d, dtype=np.float32)
    expect[kept] = v[kept]
    assert np.array_equal(p.view(np.uint32), expect.view(np.uint32))
    # descriptor: k-th kept entry in the (|v| desc, index asc) order
    kth = sorted(kept, key=lambda j: (-abs(float(v[j])), j))[-1]
    assert desc.cutoff == kth
    assert desc.tau_key == (int(v[kth:kth + 1].view(np.uint32)[0]) & 0x7FFFFFFF)
    assert desc.count_above == sum(abs(float(v[j])) > abs(float(v[kth])) for j in range(d))


def test_topk_descriptor_defines_the_kept_set(oracle):
    rng = np.random.default_rng(7)
    v = _tricky(rng, 5000)
    k = 1234
    p, desc = oracle.compress("topk", v, k)
    key = v.view(np.uint32) & np.uint32(0x7FFFFFFF)
    idx = np.arange(v.size)
    sel = (key > desc.tau_key) | ((key == desc.tau_key) & (idx <= desc.cutoff))
    assert sel.sum() == k
    assert np.array_equal(p.view(np.uint32), np.where(sel, v, np.float32(0)).view(np.uint32))
    # everything kept is at least as large as everything dropped
    assert np.abs(v[sel]).min() >= np.abs(v[~sel]).max()


def test_topk_keeps_exactly_k_even_when_zeros_must_be_admitted(oracle):
    v = np.zeros(32, dtype=np.float32)
    v[[3, 17]] = [1.5, -2.0]
    p, desc = oracle.compress("topk", v, 5)
    assert desc.tau_key == 0 and desc.count_above == 2
    assert desc.cutoff == 2  # zeros at indices 0,1,2 are admitted, lower index first
    assert np.array_equal(p, v)


def test_topk_with_k_equal_d_is_identity(oracle):
    rng = np.random.default_rng(3)
    v = _tricky(rng, 777)
    p, _ = oracle.compress("topk", v, v.size)
    q, _ = oracle.compress("identity", v)
    assert np.array_equal(p.view(np.uint32), v.view(np.uint32))
    assert np.array_equal(q.view(np.uint32), v.view(np.uint32))


def test_topk_all_equal_magnitudes_takes_lowest_indices(oracle):
    v = np.full(100, 0.75, dtype=np.float32)
    v[::2] *= -1
    p, desc = oracle.compress("topk", v, 10)
    assert np.array_equal(np.nonzero(p)[0], np.arange(10))
    assert desc.cutoff == 9 and desc.count_above == 0


@pytest.mark.parametrize("frac", [0.001, 0.01, 0.1, 0.5])
def test_topk_is_a_contraction_with_delta_at_least_k_over_d(oracle, frac):
    # Definition 1 with delta = k/d (the bound the paper states for top-k)
    rng = np.random.default_rng(11)
    d = 20000
    v = (rng.standard_normal(d) * np.exp(rng.standard_normal(d))).astype(np.float32)
    k = max(1, int(frac * d))
    p, _ = oracle.compress("topk", v, k)
    lhs = np.sum((v.astype(np.float64) - p) ** 2)
    rhs = (1 - k / d) * np.sum(v.astype(np.float64) ** 2)
    assert lhs <= rhs * (1 + 1e-12)


def test_topk_rejects_bad_k(oracle):
    v = np.ones(8, dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.compress("topk", v, 0)
    with pytest.raises(ValueError):
        oracle.compress("topk", v, 9)


def test_sign_hand_example(oracle):
    # ||v||_1 = 5, d = 4 -> scale 1.25; zero counts as positive
    v = np.array([3.0, -1.0, 0.0, -1.0], dtype=np.float32)
    p, desc = oracle.compress("sign", v)
    assert desc.scale == 1.25 and desc.l1 == 5.0
    assert np.array_equal(p, np.array([1.25, -1.25, 1.25, -1.25], dtype=np.float32))


def test_sign_of_both_zeros_is_plus_one(oracle):
    v = np.array([0.0, -0.0, -2.0, 2.0], dtype=np.float32)
    p, desc = oracle.compress("sign", v)
    assert desc.scale == 1.0
    assert np.array_equal(p, np.array([1.0, 1.0, -1.0, 1.0], dtype=np.float32))


@pytest.mark.parametrize("seed", range(5))
def test_sign_preserves_l1_norm_and_matches_closed_form_error(oracle, seed):
    rng = np.random.default_rng(seed)
    d = int(rng.integers(1000, 200000))
    v = (rng.standard_normal(d) * 10.0 ** rng.uniform(-4, 1)).astype(np.float32)
    p, desc = oracle.compress("sign", v)
    v64 = v.astype(np.float64)
    l1 = math.fsum(np.abs(v64))          # exact sum, independent of the oracle's accumulator
    l2sq = math.fsum(v64 * v64)
    # every output has magnitude `scale`, so ||C(v)||_1 = d * scale exactly
    assert np.all(np.abs(p) == np.float32(desc.scale))
    assert np.array_equal(p < 0, v < 0)
    # scale is the fp32 rounding of the exact mean magnitude
    assert desc.scale == float(np.float32(l1 / d))
    assert abs(desc.l1 - l1) <= 2.0 ** -52 * l1
    # ||v - C(v)||^2 = ||v||^2 - ||v||_1^2 / d  when scale is exact
    err = math.fsum((v64 - p.astype(np.float64)) ** 2)
    closed = l2sq - l1 * l1 / d
    assert err == pytest.approx(closed, rel=1e-6)
    # and therefore it is a contraction (Definition 1) with delta = ||v||_1^2 / (d ||v||^2)
    assert err <= l2sq


def test_sign_with_d_equal_one_is_identity_on_nonzero_input(oracle):
    for val in (2.5, -0.375):
        v = np.array([val], dtype=np.float32)
        p, desc = oracle.compress("sign", v)
        assert p[0] == v[0] and desc.scale == abs(val)


def test_sign_scale_of_standard_normal_input(oracle):
    rng = np.random.default_rng(5)
    d = 1 << 20
    v = rng.standard_normal(d).astype(np.float32)
    _, desc = oracle.compress("sign", v, want_p=False)
    assert abs(desc.scale - math.sqrt(2 / math.pi)) < 5 / math.sqrt(d)


def test_sign_accumulates_beyond_fp32_and_fp64_naive_precision(oracle):
    # one huge entry followed by many tiny ones: a naive fp32 sum loses all of them,
    # and the answer is known in closed form
    d = 1 << 16
    v = np.full(d, 2.0 ** -10, dtype=np.float32)
    v[0] = 2.0 ** 20
    _, desc = oracle.compress("sign", v, want_p=False)
    assert desc.l1 == 2.0 ** 20 + (d - 1) * 2.0 ** -10
    assert desc.scale == float(np.float32(desc.l1 / d))


@pytest.mark.parametrize("comp,k", [("sign", 0), ("topk", 50), ("identity", 0)])
def test_compressed_value_plus_error_reconstructs_input(oracle, comp, k):
    rng = np.random.default_rng(9)
    v = _tricky(rng, 400)
    p, _ = oracle.compress(comp, v, k)
    e = oracle.error_update(v, p)
    back = p.astype(np.float64) + e.astype(np.float64)
    if comp == "sign":
        ulp = np.spacing(np.maximum(np.abs(v), np.abs(p)).astype(np.float32))
        assert np.all(np.abs(back - v) <= ulp)
    else:
        assert np.array_equal(back.astype(np.float32), v + np.float32(0))
