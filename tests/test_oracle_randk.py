"""Pins of the oracle's random-k operator (Definition 3) and of the generator behind its draws.

What the paper fixes: exactly k coordinates survive unchanged and the rest become zero; the kept
set S is uniform over the k-element subsets of [d] (so every index is kept with probability k/d,
every pair with k(k-1)/(d(d-1)), every subset equally often); E[C(x)] = (k/d) x (Assumption 4,
stated for random-k); E||x - C(x)||^2 = (1 - k/d) ||x||^2 (the contraction of Definition 1 with
delta = k/d, stated right after Definition 5).  The statistical pins use fixed seeds and bounds at
about 5 standard deviations, so they are deterministic tests of this generator.
"""
import itertools
import math

import numpy as np
import pytest

import oracle


def _mask(d, k, rng):
    v = np.arange(1, d + 1, dtype=np.float32)
    p, _ = oracle.compress("randk", v, k, rng=rng)
    return p != 0


@pytest.mark.parametrize("d,k", [(1, 1), (2, 1), (7, 3), (64, 64), (1000, 10), (4099, 2050)])
def test_keeps_exactly_k_entries_unchanged(d, k):
    g = np.random.default_rng(d * 31 + k)
    v = (g.standard_normal(d).astype(np.float32) + np.float32(3.0))   # no zeros
    for draw in range(5):
        p, desc = oracle.compress("randk", v, k, rng=(11, draw, 2))
        kept = p != 0
        assert kept.sum() == k
        assert np.array_equal(p[kept].view(np.uint32), v[kept].view(np.uint32))
        assert np.all(p[~kept].view(np.uint32) == 0)                  # +0, not -0
        if k == d:
            assert np.array_equal(p.view(np.uint32), v.view(np.uint32))


def test_the_draw_does_not_look_at_the_data():
    d, k = 5000, 137
    a = np.random.default_rng(0).standard_normal(d).astype(np.float32) + np.float32(5)
    b = np.random.default_rng(1).standard_cauchy(d).astype(np.float32) + np.float32(1e3)
    pa, da = oracle.compress("randk", a, k, rng=(3, 9, 1))
    pb, db = oracle.compress("randk", b, k, rng=(3, 9, 1))
    assert np.array_equal(pa != 0, pb != 0)
    assert (da.tau_key, da.cutoff) == (db.tau_key, db.cutoff)


def test_seed_draw_and_row_each_change_the_set():
    d, k = 4096, 64
    base = _mask(d, k, (5, 5, 5))
    for rng in [(6, 5, 5), (5, 6, 5), (5, 5, 6), (5, 5, 4)]:
        other = _mask(d, k, rng)
        # two independent 64-subsets of 4096 share about one element
        assert (base & other).sum() <= 8


def test_descriptor_defines_the_set_and_matches_a_sort_of_the_priorities():
    for d, k, rng in [(50, 7, (1, 2, 3)), (3000, 300, (9, 0, 0)), (70001, 123, (2, 2, 16))]:
        pr = oracle.randk_priorities(d, rng)
        order = np.lexsort((np.arange(d), -pr.astype(np.int64)))      # priority descending, index ascending
        want = np.zeros(d, dtype=bool)
        want[order[:k]] = True
        v = np.arange(1, d + 1, dtype=np.float32)
        p, desc = oracle.compress("randk", v, k, rng=rng)
        assert np.array_equal(p != 0, want)
        idx = np.arange(d)
        assert np.array_equal(want, (pr > desc.tau_key) | ((pr == desc.tau_key) & (idx <= desc.cutoff)))
        assert desc.tau_key == pr[order[k - 1]] and desc.cutoff == order[k - 1]


def test_priorities_of_distinct_indices_collide_at_most_in_pairs():
    pr = oracle.randk_priorities(1 << 20, (123, 4, 5))
    _, counts = np.unique(pr, return_counts=True)
    assert counts.max() <= 2            # a 32-bit bijection with its lowest bit dropped
    assert pr.max() < (1 << 31)
    # and they fill the 31-bit range evenly: 64 equal bins, chi-square with 63 degrees of freedom
    h = np.bincount(pr >> 25, minlength=64).astype(np.float64)
    exp = pr.size / 64
    assert ((h - exp) ** 2 / exp).sum() < 130.0


def _chi2(counts, expected):
    return float(((counts - expected) ** 2 / expected).sum())


def test_every_index_is_kept_with_probability_k_over_d():
    d, k, T = 40, 7, 20000
    counts = np.zeros(d)
    for t in range(T):
        counts += _mask(d, k, (42, t, 0))
    # not independent multinomial cells (exactly k per draw), which only lowers the statistic
    assert _chi2(counts, T * k / d) < 85.0          # 39 degrees of freedom: 99.99 % point is 79


def test_every_pair_is_kept_equally_often():
    d, k, T = 12, 4, 30000
    pair = np.zeros((d, d))
    for t in range(T):
        m = _mask(d, k, (7, t, 3)).astype(np.float64)
        pair += np.outer(m, m)
    iu = np.triu_indices(d, 1)
    exp = T * k * (k - 1) / (d * (d - 1))
    assert _chi2(pair[iu], exp) < 125.0              # 65 degrees of freedom: 99.99 % point is 117


def test_every_subset_is_drawn_equally_often():
    d, k, T = 6, 3, 40000
    subsets = {s: 0 for s in itertools.combinations(range(d), k)}
    for t in range(T):
        subsets[tuple(np.flatnonzero(_mask(d, k, (1, t, 1))))] += 1
    counts = np.array(list(subsets.values()), dtype=np.float64)
    assert len(subsets) == math.comb(d, k)
    assert _chi2(counts, T / len(subsets)) < 52.0    # 19 degrees of freedom: 99.99 % point is 50


def test_rows_of_one_draw_and_consecutive_draws_are_independent():
    d, k, T = 30, 6, 20000
    both_rows = np.zeros(d)
    both_draws = np.zeros(d)
    for t in range(T):
        a, b, c = _mask(d, k, (9, t, 0)), _mask(d, k, (9, t, 1)), _mask(d, k, (9, t + 1, 0))
        both_rows += a & b
        both_draws += a & c
    exp = T * (k / d) ** 2
    sd = math.sqrt(exp)
    assert np.all(np.abs(both_rows - exp) < 5 * sd)
    assert np.all(np.abs(both_draws - exp) < 5 * sd)


def test_expectation_and_contraction_of_definition_1_and_assumption_4():
    d, k, T = 200, 30, 6000
    v = np.random.default_rng(3).standard_normal(d).astype(np.float32)
    mean = np.zeros(d)
    err = 0.0
    for t in range(T):
        p, _ = oracle.compress("randk", v, k, rng=(77, t, 4))
        mean += p
        err += float(np.sum((v.astype(np.float64) - p) ** 2))
    mean /= T
    err /= T
    n2 = float(np.sum(v.astype(np.float64) ** 2))
    delta = k / d
    # E[C(x)]_j = delta x_j with standard deviation |x_j| sqrt(delta (1 - delta) / T)
    tol = 5 * np.abs(v) * math.sqrt(delta * (1 - delta) / T) + 1e-9
    assert np.all(np.abs(mean - delta * v) <= tol)
    # E||x - C(x)||^2 = (1 - delta)||x||^2; the sample mean's spread is below ||x||^2 / sqrt(T)
    assert abs(err - (1 - delta) * n2) < 5 * n2 / math.sqrt(T)


def test_threshold_sits_where_a_uniform_priority_puts_it():
    d, k = 1 << 20, 10485
    _, desc = oracle.compress("randk", np.ones(d, dtype=np.float32), k, want_p=False, rng=(2024, 0, 0))
    centre = (1 << 31) * (1 - k / d)
    sigma = (1 << 31) * math.sqrt(k * (d - k) / d) / d
    assert abs(desc.tau_key - centre) < 6 * sigma


def test_wire_form_round_trip():
    d, k, rng = 3001, 77, (5, 6, 7)
    v = np.random.default_rng(8).standard_normal(d).astype(np.float32)
    idx, val = oracle.pack_randk(v, k, rng)
    assert np.all(np.diff(idx.astype(np.int64)) > 0) and idx.size == k
    p, _ = oracle.compress("randk", v, k, rng=rng)
    assert np.array_equal(oracle.unpack_topk(idx, val, d).view(np.uint32), p.view(np.uint32))


def test_bad_k_is_rejected():
    v = np.ones(8, dtype=np.float32)
    for k in (0, 9, -1):
        with pytest.raises(ValueError):
            oracle.compress("randk", v, k)


def test_lemma_1_bound_on_the_global_error_with_random_k():
    # Lemma 1 (needs Assumption 4, which random-k satisfies with delta = k/d):
    #   E||e_t||^2 <= 4 (1 - delta) (2 (2 - delta) + delta^2 (N - 1)) M^2 / (delta^2 N),
    # M^2 a bound on ||g_i||^2.  Checked at every step of a long chain, on the running mean over steps
    # (the expectation is over the draws) and, with the bound's slack, on every single step.
    N, d, k, T, lr = 4, 400, 100, 300, 0.05
    delta = k / d
    g_rng = np.random.default_rng(6)
    x = np.zeros((N, d), dtype=np.float32)
    e = np.zeros(d, dtype=np.float32)
    m2, norms = 0.0, []
    for t in range(T):
        g = g_rng.standard_normal((N, d)).astype(np.float32)
        m2 = max(m2, float((g.astype(np.float64) ** 2).sum(axis=1).max()))
        oracle.step(g, x, e, "randk", "randk", lr, worker_k=k, server_k=k, rng=(31, t))
        norms.append(float((e.astype(np.float64) ** 2).sum()))
    bound = 4 * (1 - delta) * (2 * (2 - delta) + delta ** 2 * (N - 1)) * m2 / (delta ** 2 * N)
    assert max(norms) <= bound
    assert np.mean(norms[T // 2:]) <= bound
    assert np.mean(norms[T // 2:]) > 0.0          # the error is really carried from step to step


def test_generator_is_the_one_the_public_header_states():
    """include/liec.h states the generator in words and formulas; this re-states those formulas with
    Python integers (a cross-language check of wrap-around and shifts, not a pin of the design)."""
    M64, M32 = (1 << 64) - 1, (1 << 32) - 1

    def mix(z):
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
        return z ^ (z >> 31)

    def priority(seed, draw, row, j):
        G = 0x9E3779B97F4A7C15
        s = mix((mix((mix((seed + G) & M64) + draw + G) & M64) + row + G) & M64)
        h = (j ^ (s & M32)) & M32
        h ^= h >> 16
        h = (h * 0x85EBCA6B) & M32
        h ^= h >> 13
        h = (h + (s >> 32)) & M32
        h = (h * 0xC2B2AE35) & M32
        h ^= h >> 16
        return h >> 1

    rng = np.random.default_rng(12)
    for _ in range(40):
        seed, draw = int(rng.integers(0, 1 << 63)) * 2 + 1, int(rng.integers(0, 1 << 62))
        row, d = int(rng.integers(0, 70)), int(rng.integers(1, 300))
        got = oracle.randk_priorities(d, (seed, draw, row))
        assert got.tolist() == [priority(seed, draw, row, j) for j in range(d)]
    # the largest values of every argument
    got = oracle.randk_priorities(3, (M64, M64, M32))
    assert got.tolist() == [priority(M64, M64, M32, j) for j in range(3)]
