"""Seeded sweeps and edge cases on the GPU: random shapes over all operator pairs, jumps of the gradient
scale, subnormal and huge magnitudes, the largest sizes the library accepts, error-norm telemetry.
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


ALL_OPS = ["identity", "sign", "topk", "randk", "blocksign"]


@pytest.mark.parametrize("case", range(48))
def test_random_shapes_and_operator_pairs(case):
    """Seeded sweep over worker counts (odd, above the 8-row batches of the aggregation, not powers of
    two), dimensions (log-uniform, ragged against every tile size), k and all 25 operator pairs."""
    import oracle
    from paper_2402_11857_amd import LiecContext

    rng = np.random.default_rng(1000 + case)
    wc, sc = ALL_OPS[case % 5], ALL_OPS[(case // 5 + case) % 5]
    N = int(rng.choice([1, 2, 3, 5, 7, 9, 12, 17, 24, 33, 70]))
    d = int(np.exp(rng.uniform(np.log(1), np.log(400_000 // max(1, N // 8)))))
    wk = int(rng.integers(1, d + 1)) if rng.random() < 0.3 else max(1, d // int(rng.choice([10, 100, 1000])))
    sk = int(rng.integers(1, d + 1)) if rng.random() < 0.3 else max(1, d // int(rng.choice([10, 100, 1000])))
    wk = wk if wc in ("topk", "randk") else 0
    sk = sk if sc in ("topk", "randk") else 0
    lr = float(rng.choice([0.5, 0.1, 0.01]))
    nb = int(rng.integers(1, min(d, 40) + 1))
    off = sorted({0, d, *map(int, rng.integers(0, d + 1, size=nb - 1))})
    say(f"case sweep {case}: N={N} d={d} {wc}/{sc} k={wk}/{sk} lr={lr} blocks={len(off) - 1}")
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp=wc, server_comp=sc, worker_k=wk, server_k=sk, lr=lr)
    src = workloads.GradientSource(w, seed=case, device=DEV)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    with LiecContext(N, d, wc, sc, wk, sk, lr) as ctx:
        ctx.set_random(case, 5)
        if wc == "topk":
            ctx.set_group_bitmap((case // 5) & 1)    # both forms of the candidate bitmap
            ctx.set_gather_batching((case // 10) & 1)   # both ways the aggregation fetches the candidates
        if "blocksign" in (wc, sc):
            ctx.set_blocks(off)
        for t in range(3):
            g = src.grads(t)
            if case % 3 == 0:
                g = workloads.inject_ties(g, seed=t, frac_zero=0.2, frac_dup=0.3)
            ctx.step(g, x, e)
            tr = oracle.step_blocks(g.cpu().numpy(), xo, eo, wc, sc, lr, off, wk, sk, rng=(case, 5 + t))
            assert H.bit_equal(e.cpu().numpy(), eo), f"step {t}: server error"
            assert H.bit_equal(x.cpu().numpy(), xo), f"step {t}: models"
        assert ctx.info().nonfinite == 0


def _random_chain(case, degenerate):
    """One seeded chain of 4-8 iterations of Algorithm 1 as a whole (liec_iteration; period 0, 3 or 4) on a random
    shape up to 3 million columns, random k (also 1, d - 1, d) and operator pair, with the gradient scale drifting
    or jumping between iterations and ties injected; compared bit for bit after every iteration.  With
    `degenerate` the gradients are also cut to a few mantissa bits, made constant, made sparse or rounded to a
    few levels, and in half of the cases the general search runs with its single-block fallback forced."""
    import oracle
    from paper_2402_11857_amd import LiecContext

    rng = np.random.default_rng(50_000 + case)
    wc, sc = ALL_OPS[int(rng.integers(5))], ALL_OPS[int(rng.integers(5))]
    if rng.random() < 0.5:                       # weight the threshold searches
        wc = str(rng.choice(["topk", "randk", "topk"]))
    N = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16, 17, 31, 40]))
    d = int(np.exp(rng.uniform(np.log(1), np.log(3_000_000 // max(1, N // 4)))))
    if rng.random() < 0.3:
        d = max(1, (d // 1024) * 1024 + int(rng.choice([0, 1, 3, 4, 1020, 1023])))

    def pick_k():
        r = rng.random()
        if r < 0.2:
            return int(rng.integers(1, d + 1))
        if r < 0.3:
            return int(rng.choice([1, d, max(1, d - 1), max(1, d // 2)]))
        return max(1, d // int(rng.choice([10, 100, 200, 1000])))

    wk = pick_k() if wc in ("topk", "randk") else 0
    sk = pick_k() if sc in ("topk", "randk") else 0
    lr = float(rng.choice([0.5, 0.1, 0.01]))
    nb = int(rng.integers(1, min(d, 40) + 1))
    off = sorted({0, d, *map(int, rng.integers(0, d + 1, size=nb - 1))})
    steps = int(rng.integers(4, 9))
    period = int(rng.choice([0, 0, 3, 4]))
    drift = str(rng.choice(["none", "none", "slow", "jump"]))
    ties = rng.random() < 0.3
    kind = str(rng.choice(["quant", "const", "sparse", "levels"])) if degenerate else "none"
    wait = 0 if degenerate and rng.random() < 0.5 else None
    say(f"case chain {case}: N={N} d={d} {wc}/{sc} k={wk}/{sk} lr={lr} blocks={len(off) - 1} steps={steps} "
        f"period={period} drift={drift} ties={ties} gradients={kind} wait={wait}")
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp=wc, server_comp=sc, worker_k=wk, server_k=sk, lr=lr)
    src = workloads.GradientSource(w, seed=case, device=DEV)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    draw, scale = 0, 1.0
    with LiecContext(N, d, wc, sc, wk, sk, lr) as ctx:
        ctx.set_random(case, 0)
        if wait is not None:
            ctx.set_search_wait(wait)
        if wc == "topk":
            ctx.set_group_bitmap(case & 1)           # both forms of the candidate bitmap
            ctx.set_gather_batching((case >> 1) & 1)    # both ways the aggregation fetches the candidates
        if "blocksign" in (wc, sc):
            ctx.set_blocks(off)
        for t in range(steps):
            g = src.grads(t)
            if drift == "slow":
                scale *= float(rng.choice([0.9, 1.05, 1.2]))
            elif drift == "jump" and rng.random() < 0.4:
                scale *= float(rng.choice([1e-3, 30.0, 1e3, 0.2]))
            if scale != 1.0:
                g = g * np.float32(scale)
            if ties:
                g = workloads.inject_ties(g, seed=t, frac_zero=float(rng.choice([0.0, 0.2, 0.9])),
                                          frac_dup=float(rng.choice([0.0, 0.3])))
            if kind == "quant":                  # 7, 5, 2 or 0 mantissa bits
                g = (g.contiguous().view(torch.int32) & -(1 << int(rng.choice([16, 18, 21, 23])))).view(torch.float32)
            elif kind == "const" and rng.random() < 0.7:
                g = torch.full_like(g, 0.5)
                g[:, int(rng.integers(0, 3))::3] *= -1
            elif kind == "sparse":
                keep = torch.rand(g.shape, device=g.device) < float(rng.choice([1e-4, 1e-3, 1e-2]))
                g = torch.where(keep, g, torch.zeros_like(g))
            elif kind == "levels":
                g = torch.round(g * float(rng.choice([0.7, 2.0, 8.0])))
            g = g.contiguous()
            gh = g.cpu().numpy()
            ctx.iteration(t, period, g, x, e)
            if period >= 2 and (t + 1) % period == 0:
                oracle.step_sync(gh, xo, eo, lr)
            else:
                oracle.step_blocks(gh, xo, eo, wc, sc, lr, off, wk, sk, rng=(case, draw))
                draw += 1                        # only compressed iterations draw
            assert H.bit_equal(e.cpu().numpy(), eo), f"iteration {t}: server error"
            assert H.bit_equal(x.cpu().numpy(), xo), f"iteration {t}: models"
        assert ctx.info().nonfinite == 0


@pytest.mark.parametrize("case", range(40))
def test_random_chains_with_drift_ties_and_averaging_iterations(case):
    _random_chain(case, degenerate=False)


@pytest.mark.parametrize("case", range(100_000, 100_040))
def test_random_chains_on_degenerate_gradients(case):
    _random_chain(case, degenerate=True)


@pytest.mark.parametrize("wc,sc", [("topk", "topk"), ("topk", "sign")])
def test_quantised_gradients_with_thousands_of_ties_at_the_threshold(wc, sc):
    """Gradients that carry 5 mantissa bits (as after a low-precision backward pass): about 10^4 entries of a
    row share the threshold magnitude, more than the tie buffer holds.  The result must still be the oracle's,
    and the rows must not fall to the general single-block search (slow_rows stays 0)."""
    import oracle
    from paper_2402_11857_amd import LiecContext

    N, d = 3, 6_000_000
    k = d // 100
    say(f"case quantised gradients N={N} d={d} {wc}/{sc} k={k}")
    w = workloads.scaled(WL["c1_tiny_sign"], N=N, d=d, worker_comp=wc, server_comp=sc, worker_k=k, server_k=k, lr=0.1)
    src = workloads.GradientSource(w, seed=77, device=DEV)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    with LiecContext(N, d, wc, sc, k, k if sc == "topk" else 0, 0.1) as ctx:
        for t in range(3):
            g = (src.grads(t).view(torch.int32) & -(1 << 18)).view(torch.float32).contiguous()
            gh = g.cpu().numpy()
            keys = gh.view(np.uint32) & np.uint32(0x7FFFFFFF)
            for i in range(N):
                tau = np.partition(keys[i], d - k)[d - k]
                assert int((keys[i] == tau).sum()) > 4096, "the case must exceed the tie buffer"
            ctx.step(g, x, e)
            oracle.step(gh, xo, eo, wc, sc, 0.1, k, k if sc == "topk" else 0)
            say(f"  step {t} done")
            assert H.bit_equal(e.cpu().numpy(), eo), f"step {t}: server error"
            assert H.bit_equal(x.cpu().numpy(), xo), f"step {t}: models"
            info = ctx.info()
            assert info.nonfinite == 0 and info.slow_rows == 0, f"step {t}: {info.slow_rows} rows took the slow search"


@pytest.mark.parametrize("kind", ["constant", "mostly_zero", "four_levels", "one_level_rest_noise"])
@pytest.mark.parametrize("wait", [None, 0, 1, 2, 8])
def test_degenerate_rows_at_a_size_where_thread_blocks_share_a_row(kind, wait):
    """Rows whose threshold is shared by more entries than the candidate list holds take the general search,
    in which several thread blocks split a row (wait=None) or, when their bounded wait for one another runs
    out (wait=0 forces that for every block; 1, 2 and 8 polls let some blocks pass a meeting that others
    give up at), one block does it alone.  Either way the result is the oracle's and every kernel ends."""
    import oracle
    from paper_2402_11857_amd import LiecContext

    N, d, k = 3, 2_600_003, 26_000
    say(f"case degenerate rows, shared search: {kind} wait={wait}")
    gen = torch.Generator(device="cpu")
    gen.manual_seed(11)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    with LiecContext(N, d, "topk", "topk", k, k, 0.1) as ctx:
        if wait is not None:
            ctx.set_search_wait(wait)
        for t in range(2):
            if kind == "constant":
                g = torch.full((N, d), 0.5, dtype=torch.float32)
                g[:, t::3] *= -1
            elif kind == "mostly_zero":                     # fewer non-zeros than k: the threshold is zero
                g = torch.zeros((N, d), dtype=torch.float32)
                idx = torch.randint(0, d, (N, k // 3), generator=gen)
                g.scatter_(1, idx, torch.randn((N, k // 3), generator=gen))
            elif kind == "four_levels":
                g = torch.randint(-2, 2, (N, d), generator=gen).to(torch.float32)
            else:                                           # 99 % of the row on one magnitude above the noise
                g = torch.randn((N, d), generator=gen) * 1e-3
                mask = torch.rand((N, d), generator=gen) < 0.99
                g[mask] = 1.0
            g = g.to(DEV).contiguous()
            ctx.step(g, x, e)
            oracle.step(g.cpu().numpy(), xo, eo, "topk", "topk", 0.1, k, k)
            assert H.bit_equal(e.cpu().numpy(), eo), f"step {t}: server error"
            assert H.bit_equal(x.cpu().numpy(), xo), f"step {t}: models"
            assert ctx.info().slow_rows >= N, "the worker rows must have taken the general search"


def test_constant_rows_are_reported_as_slow_rows():
    """Rows whose entries all share one magnitude cannot be listed: they take the general search, and the
    context says so."""
    from paper_2402_11857_amd import LiecContext

    N, d, k = 2, 50_000, 500
    say("case slow_rows telemetry")
    g = torch.full((N, d), 0.25, dtype=torch.float32, device=DEV)
    g[:, ::2] *= -1
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    with LiecContext(N, d, "topk", "identity", k, 0, 0.1) as ctx:
        ctx.step(g, x, e)
        assert ctx.info().slow_rows == N
        g2 = torch.randn((N, d), dtype=torch.float32, device=DEV)
        ctx.step(g2, x, e)
        ctx.step(g2, x, e)
        assert ctx.info().slow_rows == 0


@pytest.mark.parametrize("wc,sc", [("topk", "topk"), ("topk", "sign")])
def test_threshold_prediction_survives_jumps_of_the_gradient_scale(wc, sc):
    """The band predicted from the last thresholds misses when the gradients' scale jumps; the step must
    then find the threshold the long way and still match the oracle (drifts are followed by the trend)."""
    say(f"case scale jumps {wc}/{sc}")
    w = workloads.scaled(WL["c2_topk_mid"], N=3, d=180_000, worker_comp=wc, server_comp=sc, worker_k=1800,
                         server_k=4000 if sc == "topk" else 0)
    scales = [1.0, 1.0, 4.0, 4.2, 4.4, 0.05, 0.05, 0.049, 1e-6, 3.0]

    def mutate(g, t):
        return g * scales[t]

    stats = {}
    assert run_chain(w, steps=len(scales), seed=17, mutate=mutate, stats=stats)
    # four jumps, three worker rows each: the context counts the predictions that failed
    assert stats["band_misses"] >= 12, f"only {stats['band_misses']} failed predictions were counted"


@pytest.mark.parametrize("wc,sc", [("sign", "sign"), ("topk", "topk"), ("identity", "identity")])
def test_subnormal_and_huge_magnitudes(wc, sc):
    """fp32 subnormals must be kept, not flushed, and magnitudes near the top of the range must not overflow
    the fp64 L1 sums: gradients span 1e-44 .. 1e37."""
    say(f"case subnormal / huge {wc}/{sc}")
    w = workloads.scaled(WL["c2_topk_mid"], N=3, d=20_000, worker_comp=wc, server_comp=sc,
                         worker_k=300 if wc == "topk" else 0, server_k=700 if sc == "topk" else 0, lr=0.5)

    def mutate(g, t):
        g = g.clone()
        g[:, 0::3] *= 1e-41          # subnormal range
        g[:, 1::3] *= 1e-38          # around the smallest normal number
        if t == 1:
            g[:, 2::3] *= 1e34       # large but finite: sums of 2e4 of them stay finite in fp32 messages too
        tiny = g[:, 0::3].abs()
        assert ((tiny > 0) & (tiny < 1.1754944e-38)).float().mean() > 0.9, "the inputs must really be subnormal"
        return g

    assert run_chain(w, steps=3, seed=23, mutate=mutate)


@pytest.mark.parametrize("N,d,wc,sc", [(65535, 5, "sign", "sign"), (65535, 8, "identity", "sign"), (20_000, 9, "topk", "topk"),
                                        (20_000, 12, "randk", "sign")])
def test_largest_worker_counts(N, d, wc, sc):
    """As many rows as a launch grid's second dimension holds (liec_create's limit on N), short rows."""
    say(f"case many workers N={N} d={d} {wc}/{sc}")
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp=wc, server_comp=sc,
                         worker_k=2 if wc in ("topk", "randk") else 0, server_k=3 if sc == "topk" else 0, lr=0.05)
    assert run_chain(w, steps=2, seed=N + d, rk_seed=4, check_descs=False)


def test_largest_dimension_the_library_accepts():
    """d just below the limit of liec_create (2^31 - 2^20): column indices and tile counts near the top
    of the 32-bit range; one worker, scaled sign on both sides, every element compared."""
    import oracle
    from paper_2402_11857_amd import LiecContext, LiecError

    d = (1 << 31) - (1 << 20) - 4
    say(f"case largest dimension d={d}")
    with pytest.raises(LiecError):
        LiecContext(1, d + 4, "sign", "sign", 0, 0, 0.1)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(77)
    g = torch.empty((1, d), dtype=torch.float32, device=DEV)
    g.normal_(generator=gen)
    g[0, -5:] = torch.tensor([3.0, -0.0, 0.0, -2.0, 1.5], device=DEV)      # the last columns, exactly known
    x = torch.zeros((1, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    with LiecContext(1, d, "sign", "sign", 0, 0, 0.1) as ctx:
        ctx.step(g, x, e)
        torch.cuda.synchronize()
        scale = ctx.worker_desc()["scale"][0]
        assert ctx.info().nonfinite == 0
    gh = g.cpu().numpy()
    del g
    xo, eo = np.zeros((1, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    tr = oracle.step(gh, xo, eo, "sign", "sign", 0.1)
    say("  oracle step done")
    assert scale == np.float32(tr.worker[0].scale)
    assert H.bit_equal(e.cpu().numpy(), eo)
    assert H.bit_equal(x.cpu().numpy(), xo)


def test_largest_dimension_with_top_k():
    """The same dimension with top-k on both sides.  A full sort of 2^31 keys is beyond what the oracle
    finishes in the time a test has, so Definition 2 is checked through what is unique in it: the k-th
    largest key (numpy's selection), the number of larger keys, the cut-off among the ties, and then
    every element of the new state recomputed from those with single IEEE operations."""
    from paper_2402_11857_amd import LiecContext

    d, kw, ks, lr = (1 << 31) - (1 << 20) - 4, 100_000, 40_000, np.float32(0.1)
    say(f"case largest dimension, top-k d={d}")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(78)
    g = torch.empty((1, d), dtype=torch.float32, device=DEV)
    g.normal_(generator=gen)
    g[0, -3:] = torch.tensor([9.0, -9.0, 9.0], device=DEV)          # ties of the largest magnitude in the last columns
    x = torch.zeros((1, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    with LiecContext(1, d, "topk", "topk", kw, ks, float(lr)) as ctx:
        ctx.step(g, x, e)
        torch.cuda.synchronize()
        wd, info = ctx.worker_desc(), ctx.info()
        assert info.nonfinite == 0
    gh = g.cpu().numpy()[0]
    del g

    def select(vals, k):
        keys = vals.view(np.uint32) & np.uint32(0x7FFFFFFF)
        tau = np.partition(keys, vals.size - k)[vals.size - k]
        above = int((keys > tau).sum())
        ties = np.flatnonzero(keys == tau)
        cut = int(ties[k - above - 1])
        mask = keys > tau
        mask[ties[:k - above]] = True
        return int(tau), cut, mask

    tau_w, cut_w, mask_w = select(gh, kw)
    say("  worker selection done")
    assert (wd["tau_key"][0], wd["cutoff"][0]) == (tau_w, cut_w)
    p1 = np.where(mask_w, gh, np.float32(0.0))
    v = (np.float32(0.0) + p1) * np.float32(1.0) + np.float32(0.0)   # +0 + p, then fma(acc, 1/N = 1, e = 0)
    tau_s, cut_s, mask_s = select(v, ks)
    say("  server selection done")
    assert (info.server_tau_key, info.server_cutoff) == (tau_s, cut_s)
    p = np.where(mask_s, v, np.float32(0.0))
    assert H.bit_equal(e.cpu().numpy(), v - p)
    u = p + (gh - p1)
    assert H.bit_equal(x.cpu().numpy()[0], (-lr) * u + np.float32(0.0))


def test_error_norm_telemetry():
    """The l2 norm of the error variable (what Lemma 1 bounds) against a float64 sum of the oracle's state."""
    say("case l2 norm")
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=300_001, worker_comp="topk", server_comp="topk", worker_k=3000, server_k=3000)
    src = workloads.GradientSource(w, seed=2, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    with ctx_for(w) as ctx:
        assert ctx.l2_norm(e) == 0.0
        for t in range(4):
            g = src.grads(t)
            ctx.step(g, x, e)
            H.oracle_step_rows(g.cpu().numpy(), xo, eo, "topk", "topk", w.lr, w.worker_k, w.server_k)
            ref = float(np.sqrt(np.sum(eo.astype(np.float64) ** 2)))
            assert abs(ctx.l2_norm(e) - ref) <= 1e-12 * ref, f"step {t}"
        for n in (1, 5, 1023, 300_001):
            v = torch.randn(n, dtype=torch.float32, device=DEV)
            ref = float(np.sqrt(np.sum(v.cpu().numpy().astype(np.float64) ** 2)))
            assert abs(ctx.l2_norm(v) - ref) <= 1e-12 * ref
        ctx.step(src.grads(4), x, e)                      # the scratch it borrowed is the step's again
        H.oracle_step_rows(src.grads(4).cpu().numpy(), xo, eo, "topk", "topk", w.lr, w.worker_k, w.server_k)
        assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo)


def test_predicted_band_narrows_while_the_predictions_hold_and_reopens_after_a_miss():
    """The band a row is filtered against follows how far its thresholds fell from the predicted centres:
    on steady gradients it narrows step by step (fewer listed candidates, no failed prediction), a jump of
    the gradient scale makes the prediction fail once (counted) and the band restart wide.  Results are
    checked against the oracle all along."""
    import oracle
    from paper_2402_11857_amd import LiecContext

    N, d, k = 2, 2_000_000, 40_000
    say(f"case band width trajectory N={N} d={d} k={k}")
    w = workloads.scaled(WL["c1_tiny_sign"], N=N, d=d, worker_comp="topk", server_comp="sign", worker_k=k, lr=0.1)
    src = workloads.GradientSource(w, seed=5, device=DEV)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    widths, listed = [], []
    with LiecContext(N, d, "topk", "sign", k, 0, 0.1) as ctx:
        with pytest.raises(Exception):
            ctx.search_state(N)                         # the server's operator has no threshold search
        for t in range(24):
            g = src.grads(t)
            if t >= 20:
                g = g * 8.0
            ctx.step(g, x, e)
            oracle.step(g.cpu().numpy(), xo, eo, "topk", "sign", 0.1, k, 0)
            st = ctx.search_state(0)
            widths.append(st["hi"] - st["lo"])
            listed.append(st["listed"])
            assert st["mode"] == 0 and st["general_search"] == 0
            if t == 19:
                assert ctx.info().band_misses == 0, "steady gradients: no prediction may fail"
        assert ctx.info().band_misses == N, "the jump of the scale makes each worker row's prediction fail once"
        assert H.bit_equal(e.cpu().numpy(), eo) and H.bit_equal(x.cpu().numpy(), xo)
    assert widths[0] == 2 << 20, "after the first step the band is 2^20 keys on either side"
    assert min(widths[:20]) < widths[0] // 4 and widths[19] < widths[0], f"the band must narrow on steady gradients: {widths}"
    assert min(widths) >= 2 << 15, "the band never gets narrower than its floor"
    assert widths[20] == 2 << 20, "a failed prediction restarts the band wide"
    assert min(listed[2:20]) < listed[1] // 2, f"fewer candidates are listed once the band has narrowed: {listed}"


def test_more_candidates_in_one_block_than_its_stage_holds():
    """A stretch of 6000 neighbouring columns whose magnitudes lie within 0.02 % of the threshold: the filter
    blocks that cover it find four times as many candidates as their LDS stage holds, in the pass over the
    first-digit band of the first step and, once the band is predicted, in the pass over the predicted band,
    so the entries beyond the stage go through the waves' own stages to list slots reserved a batch at a time.  Checked against the oracle
    every step; the predictions must hold and the lists must contain the whole stretch."""
    import oracle
    from paper_2402_11857_amd import LiecContext

    N, d, k = 2, 150_000, 4000
    say(f"case stage overflow N={N} d={d} k={k}")
    rng = np.random.default_rng(77)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    with LiecContext(N, d, "topk", "sign", k, 0, 0.05) as ctx:
        for t in range(5):
            gh = (rng.standard_normal((N, d)) * 1e-3).astype(np.float32)
            gh[:, 100:1100] = np.where(rng.random((N, 1000)) < 0.5, -8.0, 8.0) * (1 + rng.random((N, 1000)))   # 1000 above
            near = 1.0 + 2e-4 * rng.random((N, 6000))                                                      # rank k falls in here
            gh[:, 20_000:26_000] = (np.where(rng.random((N, 6000)) < 0.5, -1.0, 1.0) * near).astype(np.float32)
            g = torch.from_numpy(gh).to(DEV)
            ctx.step(g, x, e)
            oracle.step(gh, xo, eo, "topk", "sign", 0.05, k, 0)
            assert H.bit_equal(e.cpu().numpy(), eo) and H.bit_equal(x.cpu().numpy(), xo), f"step {t}"
            for row in range(N):
                st = ctx.search_state(row)
                assert st["mode"] == 0 and st["general_search"] == 0
                assert st["listed"] >= 6000, f"step {t} row {row}: the stretch must be listed: {st}"
        assert ctx.info().band_misses == 0, "the threshold does not move: no prediction may fail"


@pytest.mark.parametrize("frac,sc", [(0.10, "topk"), (0.5, "sign"), (0.006, "topk")])
def test_long_candidate_lists_take_the_shared_passes(frac, sc):
    """Large k and the wide band of the first predicted steps give candidate lists far beyond what one block
    selects on its own (16 384 entries): the first list digit is counted and its bin collected by many blocks,
    or, when the bin itself is too large for the short list, the list is walked.  Gradients cut to 9 mantissa
    bits add thousands of equal keys.  Every step is checked against the oracle."""
    import oracle
    from paper_2402_11857_amd import LiecContext

    N, d = 2, 3_000_000
    k = int(frac * d)
    sk = k if sc == "topk" else 0
    say(f"case long candidate lists N={N} d={d} k={k} server {sc}")
    w = workloads.scaled(WL["c1_tiny_sign"], N=N, d=d, worker_comp="topk", server_comp=sc, worker_k=k, server_k=sk, lr=0.1)
    src = workloads.GradientSource(w, seed=31, device=DEV)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    longest = 0
    with LiecContext(N, d, "topk", sc, k, sk, 0.1) as ctx:
        for t in range(4):
            g = src.grads(t)
            if t >= 2:
                g = (g.view(torch.int32) & -(1 << 14)).view(torch.float32).contiguous()
            ctx.step(g, x, e)
            oracle.step(g.cpu().numpy(), xo, eo, "topk", sc, 0.1, k, sk)
            assert H.bit_equal(e.cpu().numpy(), eo), f"step {t}: server error"
            assert H.bit_equal(x.cpu().numpy(), xo), f"step {t}: models"
            longest = max(longest, ctx.search_state(0)["listed"])
            assert ctx.info().slow_rows == 0
    assert longest > 16_384, f"the case must list more candidates than one block takes on its own ({longest})"
