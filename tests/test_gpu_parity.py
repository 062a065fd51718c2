"""Parity of the HIP path against the CPU oracle, through the C ABI (via the thin binding).

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

import workloads  # noqa: E402

pytestmark = [pytest.mark.gpu,
              pytest.mark.skipif(not torch.cuda.is_available(), reason="needs an MI355X")]

DEV = "cuda:0"
WL = workloads.workloads()


def _ctx(w, **kw):
    from paper_2402_11857_amd import LiecContext

    return LiecContext(w.N, w.d, w.worker_comp, w.server_comp, w.worker_k, w.server_k, w.lr, **kw)


def _say(msg):
    print(msg, flush=True)


def _check_descs(ctx, w, wdesc, sdesc, g_host, v_host, label):
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


def _run_chain(w, steps, seed=0, teacher_forced=False, mutate=None, check_descs=True, tol_end=H.TOL_CHAIN,
               rk_seed=0, force_mode=None):
    """Runs `steps` chained steps on both sides and compares after every step.  rk_seed seeds the
    random-k draws (draw t in step t); force_mode[t], when given, is the search mode forced before step t."""
    src = workloads.GradientSource(w, seed=seed, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo = np.zeros((w.N, w.d), dtype=np.float32)
    eo = np.zeros(w.d, dtype=np.float32)
    exact = True
    with _ctx(w) as ctx:
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
                _check_descs(ctx, w, wdesc, sdesc, gh, v, label)
            tol = H.TOL_STEP if (t == 0 or teacher_forced) else tol_end
            assert H.rel_err(eg, eo) <= tol, f"{label}: server error"
            assert H.rel_err(xg, xo) <= tol, f"{label}: models"
            # integer-valued parts of the state: the sign pattern / support of the new error
            if w.server_comp in ("topk", "randk"):
                assert np.array_equal(eg == 0, eo == 0), f"{label}: server index set"
            exact = exact and H.bit_equal(xg, xo) and H.bit_equal(eg, eo)
    return exact


SMALL_SHAPES = [(1, 1), (2, 3), (3, 255), (4, 1024), (2, 1025), (5, 4100), (3, 50_003), (8, 70_000)]
PAIRS = [("sign", "sign"), ("topk", "topk"), ("topk", "sign"), ("sign", "topk"), ("identity", "identity"),
         ("identity", "sign"), ("topk", "identity"), ("sign", "identity"), ("identity", "topk")]


@pytest.mark.parametrize("wc,sc", PAIRS)
@pytest.mark.parametrize("N,d", SMALL_SHAPES)
def test_small_shapes_all_operator_pairs(N, d, wc, sc):
    _say(f"case small N={N} d={d} {wc}/{sc}")
    base = WL["c2_topk_mid"]
    k = max(1, d // 50)
    w = workloads.scaled(base, N=N, d=d, worker_comp=wc, server_comp=sc,
                         worker_k=k if wc == "topk" else 0, server_k=max(1, d // 20) if sc == "topk" else 0,
                         lr=0.05)
    assert _run_chain(w, steps=3, seed=N * 1000 + d), "expected bit identity with the oracle"


@pytest.mark.parametrize("wc,sc", [("topk", "topk"), ("topk", "sign"), ("sign", "topk")])
def test_ties_zeros_and_negative_zeros(wc, sc):
    _say(f"case ties {wc}/{sc}")
    base = WL["c2_topk_mid"]
    w = workloads.scaled(base, N=4, d=33_000, worker_comp=wc, server_comp=sc,
                         worker_k=3000 if wc == "topk" else 0, server_k=5000 if sc == "topk" else 0)

    def mutate(g, t):
        return workloads.inject_ties(g, seed=t, frac_zero=0.3, frac_dup=0.5)

    assert _run_chain(w, steps=4, seed=5, mutate=mutate)


@pytest.mark.parametrize("kind", ["all_zero", "all_equal", "one_hot", "k_equals_d", "k_equals_1"])
def test_degenerate_topk_inputs(kind):
    _say(f"case degenerate {kind}")
    base = WL["c2_topk_mid"]
    d = 5000
    k = {"k_equals_d": d, "k_equals_1": 1}.get(kind, 100)
    w = workloads.scaled(base, N=3, d=d, worker_comp="topk", server_comp="topk", worker_k=k, server_k=k)

    def mutate(g, t):
        if kind == "all_zero":
            g.zero_()
        elif kind == "all_equal":
            g.fill_(0.125)
            g[:, ::3] *= -1
        elif kind == "one_hot":
            g.zero_()
            g[:, 4321] = -7.0
        return g

    assert _run_chain(w, steps=3, seed=1, mutate=mutate)


def test_sign_with_zero_gradient_rows():
    _say("case sign zero rows")
    w = workloads.scaled(WL["c1_tiny_sign"], N=3, d=2048)

    def mutate(g, t):
        g[1].zero_()
        g[2, ::2] = -0.0
        return g

    assert _run_chain(w, steps=3, seed=2, mutate=mutate)


def test_c1_tiny_full_chain():
    w = WL["c1_tiny_sign"]
    _say(f"case {w.name} {w.steps} chained steps")
    assert _run_chain(w, steps=w.steps, seed=0)


def test_c2_topk_mid_full_chain():
    w = WL["c2_topk_mid"]
    _say(f"case {w.name} {w.steps} chained steps")
    assert _run_chain(w, steps=w.steps, seed=0)


def test_c2_teacher_forced():
    w = WL["c2_topk_mid"]
    _say(f"case {w.name} teacher forced")
    _run_chain(w, steps=5, seed=3, teacher_forced=True)


def test_unaligned_pointers_take_the_elementwise_path():
    _say("case unaligned pointers")
    from paper_2402_11857_amd import LiecContext

    N, d = 3, 6000
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp="topk", server_comp="sign", worker_k=77)
    src = workloads.GradientSource(w, seed=9, device=DEV)
    g = src.grads(0)
    pad = torch.zeros(N * d + 1, dtype=torch.float32, device=DEV)
    x = pad[1:].view(N, d)              # 4-byte aligned only
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    with LiecContext(N, d, "topk", "sign", 77, 0, 0.1) as ctx:
        for t in range(2):
            g = src.grads(t)
            ctx.step(g, x, e)
            H.oracle_step_rows(g.cpu().numpy(), xo, eo, "topk", "sign", 0.1, 77, 0)
    assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo)


def test_runs_are_bit_reproducible_and_resumable():
    _say("case determinism / resume")
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=300_000, worker_comp="topk", server_comp="sign", worker_k=3000)
    src = workloads.GradientSource(w, seed=4, device=DEV)
    gs = [src.grads(t) for t in range(6)]

    def run(split):
        x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
        e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
        ctx = _ctx(w)
        for t, g in enumerate(gs):
            if t == split:          # all algorithm state lives in x and e: a new context resumes
                ctx.close()
                ctx = _ctx(w)
            ctx.step(g, x, e)
        torch.cuda.synchronize()
        ctx.close()
        return x.cpu().numpy(), e.cpu().numpy()

    a, b, c = run(None), run(None), run(3)
    assert H.bit_equal(a[0], b[0]) and H.bit_equal(a[1], b[1])
    assert H.bit_equal(a[0], c[0]) and H.bit_equal(a[1], c[1])


def test_non_default_stream_and_lr_schedule():
    _say("case stream / set_lr")
    w = workloads.scaled(WL["c1_tiny_sign"], N=4, d=40_000)
    src = workloads.GradientSource(w, seed=6, device=DEV)
    s = torch.cuda.Stream()
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    gs = [src.grads(t) for t in range(4)]
    torch.cuda.synchronize()
    with _ctx(w, stream=s) as ctx:
        for t, g in enumerate(gs):
            lr = 0.1 / (1 + t)
            ctx.set_lr(lr)
            ctx.step(g, x, e)
            H.oracle_step_rows(g.cpu().numpy(), xo, eo, "sign", "sign", lr)
        s.synchronize()
    assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo)


def test_step_rejects_bad_buffers_and_reports_nonfinite_input():
    _say("case errors")
    from paper_2402_11857_amd import LiecContext, LiecError, liec_step

    N, d = 2, 4096
    g = torch.randn((N, d), device=DEV)
    x = torch.zeros((N, d), device=DEV)
    e = torch.zeros(d, device=DEV)
    with LiecContext(N, d, "sign", "topk", 0, 10, 0.1) as ctx:
        with pytest.raises(LiecError):
            liec_step(ctx._h, g.data_ptr(), g.data_ptr(), e.data_ptr())      # x overlaps grads
        with pytest.raises(LiecError):
            liec_step(ctx._h, g.data_ptr(), x.data_ptr(), x.data_ptr())      # e overlaps x
        with pytest.raises(LiecError):
            liec_step(ctx._h, g.data_ptr(), None, e.data_ptr())
        with pytest.raises((TypeError, ValueError)):
            ctx.step(g[:, :100], x, e)
        ctx.step(g, x, e)
        assert ctx.info_status()[1] == 0
        g[1, 17] = float("inf")
        ctx.step(g, x, e)
        info, st = ctx.info_status()
        assert st == 4 and info.nonfinite == 1
    with LiecContext(N, d, "topk", "sign", 10, 0, 0.1) as ctx:
        x.zero_(), e.zero_()
        g[1, 17] = float("nan")
        ctx.step(g, x, e)
        assert ctx.info_status()[1] == 4


def test_two_contexts_on_two_streams_do_not_interfere():
    """The library keeps no global state: two contexts with different operators, sizes and streams,
    stepping in turns without synchronising in between, give what each gives alone."""
    _say("case two contexts")
    wa = workloads.scaled(WL["c2_topk_mid"], N=4, d=150_000, worker_comp="topk", server_comp="sign", worker_k=1500)
    wb = workloads.scaled(WL["c2_topk_mid"], N=3, d=90_001, worker_comp="randk", server_comp="topk", worker_k=900, server_k=2000)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    srcs = [workloads.GradientSource(w, seed=5 + q, device=DEV) for q, w in enumerate((wa, wb))]
    gs = [[src.grads(t) for t in range(4)] for src in srcs]
    xs = [torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV) for w in (wa, wb)]
    es = [torch.zeros(w.d, dtype=torch.float32, device=DEV) for w in (wa, wb)]
    torch.cuda.synchronize()
    with _ctx(wa, stream=sa) as ca, _ctx(wb, stream=sb) as cb:
        cb.set_random(3, 0)
        for t in range(4):
            ca.step(gs[0][t], xs[0], es[0])
            cb.step(gs[1][t], xs[1], es[1])
        sa.synchronize()
        sb.synchronize()
    for q, w in enumerate((wa, wb)):
        xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
        for t in range(4):
            H.oracle_step_rows(gs[q][t].cpu().numpy(), xo, eo, w.worker_comp, w.server_comp, w.lr, w.worker_k, w.server_k,
                               rng=(3, t))
        assert H.bit_equal(xs[q].cpu().numpy(), xo) and H.bit_equal(es[q].cpu().numpy(), eo), f"context {q}"


def test_out_of_memory_is_reported_and_leaves_the_library_usable():
    _say("case out of memory")
    from paper_2402_11857_amd import LiecContext, LiecError

    with pytest.raises(LiecError) as err:          # the candidate lists alone would take about 1 TB
        LiecContext(1000, 2_000_000_000, "topk", "topk", 1000, 1000, 0.1)
    assert err.value.status == 2
    w = workloads.scaled(WL["c1_tiny_sign"], N=2, d=5000)
    assert _run_chain(w, steps=2, seed=1)


def test_per_kernel_timing_and_scratch_accounting():
    _say("case profile api")
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=200_000, worker_comp="topk", server_comp="sign", worker_k=2000)
    g = workloads.GradientSource(w, seed=1, device=DEV).grads(0)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    with _ctx(w) as ctx:
        assert ctx.scratch_bytes() > w.d * 4                  # at least the v buffer
        ctx.step(g, x, e)
        ctx.profile_begin(2, update_only=True)
        for _ in range(3):                                    # only the first two steps are recorded
            ctx.step(g, x, e)
        got = ctx.profile_end()
        assert set(got) == {"update"} and got["update"][1] == 2 and got["update"][0] > 0
        ctx.profile_begin(1)
        ctx.step(g, x, e)
        got = ctx.profile_end()
        assert {"worker_filter_warm", "server_aggregate", "update"} <= set(got)
        assert all(n == 1 and ms >= 0 for ms, n in got.values())
        ctx.step(g, x, e)                                     # recording is off again
        assert ctx.profile_end() == {}
        assert ctx.info().steps_done == 6


# ---- random-k (Definition 3) -----------------------------------------------------------------------
RK_PAIRS = [("randk", "randk"), ("randk", "sign"), ("topk", "randk"), ("sign", "randk"), ("randk", "identity"),
            ("identity", "randk"), ("randk", "topk")]


@pytest.mark.parametrize("wc,sc", RK_PAIRS)
@pytest.mark.parametrize("N,d", SMALL_SHAPES)
def test_random_k_small_shapes(N, d, wc, sc):
    _say(f"case randk small N={N} d={d} {wc}/{sc}")
    wk = max(1, d // 50) if wc in ("topk", "randk") else 0
    sk = max(1, d // 20) if sc in ("topk", "randk") else 0
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp=wc, server_comp=sc, worker_k=wk, server_k=sk, lr=0.05)
    assert _run_chain(w, steps=3, seed=N * 1000 + d, rk_seed=d * 7 + N), "expected bit identity with the oracle"


@pytest.mark.parametrize("d,k", [(5000, 5000), (5000, 1), (5000, 4999), (1024, 512), (262_144, 131_072), (4097, 4096)])
def test_random_k_extreme_k(d, k):
    _say(f"case randk extreme d={d} k={k}")
    w = workloads.scaled(WL["c2_topk_mid"], N=3, d=d, worker_comp="randk", server_comp="randk", worker_k=k, server_k=k)
    assert _run_chain(w, steps=3, seed=3, rk_seed=1)


@pytest.mark.parametrize("modes", [None, [1, 0, 4]])
def test_random_k_with_a_thin_band_walks_the_priorities(modes):
    """k * 2^32 / d far below d: the library inverts the priority permutation over the words above the
    band instead of hashing every column; same kept sets, in every search mode."""
    _say(f"case randk thin band modes={modes}")
    w = workloads.scaled(WL["c2_topk_mid"], N=3, d=4_000_003, worker_comp="randk", server_comp="randk",
                         worker_k=400, server_k=1000)
    assert _run_chain(w, steps=3, seed=12, rk_seed=99, force_mode=modes)


@pytest.mark.parametrize("modes", [[1, 0, 1], [4, 0, 4], [0, 4, 1]])
@pytest.mark.parametrize("wc,sc", [("randk", "randk"), ("topk", "topk")])
def test_every_search_mode_gives_the_same_result(wc, sc, modes):
    """Predicted band, first-digit histogram and the general search are forced in turn."""
    _say(f"case forced search modes {wc}/{sc} {modes}")
    w = workloads.scaled(WL["c2_topk_mid"], N=3, d=150_001, worker_comp=wc, server_comp=sc, worker_k=1500, server_k=7000)
    assert _run_chain(w, steps=3, seed=8, rk_seed=21, force_mode=modes)


def test_random_k_draws_follow_seed_and_counter_and_resume():
    _say("case randk seed / counter / resume")
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=100_000, worker_comp="randk", server_comp="randk",
                         worker_k=1000, server_k=5000)
    src = workloads.GradientSource(w, seed=4, device=DEV)
    gs = [src.grads(t) for t in range(5)]

    def run(seed, split=None, sync_at=None):
        x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
        e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
        ctx = _ctx(w)
        ctx.set_random(seed, 0)
        for t, g in enumerate(gs):
            if t == split:              # a new context resumes from x, e and the generator's (seed, draw)
                state = ctx.get_random()
                ctx.close()
                ctx = _ctx(w)
                ctx.set_random(*state)
            ctx.step(g, x, e)
        torch.cuda.synchronize()
        assert ctx.get_random() == (seed, len(gs))
        ctx.close()
        return x.cpu().numpy(), e.cpu().numpy()

    a, b, c, other = run(5), run(5), run(5, split=2), run(6)
    assert H.bit_equal(a[0], b[0]) and H.bit_equal(a[1], b[1])
    assert H.bit_equal(a[0], c[0]) and H.bit_equal(a[1], c[1])
    assert not H.bit_equal(a[1], other[1])


@pytest.mark.parametrize("N,d,k", [(2, 9, 3), (3, 1001, 50), (4, 70_003, 700), (2, 5000, 5000)])
def test_random_k_message_wire_form_round_trip(N, d, k):
    _say(f"case wire randk N={N} d={d} k={k}")
    import oracle
    from paper_2402_11857_amd import LiecContext

    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp="randk", server_comp="sign", worker_k=k, server_k=0)
    g = workloads.GradientSource(w, seed=d + k, device=DEV).grads(0)
    gh = g.cpu().numpy()
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    idx = torch.empty(k, dtype=torch.int32, device=DEV)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    p = torch.empty(d, dtype=torch.float32, device=DEV)
    with LiecContext(N, d, "randk", "sign", k, 0, 0.1) as ctx:
        ctx.set_random(77, 3)
        ctx.step(g, x, e)
        for i in range(N):
            idx.fill_(-1)
            ctx.pack_topk_message(g, i, idx, val)
            ctx.unpack_topk_message(idx, val, p)
            torch.cuda.synchronize()
            ri, rv = oracle.pack_randk(gh[i], k, (77, 3, i))
            assert np.array_equal(idx.cpu().numpy().view(np.uint32), ri), f"worker {i}: indices"
            assert H.bit_equal(val.cpu().numpy(), rv), f"worker {i}: values"
            assert H.bit_equal(p.cpu().numpy(), oracle.compress("randk", gh[i], k, rng=(77, 3, i))[0])


def test_wire_scratch_survives_a_sign_unpack_between_two_topk_packs():
    _say("case wire scratch reuse")
    import oracle
    from paper_2402_11857_amd import LiecContext

    N, d, k = 2, 20_000, 200
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp="topk", server_comp="sign", worker_k=k, server_k=0)
    g = workloads.GradientSource(w, seed=1, device=DEV).grads(0)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    idx = torch.empty(k, dtype=torch.int32, device=DEV)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    p = torch.empty(d, dtype=torch.float32, device=DEV)
    bits = torch.zeros((d + 7) // 8, dtype=torch.uint8, device=DEV)
    with LiecContext(N, d, "topk", "sign", k, 0, 0.1) as ctx:
        ctx.step(g, x, e)
        ctx.pack_topk_message(g, 0, idx, val)
        ctx.unpack_sign_message(bits, [0.5], False, p)        # allocates the scale staging
        ctx.pack_topk_message(g, 1, idx, val)
        torch.cuda.synchronize()
        ri, rv = oracle.pack_topk(g[1].cpu().numpy(), k)
        assert np.array_equal(idx.cpu().numpy().view(np.uint32), ri) and H.bit_equal(val.cpu().numpy(), rv)
        assert np.all(p.cpu().numpy() == 0.5)


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
    _say(f"case sweep {case}: N={N} d={d} {wc}/{sc} k={wk}/{sk} lr={lr} blocks={len(off) - 1}")
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp=wc, server_comp=sc, worker_k=wk, server_k=sk, lr=lr)
    src = workloads.GradientSource(w, seed=case, device=DEV)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    with LiecContext(N, d, wc, sc, wk, sk, lr) as ctx:
        ctx.set_random(case, 5)
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


@pytest.mark.parametrize("wc,sc", [("topk", "topk"), ("topk", "sign")])
def test_threshold_prediction_survives_jumps_of_the_gradient_scale(wc, sc):
    """The band predicted from the last thresholds misses when the gradients' scale jumps; the step must
    then find the threshold the long way and still match the oracle (drifts are followed by the trend)."""
    _say(f"case scale jumps {wc}/{sc}")
    w = workloads.scaled(WL["c2_topk_mid"], N=3, d=180_000, worker_comp=wc, server_comp=sc, worker_k=1800,
                         server_k=4000 if sc == "topk" else 0)
    scales = [1.0, 1.0, 4.0, 4.2, 4.4, 0.05, 0.05, 0.049, 1e-6, 3.0]

    def mutate(g, t):
        return g * scales[t]

    assert _run_chain(w, steps=len(scales), seed=17, mutate=mutate)


@pytest.mark.parametrize("wc,sc", [("sign", "sign"), ("topk", "topk"), ("identity", "identity")])
def test_subnormal_and_huge_magnitudes(wc, sc):
    """fp32 subnormals must be kept, not flushed, and magnitudes near the top of the range must not overflow
    the fp64 L1 sums: gradients span 1e-44 .. 1e37."""
    _say(f"case subnormal / huge {wc}/{sc}")
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

    assert _run_chain(w, steps=3, seed=23, mutate=mutate)


@pytest.mark.parametrize("N,d,wc,sc", [(65535, 5, "sign", "sign"), (65535, 8, "identity", "sign"), (20_000, 9, "topk", "topk"),
                                        (20_000, 12, "randk", "sign")])
def test_largest_worker_counts(N, d, wc, sc):
    """As many rows as a launch grid's second dimension holds (liec_create's limit on N), short rows."""
    _say(f"case many workers N={N} d={d} {wc}/{sc}")
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp=wc, server_comp=sc,
                         worker_k=2 if wc in ("topk", "randk") else 0, server_k=3 if sc == "topk" else 0, lr=0.05)
    assert _run_chain(w, steps=2, seed=N + d, rk_seed=4, check_descs=False)


def test_largest_dimension_the_library_accepts():
    """d just below the limit of liec_create (2^31 - 2^20): column indices and tile counts near the top
    of the 32-bit range; one worker, scaled sign on both sides, every element compared."""
    import oracle
    from paper_2402_11857_amd import LiecContext, LiecError

    d = (1 << 31) - (1 << 20) - 4
    _say(f"case largest dimension d={d}")
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
    _say("  oracle step done")
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
    _say(f"case largest dimension, top-k d={d}")
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
    _say("  worker selection done")
    assert (wd["tau_key"][0], wd["cutoff"][0]) == (tau_w, cut_w)
    p1 = np.where(mask_w, gh, np.float32(0.0))
    v = (np.float32(0.0) + p1) * np.float32(1.0) + np.float32(0.0)   # +0 + p, then fma(acc, 1/N = 1, e = 0)
    tau_s, cut_s, mask_s = select(v, ks)
    _say("  server selection done")
    assert (info.server_tau_key, info.server_cutoff) == (tau_s, cut_s)
    p = np.where(mask_s, v, np.float32(0.0))
    assert H.bit_equal(e.cpu().numpy(), v - p)
    u = p + (gh - p1)
    assert H.bit_equal(x.cpu().numpy()[0], (-lr) * u + np.float32(0.0))


def test_error_norm_telemetry():
    """The l2 norm of the error variable (what Lemma 1 bounds) against a float64 sum of the oracle's state."""
    _say("case l2 norm")
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=300_001, worker_comp="topk", server_comp="topk", worker_k=3000, server_k=3000)
    src = workloads.GradientSource(w, seed=2, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    with _ctx(w) as ctx:
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


# ---- the step under HIP graph capture ----------------------------------------------------------------
@pytest.mark.parametrize("wc,sc", [("sign", "sign"), ("topk", "topk"), ("topk", "sign"), ("randk", "randk")])
def test_step_captured_in_a_hip_graph_replays_like_eager_steps(wc, sc):
    """liec_step neither allocates, synchronises nor copies, and every decision of the threshold
    search is taken on the device, so a caller may capture it once and replay it; each replay is
    compared with the oracle, with eager work and synchronisation between the replays."""
    _say(f"case graph capture {wc}/{sc}")
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
    with _ctx(w, stream=s) as ctx, torch.cuda.stream(s):
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


# ---- Blockwise-SignSGD (Definition 5) --------------------------------------------------------------
BLOCK_TABLES = {
    "one": lambda d: [0, d],
    "aligned": lambda d: [0, d // 4 // 4 * 4, d // 2 // 4 * 4, d],
    "ragged": lambda d: sorted({0, 1, 7, d // 3, d // 3 + 1, 2 * d // 3 + 5, d - 1, d}),
    "many": lambda d: list(range(0, d, max(1, d // 37))) + [d] if d % max(1, d // 37) else list(range(0, d + 1, max(1, d // 37))),
}


@pytest.mark.parametrize("table", list(BLOCK_TABLES))
@pytest.mark.parametrize("wc,sc", [("blocksign", "blocksign"), ("blocksign", "sign"), ("topk", "blocksign"),
                                   ("blocksign", "topk"), ("identity", "blocksign")])
@pytest.mark.parametrize("N,d", [(3, 5000), (4, 70_001), (2, 12_288)])
def test_blockwise_sign(N, d, wc, sc, table):
    _say(f"case blocksign N={N} d={d} {wc}/{sc} table={table}")
    import oracle
    from paper_2402_11857_amd import LiecContext

    off = BLOCK_TABLES[table](d)
    assert off[0] == 0 and off[-1] == d and all(a < b for a, b in zip(off, off[1:]))
    k = max(1, d // 50)
    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp=wc, server_comp=sc,
                         worker_k=k if wc == "topk" else 0, server_k=k if sc == "topk" else 0, lr=0.05)
    src = workloads.GradientSource(w, seed=d + N, device=DEV)
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((N, d), dtype=np.float32), np.zeros(d, dtype=np.float32)
    with LiecContext(N, d, wc, sc, w.worker_k, w.server_k, w.lr) as ctx:
        ctx.set_blocks(off)
        for t in range(3):
            g = src.grads(t)
            ctx.step(g, x, e)
            tr = oracle.step_blocks(g.cpu().numpy(), xo, eo, wc, sc, w.lr, off, w.worker_k, w.server_k)
            ws, ss = ctx.block_scales()
            if wc == "blocksign":
                assert np.array_equal(np.array(ws, dtype=np.float32), tr.worker_scales), f"step {t}: worker block scales"
            if sc == "blocksign":
                assert np.array_equal(np.array(ss, dtype=np.float32), tr.server_scales), f"step {t}: server block scales"
            assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo), f"step {t}"
        assert ctx.info().nonfinite == 0


def test_blockwise_sign_needs_a_block_table_and_validates_it():
    _say("case blocksign errors")
    from paper_2402_11857_amd import LiecContext, LiecError

    N, d = 2, 4096
    g = torch.randn((N, d), device=DEV)
    x = torch.zeros((N, d), device=DEV)
    e = torch.zeros(d, device=DEV)
    with LiecContext(N, d, "blocksign", "blocksign", 0, 0, 0.1) as ctx:
        with pytest.raises(LiecError):
            ctx.step(g, x, e)                       # no table yet
        for bad in ([0, 100, 100, d], [1, d], [0, d - 1], [0, 3000, 2000, d]):
            with pytest.raises(LiecError):
                ctx.set_blocks(bad)
        ctx.set_blocks([0, 1000, d])
        ctx.step(g, x, e)
        ctx.set_blocks([0, d])                      # a new table replaces the old one
        ctx.step(g, x, e)
        torch.cuda.synchronize()


def test_full_size_c3_resnet18_blocksign():
    import oracle
    w = WL["c3_resnet18_blocksign"]
    _say(f"case full size {w.name} blocks={len(w.blocks) - 1}")
    src = workloads.GradientSource(w, seed=0, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    with _ctx(w) as ctx:
        ctx.set_blocks(w.blocks)
        for t in range(2):
            g = src.grads(t)
            ctx.step(g, x, e)
            tr = oracle.step_blocks(g.cpu().numpy(), xo, eo, "blocksign", "blocksign", w.lr, w.blocks)
            ws, ss = ctx.block_scales()
            assert np.array_equal(np.array(ws, dtype=np.float32), tr.worker_scales)
            assert np.array_equal(np.array(ss, dtype=np.float32), tr.server_scales)
            assert H.bit_equal(e.cpu().numpy(), eo)
            for i in range(w.N):
                assert H.bit_equal(x[i].cpu().numpy(), xo[i]), f"step {t} row {i}"


# ---- wire form of the sign messages ----------------------------------------------------------------
@pytest.mark.parametrize("comp", ["sign", "blocksign"])
@pytest.mark.parametrize("N,d", [(2, 8), (3, 1001), (4, 70_003), (2, 262_144)])
def test_sign_message_wire_form_round_trip(N, d, comp):
    _say(f"case wire N={N} d={d} {comp}")
    import oracle
    from paper_2402_11857_amd import LiecContext

    off = [0, d] if d < 16 else sorted({0, 5, d // 3, d // 2 + 1, d})
    w = workloads.scaled(WL["c1_tiny_sign"], N=N, d=d, worker_comp=comp, server_comp=comp)
    g = workloads.GradientSource(w, seed=d, device=DEV).grads(0)
    g[0, ::3] = 0.0
    g[0, 1::5] = -0.0
    gh = g.cpu().numpy()
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    bits = torch.empty((d + 7) // 8, dtype=torch.uint8, device=DEV)
    p = torch.empty(d, dtype=torch.float32, device=DEV)
    with LiecContext(N, d, comp, comp, 0, 0, 0.1) as ctx:
        if comp == "blocksign":
            ctx.set_blocks(off)
        ctx.step(g, x, e)
        scales = ctx.block_scales()[0] if comp == "blocksign" else [[s] for s in ctx.worker_desc()["scale"]]
        for i in range(N):
            ctx.pack_sign_bits(i, bits)
            ctx.unpack_sign_message(bits, scales[i], comp == "blocksign", p)
            torch.cuda.synchronize()
            assert np.array_equal(bits.cpu().numpy(), oracle.pack_sign(gh[i])), f"worker {i}: wire bits"
            ref = oracle.compress_blocksign(gh[i], off)[0] if comp == "blocksign" else oracle.compress("sign", gh[i])[0]
            assert H.bit_equal(p.cpu().numpy(), ref), f"worker {i}: decompressed message"


@pytest.mark.parametrize("N,d,k", [(2, 9, 3), (3, 1001, 50), (4, 70_003, 700), (2, 262_144, 262_144), (2, 5000, 1)])
def test_topk_message_wire_form_round_trip(N, d, k):
    _say(f"case wire topk N={N} d={d} k={k}")
    import oracle
    from paper_2402_11857_amd import LiecContext

    w = workloads.scaled(WL["c2_topk_mid"], N=N, d=d, worker_comp="topk", server_comp="sign", worker_k=k, server_k=0)
    g = workloads.GradientSource(w, seed=d + k, device=DEV).grads(0)
    g = workloads.inject_ties(g, seed=k, frac_zero=0.2, frac_dup=0.3)
    gh = g.cpu().numpy()
    x = torch.zeros((N, d), dtype=torch.float32, device=DEV)
    e = torch.zeros(d, dtype=torch.float32, device=DEV)
    idx = torch.empty(k, dtype=torch.int32, device=DEV)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    p = torch.empty(d, dtype=torch.float32, device=DEV)
    with LiecContext(N, d, "topk", "sign", k, 0, 0.1) as ctx:
        ctx.step(g, x, e)
        for i in range(N):
            idx.fill_(-1)
            ctx.pack_topk_message(g, i, idx, val)
            ctx.unpack_topk_message(idx, val, p)
            torch.cuda.synchronize()
            ri, rv = oracle.pack_topk(gh[i], k)
            assert np.array_equal(idx.cpu().numpy().view(np.uint32), ri), f"worker {i}: indices"
            assert H.bit_equal(val.cpu().numpy(), rv), f"worker {i}: values"
            assert H.bit_equal(p.cpu().numpy(), oracle.compress("topk", gh[i], k)[0]), f"worker {i}: decompressed"


# ---- averaging iteration of Algorithm 1 ------------------------------------------------------------
@pytest.mark.parametrize("N,d", [(1, 1), (3, 1023), (4, 4096), (5, 50_003), (16, 70_000)])
def test_sync_iteration_small_shapes(N, d):
    _say(f"case sync N={N} d={d}")
    from paper_2402_11857_amd import LiecContext

    import oracle
    rng = np.random.default_rng(N * 7 + d)
    g = rng.standard_normal((N, d)).astype(np.float32)
    x = rng.standard_normal((N, d)).astype(np.float32)
    e = (0.1 * rng.standard_normal(d)).astype(np.float32)
    gd, xd, ed = (torch.from_numpy(a).to(DEV) for a in (g, x, e))
    with LiecContext(N, d, "sign", "sign", 0, 0, 0.05) as ctx:
        ctx.step_sync(gd, xd, ed)
        torch.cuda.synchronize()
    oracle.step_sync(g, x, e, 0.05)
    assert H.bit_equal(xd.cpu().numpy(), x) and H.bit_equal(ed.cpu().numpy(), e)
    assert not e.any()


@pytest.mark.parametrize("wc,sc", [("sign", "sign"), ("topk", "topk"), ("topk", "sign")])
def test_mixed_chain_with_averaging_period(wc, sc):
    """Algorithm 1 in full: compressed iterations, an averaging iteration every 4th step."""
    _say(f"case period chain {wc}/{sc}")
    import oracle
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=120_000, worker_comp=wc, server_comp=sc,
                         worker_k=1200 if wc == "topk" else 0, server_k=1200 if sc == "topk" else 0)
    src = workloads.GradientSource(w, seed=11, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    with _ctx(w) as ctx:
        for t in range(13):
            g = src.grads(t)
            gh = g.cpu().numpy()
            ctx.iteration(t, 4, g, x, e)               # Algorithm 1 as a whole: the library picks the branch
            if (t + 1) % 4 == 0:
                oracle.step_sync(gh, xo, eo, w.lr)
            else:
                H.oracle_step_rows(gh, xo, eo, wc, sc, w.lr, w.worker_k, w.server_k)
            assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo), f"step {t}"


def test_full_size_c3_sync_iteration():
    import oracle
    w = WL["c3_resnet18_sign"]
    _say(f"case full size sync {w.name}")
    src = workloads.GradientSource(w, seed=2, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    with _ctx(w) as ctx:
        g = src.grads(0)
        ctx.step(g, x, e)                      # make the local models differ first
        H.oracle_step_rows(g.cpu().numpy(), xo, eo, "sign", "sign", w.lr)
        g = src.grads(1)
        ctx.step_sync(g, x, e)
        oracle.step_sync(g.cpu().numpy(), xo, eo, w.lr)
    assert H.bit_equal(e.cpu().numpy(), eo)
    for i in range(w.N):
        assert H.bit_equal(x[i].cpu().numpy(), xo[i]), f"row {i}"


# ---- full-size configurations, in the launch configuration the bench times -------------------
def _full_size_steps(name, steps, seed=0):
    w = WL[name]
    _say(f"case full size {name} N={w.N} d={w.d} steps={steps}")
    src = workloads.GradientSource(w, seed=seed, device=DEV)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo = np.zeros((w.N, w.d), dtype=np.float32)
    eo = np.zeros(w.d, dtype=np.float32)
    with _ctx(w) as ctx:
        ctx.set_random(seed + 1000, 0)
        for t in range(steps):
            g = src.grads(t)
            ctx.step(g, x, e)
            gh = g.cpu().numpy()
            del g
            wdesc, sdesc, v, p, P = H.oracle_step_rows(gh, xo, eo, w.worker_comp, w.server_comp, w.lr,
                                                       w.worker_k, w.server_k, rng=(seed + 1000, t))
            _say(f"  oracle step {t} done")
            _check_descs(ctx, w, wdesc, sdesc, gh, v, f"{name} step {t}")
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
