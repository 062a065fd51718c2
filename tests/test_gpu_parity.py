"""Parity of the HIP path against the CPU oracle through the C ABI: every operator pair on small shapes,
ties and degenerate inputs, the two small configurations' chains, streams, errors, timing.
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


@pytest.mark.parametrize("wc,sc", PAIRS)
@pytest.mark.parametrize("N,d", SMALL_SHAPES)
def test_small_shapes_all_operator_pairs(N, d, wc, sc):
    say(f"case small N={N} d={d} {wc}/{sc}")
    base = WL["c2_topk_mid"]
    k = max(1, d // 50)
    w = workloads.scaled(base, N=N, d=d, worker_comp=wc, server_comp=sc,
                         worker_k=k if wc == "topk" else 0, server_k=max(1, d // 20) if sc == "topk" else 0,
                         lr=0.05)
    assert run_chain(w, steps=3, seed=N * 1000 + d), "expected bit identity with the oracle"


@pytest.mark.parametrize("wc,sc", [("topk", "topk"), ("topk", "sign"), ("sign", "topk")])
def test_ties_zeros_and_negative_zeros(wc, sc):
    say(f"case ties {wc}/{sc}")
    base = WL["c2_topk_mid"]
    w = workloads.scaled(base, N=4, d=33_000, worker_comp=wc, server_comp=sc,
                         worker_k=3000 if wc == "topk" else 0, server_k=5000 if sc == "topk" else 0)

    def mutate(g, t):
        return workloads.inject_ties(g, seed=t, frac_zero=0.3, frac_dup=0.5)

    assert run_chain(w, steps=4, seed=5, mutate=mutate)


@pytest.mark.parametrize("kind", ["all_zero", "all_equal", "one_hot", "k_equals_d", "k_equals_1"])
def test_degenerate_topk_inputs(kind):
    say(f"case degenerate {kind}")
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

    assert run_chain(w, steps=3, seed=1, mutate=mutate)


def test_sign_with_zero_gradient_rows():
    say("case sign zero rows")
    w = workloads.scaled(WL["c1_tiny_sign"], N=3, d=2048)

    def mutate(g, t):
        g[1].zero_()
        g[2, ::2] = -0.0
        return g

    assert run_chain(w, steps=3, seed=2, mutate=mutate)


def test_c1_tiny_full_chain():
    w = WL["c1_tiny_sign"]
    say(f"case {w.name} {w.steps} chained steps")
    assert run_chain(w, steps=w.steps, seed=0)


def test_c2_topk_mid_full_chain():
    w = WL["c2_topk_mid"]
    say(f"case {w.name} {w.steps} chained steps")
    assert run_chain(w, steps=w.steps, seed=0)


def test_c2_teacher_forced():
    w = WL["c2_topk_mid"]
    say(f"case {w.name} teacher forced")
    run_chain(w, steps=5, seed=3, teacher_forced=True)


def test_unaligned_pointers_take_the_elementwise_path():
    say("case unaligned pointers")
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
    say("case determinism / resume")
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=300_000, worker_comp="topk", server_comp="sign", worker_k=3000)
    src = workloads.GradientSource(w, seed=4, device=DEV)
    gs = [src.grads(t) for t in range(6)]

    def run(split):
        x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
        e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
        ctx = ctx_for(w)
        for t, g in enumerate(gs):
            if t == split:          # all algorithm state lives in x and e: a new context resumes
                ctx.close()
                ctx = ctx_for(w)
            ctx.step(g, x, e)
        torch.cuda.synchronize()
        ctx.close()
        return x.cpu().numpy(), e.cpu().numpy()

    a, b, c = run(None), run(None), run(3)
    assert H.bit_equal(a[0], b[0]) and H.bit_equal(a[1], b[1])
    assert H.bit_equal(a[0], c[0]) and H.bit_equal(a[1], c[1])


def test_non_default_stream_and_lr_schedule():
    say("case stream / set_lr")
    w = workloads.scaled(WL["c1_tiny_sign"], N=4, d=40_000)
    src = workloads.GradientSource(w, seed=6, device=DEV)
    s = torch.cuda.Stream()
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xo, eo = np.zeros((w.N, w.d), dtype=np.float32), np.zeros(w.d, dtype=np.float32)
    gs = [src.grads(t) for t in range(4)]
    torch.cuda.synchronize()
    with ctx_for(w, stream=s) as ctx:
        for t, g in enumerate(gs):
            lr = 0.1 / (1 + t)
            ctx.set_lr(lr)
            ctx.step(g, x, e)
            H.oracle_step_rows(g.cpu().numpy(), xo, eo, "sign", "sign", lr)
        s.synchronize()
    assert H.bit_equal(x.cpu().numpy(), xo) and H.bit_equal(e.cpu().numpy(), eo)


def test_step_rejects_bad_buffers_and_reports_nonfinite_input():
    say("case errors")
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
        with pytest.raises(LiecError):
            ctx.set_group_bitmap(1)                  # the workers' operator is not top-k
        with pytest.raises(LiecError):
            ctx.set_search_wait(-1)
    with LiecContext(N, d, "topk", "sign", 10, 0, 0.1) as ctx:
        with pytest.raises(LiecError):
            ctx.set_group_bitmap(2)
        ctx.set_group_bitmap(1)
        x.zero_(), e.zero_()
        g[1, 17] = float("nan")
        ctx.step(g, x, e)
        assert ctx.info_status()[1] == 4


def test_two_contexts_on_two_streams_do_not_interfere():
    """The library keeps no global state: two contexts with different operators, sizes and streams,
    stepping in turns without synchronising in between, give what each gives alone."""
    say("case two contexts")
    wa = workloads.scaled(WL["c2_topk_mid"], N=4, d=150_000, worker_comp="topk", server_comp="sign", worker_k=1500)
    wb = workloads.scaled(WL["c2_topk_mid"], N=3, d=90_001, worker_comp="randk", server_comp="topk", worker_k=900, server_k=2000)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    srcs = [workloads.GradientSource(w, seed=5 + q, device=DEV) for q, w in enumerate((wa, wb))]
    gs = [[src.grads(t) for t in range(4)] for src in srcs]
    xs = [torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV) for w in (wa, wb)]
    es = [torch.zeros(w.d, dtype=torch.float32, device=DEV) for w in (wa, wb)]
    torch.cuda.synchronize()
    with ctx_for(wa, stream=sa) as ca, ctx_for(wb, stream=sb) as cb:
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
    say("case out of memory")
    from paper_2402_11857_amd import LiecContext, LiecError

    with pytest.raises(LiecError) as err:          # the candidate lists alone would take about 1 TB
        LiecContext(1000, 2_000_000_000, "topk", "topk", 100_000_000, 100_000_000, 0.1)
    assert err.value.status == 2
    w = workloads.scaled(WL["c1_tiny_sign"], N=2, d=5000)
    assert run_chain(w, steps=2, seed=1)


def test_per_kernel_timing_and_scratch_accounting():
    say("case profile api")
    w = workloads.scaled(WL["c2_topk_mid"], N=4, d=200_000, worker_comp="topk", server_comp="sign", worker_k=2000)
    g = workloads.GradientSource(w, seed=1, device=DEV).grads(0)
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=DEV)
    e = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    with ctx_for(w) as ctx:
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
