"""Wire forms of the compressed messages on the GPU against the oracle.
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


# ---- wire form of the sign messages ----------------------------------------------------------------
@pytest.mark.parametrize("comp", ["sign", "blocksign"])
@pytest.mark.parametrize("N,d", [(2, 8), (3, 1001), (4, 70_003), (2, 262_144)])
def test_sign_message_wire_form_round_trip(N, d, comp):
    say(f"case wire N={N} d={d} {comp}")
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
    say(f"case wire topk N={N} d={d} k={k}")
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


def test_wire_scratch_survives_a_sign_unpack_between_two_topk_packs():
    say("case wire scratch reuse")
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
