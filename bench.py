#!/usr/bin/env python3
"""Throughput of the LIEC-SGD compressed step on one MI355X.

A "step" is one pass of the whole hot path (worker compression, server compensation and
recompression, error update, broadcast + local immediate compensation + model update) over one
[N, d] batch of synthetic gradients that is already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak
DEFAULT_WORKLOAD = "c5_vgg16_mixed"   # the largest configuration; fits one GPU (grads 8.25 GiB)
ALSO = ["c3_resnet18_sign", "c3_resnet18_blocksign", "c4_resnet50_topk", "c4_resnet50_randk", "c5_vgg16_sign",
        "c1_tiny_sign", "c2_topk_mid"]
# small configurations whose tensors fit the caches and whose step is a chain of short dependent kernels
CACHE_RESIDENT = {"c1_tiny_sign": "1 MiB of gradients: cache-resident, bound by the gaps between 5 dependent kernels",
                  "c2_topk_mid": "32 MiB of gradients: cache-resident, bound by the gaps between 20 dependent kernels"}
N_GRAD_BUFFERS = 4          # distinct gradient batches rotated through the timed steps
REPEATS = 5                 # timed regions per workload; the median one is reported
# kernels that make up a steady-state step (the rest of a profile summary -- cold and general search,
# averaging iteration, wire forms, copy probe -- is not part of it)
STEADY_STATE_KERNELS = ("k_update", "k_filter", "k_aggregate", "k_l1_bits", "k_l1_final", "k_l1_items", "k_list_",
                        "k_rk_zero", "k_rk_filter_inverse", "k_rk_mark", "k_rk_advance")


def profile_traffic(workload: str):
    """HBM bytes per launch of the update kernel and per steady-state step, read from the rocprofv3 counter
    summary of this script's own run on that workload (profiles/liec_step_<workload>.md: FETCH_SIZE and
    WRITE_SIZE, each scaled by what it reads for the 1 GiB copy probe).  (None, None) without a summary."""
    path = os.path.join(ROOT, "profiles", f"liec_step_{workload}.md")
    if not os.path.exists(path):
        return None, None
    update = step = None
    in_table = False
    for line in open(path):
        if line.startswith("## HBM traffic counters"):
            in_table = True
            continue
        if not in_table or not line.startswith("| liec::"):
            continue
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        name, read_gb, write_gb = cells[0].replace("liec::", ""), float(cells[2]), float(cells[4])
        if not name.startswith(STEADY_STATE_KERNELS):
            continue
        total = (read_gb + write_gb) * 1e9
        step = (step or 0.0) + total
        if name.startswith("k_update"):
            update = total
    return update, step


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def dominant_kernel_bytes(w) -> int:
    """Algorithmic bytes of one launch of the update kernel: grads and x read, x written
    (12 B per gradient element) plus v read and e written (8 B per column)."""
    return 12 * w.N * w.d + 8 * w.d


def run_workload(w, steps: int, warmup: int, seed: int = 0, steady_only: bool = False):
    import torch

    import workloads
    from paper_2402_11857_amd import LiecContext

    dev = "cuda:0"
    src = workloads.GradientSource(w, seed=seed, device=dev)
    nbuf = min(N_GRAD_BUFFERS, max(1, steps + warmup))
    grads = [src.grads(t) for t in range(nbuf)]
    x = torch.zeros((w.N, w.d), dtype=torch.float32, device=dev)
    e = torch.zeros(w.d, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    with LiecContext(w.N, w.d, w.worker_comp, w.server_comp, w.worker_k, w.server_k, w.lr) as ctx:
        if w.blocks is not None:
            ctx.set_blocks(w.blocks)
        for t in range(warmup):
            ctx.step(grads[t % nbuf], x, e)
        torch.cuda.synchronize()
        # REPEATS timed regions of exactly `steps` steps each; the median region is reported
        regions = []
        for rep in range(REPEATS):
            torch.cuda.synchronize()
            ctx.profile_begin(steps, update_only=True)   # HIP events around the dominant kernel, on the step's stream
            t0 = time.perf_counter()
            for t in range(steps):
                ctx.step(grads[(warmup + t) % nbuf], x, e)
            torch.cuda.synchronize()
            el = time.perf_counter() - t0
            regions.append((el, ctx.profile_end()["update"]))
        regions.sort(key=lambda r: r[0])
        elapsed, (upd_ms, upd_n) = regions[len(regions) // 2]
        info, status = ctx.info_status()
        assert status == 0, "non-finite values met during the bench"
        band_misses = int(info.band_misses)      # row-steps of warm-up + timed regions whose predicted band failed
        # diagnostic breakdown, outside the timed region: every kernel bracketed by events
        nb = min(steps, 10)
        ctx.profile_begin(nb)
        for t in range(nb):
            ctx.step(grads[t % nbuf], x, e)
        kernels = {k: (v[0] / nb, v[1]) for k, v in ctx.profile_end().items()}
        sync_ms, wire, worst = float("nan"), None, None
        if not steady_only:
            # the averaging iteration of Algorithm 1 (one in every `period` steps), timed on its own
            ns = 5
            ctx.step_sync(grads[0], x, e)
            ctx.profile_begin(ns)
            for t in range(ns):
                ctx.step_sync(grads[t % nbuf], x, e)
            sync_ms = ctx.profile_end()["sync"][0] / ns
            wire = time_wire_forms(ctx, w, grads[0], x, e)
            worst = time_worst_case_steps(ctx, w, grads, x, e)
        scratch = ctx.scratch_bytes()
    ms_per_step = 1e3 * elapsed / steps
    out = {
        "ms_per_step": ms_per_step,
        "elems_per_s": w.N * w.d * steps / elapsed,
        "alg_gbps": w.alg_bytes_per_step * steps / elapsed / 1e9,
        "kernels_ms_per_step": {k: v[0] for k, v in kernels.items()},
        "scratch_bytes": scratch,
        "region_ms_per_step": [round(1e3 * r[0] / steps, 4) for r in regions],
        "sync_ms": sync_ms,
        "wire": wire,
        "worst": worst,
        "band_misses": band_misses,
        "sync_gbps": dominant_kernel_bytes(w) / (sync_ms * 1e-3) / 1e9,   # same bytes: g, x in, x out, e in/out
    }
    out["update_avg_ms"] = upd_ms / upd_n
    out["update_gbps"] = dominant_kernel_bytes(w) / (upd_ms / upd_n * 1e-3) / 1e9
    del grads, x, e
    torch.cuda.empty_cache()
    return out


def time_worst_case_steps(ctx, w, grads, x, e, reps: int = 3):
    """Single steps outside the steady state, each timed by events on the step's stream (median of `reps`):
    `cold` -- no threshold prediction at all (what the first step of a context pays): every top-k row takes
    the first-digit histogram and a second filter pass; `failed_prediction` -- the gradients' scale jumps
    by 30 between two steps, so the band predicted from the last thresholds misses and the same two extra
    passes run after the wasted one.  Operators without a threshold search have no such cases."""
    import torch

    if "topk" not in (w.worker_comp, w.server_comp):
        return None
    alg = w.alg_bytes_per_step

    def timed_step(g):
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        ctx.step(g, x, e)
        stop.record()
        torch.cuda.synchronize()
        return start.elapsed_time(stop)

    def entry(ms_list):
        ms = sorted(ms_list)[len(ms_list) // 2]
        return {"ms": round(ms, 4), "hbm_frac": round(alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "all_ms": [round(m, 4) for m in ms_list]}

    cold = []
    for r in range(reps):
        ctx.step(grads[r % len(grads)], x, e)
        ctx.force_search_mode(1)                  # no prediction: as in the first step of a context
        cold.append(timed_step(grads[(r + 1) % len(grads)]))
    big = grads[0] * 30.0
    failed = []
    for r in range(reps):
        for q in range(3):                         # settle the prediction on the unscaled gradients
            ctx.step(grads[q % len(grads)], x, e)
        failed.append(timed_step(big))
    slow_rows = ctx.info().slow_rows
    del big
    return {"cold_step": entry(cold), "failed_prediction_step": entry(failed),
            "rows_in_general_search_after": slow_rows,
            "note": "single steps timed by events; value and roofline are the steady state, in which every row's "
                    "predicted band holds"}


def time_wire_forms(ctx, w, g, x, e, reps: int = 5):
    """Worker 0's uplink message of one more step put into its wire form and decompressed again (the step
    itself never materialises messages); events on the null stream, which the context uses here."""
    import torch

    from paper_2402_11857_amd import liec_message_bytes

    if w.worker_comp == "identity":
        return None
    ctx.step(g, x, e)
    p_out = torch.empty(w.d, dtype=torch.float32, device=g.device)
    nblocks = len(w.blocks) - 1 if w.blocks is not None else 0
    if w.worker_comp in ("sign", "blocksign"):
        bits = torch.empty((w.d + 7) // 8, dtype=torch.uint8, device=g.device)
        blockwise = w.worker_comp == "blocksign"
        scales = ctx.block_scales()[0][0] if blockwise else [ctx.worker_desc()["scale"][0]]
        pack = lambda: ctx.pack_sign_bits(0, bits)                                    # noqa: E731
        unpack = lambda: ctx.unpack_sign_message(bits, scales, blockwise, p_out)     # noqa: E731
    else:
        idx = torch.empty(w.worker_k, dtype=torch.int32, device=g.device)
        val = torch.empty(w.worker_k, dtype=torch.float32, device=g.device)
        pack = lambda: ctx.pack_topk_message(g, 0, idx, val)                          # noqa: E731
        unpack = lambda: ctx.unpack_topk_message(idx, val, p_out)                    # noqa: E731
    out = {"message_bytes": liec_message_bytes(w.worker_comp, w.d, w.worker_k, nblocks), "dense_bytes": 4 * w.d}
    for name, fn in (("pack_ms", pack), ("unpack_ms", unpack)):
        fn()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(reps):
            fn()
        stop.record()
        torch.cuda.synchronize()
        out[name] = round(start.elapsed_time(stop) / reps, 4)
    return out


def copy_ceiling_gbps(nbytes: int = 1 << 30, reps: int = 10) -> float:
    """Bytes read + written per second by a plain 128-bit device copy kernel."""
    import torch

    from paper_2402_11857_amd import device_copy

    a = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0").normal_()
    b = torch.empty_like(a)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(2):
        device_copy(b, a, stream)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        device_copy(b, a, stream)
    stop.record()
    torch.cuda.synchronize()
    ms = start.elapsed_time(stop) / reps
    return 2 * nbytes / (ms * 1e-3) / 1e9


def cpu_baseline(w, seed: int = 0):
    """The CPU oracle as it stands.  `value`: one host thread, one step at the benched configuration's full
    row length with N cut to one worker (the oracle's top-k is a full sort, so elements per second depend on
    d; they do not depend on N).  Beside it, labelled: a 2^21-column slice at full N on one thread, and the
    same slice through the -fopenmp build of the same source (workers of a step on all host threads)."""
    import numpy as np

    import oracle
    import workloads

    oracle.build()

    def run(ws, step_fn, budget_s, max_steps):
        g = workloads.GradientSource(ws, seed=seed, device="cpu").grads(0).numpy()
        x = np.zeros((ws.N, ws.d), dtype=np.float32)
        e = np.zeros(ws.d, dtype=np.float32)
        steps, threads, t0 = 0, 1, time.perf_counter()
        while True:
            r = step_fn(g, x, e, ws.worker_comp, ws.server_comp, ws.lr, ws.worker_k, ws.server_k)
            threads = r if isinstance(r, int) else 1
            steps += 1
            el = time.perf_counter() - t0
            if el > budget_s or steps >= max_steps:
                return ws.N * ws.d * steps / el, steps, el, threads

    full = workloads.scaled(w, N=1, worker_k=w.worker_k, server_k=w.server_k)
    v, steps, el, _ = run(full, oracle.step, 0.0, 1)
    out = {"value": v, "unit": "elems/s", "cores": 1, "kind": "oracle",
           "sample": f"{steps} step of the benched recipe at its full row length d={full.d} with N cut to 1 worker "
                     f"(k unchanged), {el:.1f} s of one host thread"}
    ws = workloads.scaled(w, d=min(w.d, 1 << 21))
    v, steps, el, _ = run(ws, oracle.step, 8.0, 50)
    out["column_slice"] = {"value": v, "unit": "elems/s", "cores": 1,
                           "sample": f"SLICE, not the benched size: {steps} step(s) at N={ws.N}, d={ws.d} columns "
                                     f"(k scaled with d), {el:.1f} s of one host thread"}
    v, steps, el, threads = run(ws, oracle.step_all_cores, 5.0, 50)
    out["all_host_cores"] = {"value": v, "unit": "elems/s", "threads": threads,
                             "sample": f"SLICE: the same {ws.N} x {ws.d} slice, {steps} step(s) in {el:.1f} s through the "
                                       "-fopenmp build of the same source (the workers of a step on separate threads, "
                                       "the server on one); its output is checked bit for bit against the one-thread "
                                       "build by tests/test_oracle_step.py"}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--steady-only", action="store_true",
                    help="skip the steps outside the steady state, the averaging iteration and the wire forms "
                         "(for profiler runs: every launch after the first step is then a steady-state one)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the N workers are a batch axis on a single MI355X; "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU path)", file=sys.stderr)
        return 2
    import workloads

    wl = workloads.workloads()
    w = wl[args.workload]
    torch.cuda.set_device(0)
    log(f"workload {w.name}: N={w.N} d={w.d} {w.worker_comp}/{w.server_comp}")
    copy_gbps = copy_ceiling_gbps()
    log(f"copy kernel ceiling {copy_gbps:.0f} GB/s")
    main_res = run_workload(w, args.steps, args.warmup, steady_only=args.steady_only)
    log(f"{w.name}: {main_res['ms_per_step']:.3f} ms/step, {main_res['alg_gbps']:.0f} GB/s algorithmic")
    also = {}
    if not args.no_also:
        for name in ALSO:
            if name == w.name:
                continue
            r = run_workload(wl[name], args.steps, args.warmup)
            also[name] = {"ms_per_step": round(r["ms_per_step"], 4), "elems_per_s": r["elems_per_s"],
                          "alg_gbps": round(r["alg_gbps"], 1), "hbm_frac": round(r["alg_gbps"] / HBM_PEAK_GBPS, 4),
                          "update_gbps": round(r["update_gbps"], 1),
                          "averaging_iteration_ms": round(r["sync_ms"], 4),
                          "wire_worker0": r["wire"],
                          "outside_steady_state": r["worst"],
                          "band_misses_in_warmup_and_timed_regions": r["band_misses"],
                          "kernels_ms_per_step": {k: round(v, 4) for k, v in r["kernels_ms_per_step"].items()}}
            if name in CACHE_RESIDENT:
                also[name]["note"] = CACHE_RESIDENT[name]
            log(f"{name}: {r['ms_per_step']:.3f} ms/step, {r['alg_gbps']:.0f} GB/s algorithmic")
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w)
        log(f"cpu oracle: {cpu['value']:.3e} elems/s on {cpu['cores']} core")

    line = {
        "metric": "LIEC step gradient elems/s (N*d)",
        "value": main_res["elems_per_s"],
        "unit": "elems/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "N": w.N, "d": w.d, "worker_comp": w.worker_comp,
                   "server_comp": w.server_comp, "worker_k": w.worker_k, "server_k": w.server_k,
                   "lr": w.lr, "grad_buffers_rotated": N_GRAD_BUFFERS},
        "timed_regions_ms_per_step": main_res["region_ms_per_step"],
        "step_alg_bytes": w.alg_bytes_per_step,
        "step_alg_gbps": main_res["alg_gbps"],
        "step_hbm_frac": main_res["alg_gbps"] / HBM_PEAK_GBPS,
        "step_traffic_bytes": profile_traffic(w.name)[1],
        "traffic_source": f"profiles/liec_step_{w.name}.md",
        "copy_kernel_gbps": copy_gbps,
        "roofline": {"bound": "hbm", "kernel": "update", "achieved": main_res["update_gbps"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": main_res["update_gbps"] / HBM_PEAK_GBPS,
                     "traffic": profile_traffic(w.name)[0], "alg_bytes_per_launch": dominant_kernel_bytes(w),
                     "avg_launch_ms": main_res["update_avg_ms"]},
        "kernels_ms_per_step_untimed_pass": {k: round(v, 4) for k, v in main_res["kernels_ms_per_step"].items()},
        "scratch_bytes": main_res["scratch_bytes"],
        "wire_worker0": main_res["wire"],
        "outside_steady_state": main_res["worst"],
        "band_misses_in_warmup_and_timed_regions": main_res["band_misses"],
        "averaging_iteration": None if args.steady_only else
                               {"ms": round(main_res["sync_ms"], 4), "alg_gbps": round(main_res["sync_gbps"], 1),
                                "note": "Algorithm 1's uncompressed iteration, one in every `period` steps; not part of value"},
        # Algorithm 1 as a whole with the averaging periods of the paper's experiments, from the two measured times
        "algorithm1_ms_per_iteration": None if args.steady_only else
                                       {f"period_{h}": round(((h - 1) * main_res["ms_per_step"] + main_res["sync_ms"]) / h, 4)
                                        for h in (32, 100)},
        "also": also,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
