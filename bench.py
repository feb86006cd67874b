#!/usr/bin/env python3
"""Benchmark of the Sync EASGD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1|cfg2|cfg3|cfg4|cfg5]

A step is one whole Sync EASGD round over one batch of synthetic input that is
already resident in HBM: one `easgd_mlp_round` call (the gradients of all P
workers with the elastic update fused into backward propagation).  The same
rounds are also timed through the two-call path, `easgd_grad` followed by
`easgd_sync_round` (`measgd_round` for momentum workloads), which isolates the
matrix-product kernels for the MFMA roofline.  For the update-only workloads
cfg4/cfg5 a step is the elastic update alone.
The default workload is cfg2 (MLP 784-1024-1024-10, P=16, b=128); the default
run also times the other two training workloads (cfg1, cfg3; "training_workloads"
in the JSON line), measures the elastic update at AlexNet size (cfg4, cfg5; with
fp32 and with bfloat16-stored gradients and momentum buffers, the latter an
extension) and the synchronous SGD round ("elastic_update"), and times the CPU
oracle on the host cores for every workload.

Every GPU leg starts with an untimed pre-roll of the same calls (at least
PREROLL_MIN_S, until two consecutive blocks of rounds agree within 2 %): the
first milliseconds of a process run at start-up clocks and with cold code, and
a timed region of a few milliseconds would otherwise measure those.  Then
`warmup` untimed rounds, then exactly `steps` timed rounds.

Prints ONE JSON line.  Kernel-phase durations are measured with HIP events on
the stream the kernels are launched on.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix, published

DESCRIPTIONS = {
    "cfg1": "cfg1: softmax regression 784-10, P=4 workers, batch 64 each, Sync EASGD",
    "cfg2": "cfg2: MLP 784-1024-1024-10 ReLU, P=16 workers, batch 128 each, Sync EASGD",
    "cfg3": "cfg3: MLP 3072-2048-2048-10 ReLU, P=32 workers, batch 100 each, Sync MEASGD (momentum 0.9)",
    "cfg4": "cfg4: elastic update only, P=8 replicas x 61M fp32 parameters, Sync EASGD",
    "cfg5": "cfg5: elastic update only, P=16 replicas x 61M fp32 parameters, Sync MEASGD (momentum 0.9)",
}


def update_bytes(wl) -> int:
    """Algorithmic HBM bytes of one elastic update: per worker element read W, G (and V), write W (and V);
    per center element one read and one write."""
    per_worker = 20 if wl.momentum else 12
    return wl.N * (per_worker * wl.P + 8)


def grad_flops(wl) -> int:
    """Useful flops of one easgd_grad call: forward, weight-gradient and input-gradient products."""
    total = 0
    for l in range(len(wl.dims) - 1):
        mnk = wl.batch * wl.dims[l] * wl.dims[l + 1]
        total += 2 * mnk * (3 if l > 0 else 2)
    return total * wl.P


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _sum_ms(starts, stops):
    return float(sum(a.elapsed_time(b) for a, b in zip(starts, stops)))


UPDATE_LD_ALIGN = 256          # elements: replica rows of the update-only workloads start on 1 KiB boundaries
TRAINING_LD_ALIGN = 256        # the same for the training workloads' replicas (cfg3: 2.63 -> 2.44 ms per round)
PREROLL_MIN_S = 0.25
PREROLL_MAX_S = 2.0


def preroll(step, block, first=0):
    """Untimed rounds ahead of a measurement: blocks of `block` calls of step(t) until at least PREROLL_MIN_S
    have passed and two consecutive blocks take the same time within 2 % (or PREROLL_MAX_S have passed).
    Returns (number of calls made, report)."""
    import torch
    t, prev, stable = first, None, False
    torch.cuda.synchronize()
    start = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        for _ in range(block):
            step(t)
            t += 1
        torch.cuda.synchronize()
        now = time.perf_counter()
        dt = now - t0
        if prev is not None and now - start >= PREROLL_MIN_S and abs(dt - prev) <= 0.02 * min(dt, prev):
            stable = True
            break
        if now - start >= PREROLL_MAX_S:
            break
        prev = dt
    return t - first, {"preroll_s": round(time.perf_counter() - start, 3), "preroll_rounds": t - first,
                       "preroll_stable": stable}


# ---------------------------------------------------------------------------
# GPU legs
# ---------------------------------------------------------------------------

def bench_training(hip, wl, steps, warmup, one_call=True, v_bf16=False, g_bf16=False):
    """v_bf16: momentum buffers stored as bfloat16 (an extension; momentum workloads only); g_bf16: the two-call
    path with the gradients stored as bfloat16 too (momentum workloads: together with v_bf16)."""
    import torch
    ld = workloads.round_up(wl.N, TRAINING_LD_ALIGN)
    w0 = workloads.init_packed_weights(wl)
    dW = torch.from_numpy(workloads.replicate(w0, wl.P, ld)).cuda()
    dWc = torch.from_numpy(w0.copy()).cuda()
    dV = torch.zeros_like(dW) if wl.momentum else None
    if v_bf16:
        dV = torch.zeros(dW.shape, dtype=torch.bfloat16, device="cuda")
    dG = torch.zeros(dW.shape, dtype=torch.bfloat16, device="cuda") if g_bf16 else torch.zeros_like(dW)
    n_batches = min(wl.rounds, 16)
    batches = []
    for t in range(n_batches):
        X, y = workloads.minibatch(wl, t)
        batches.append((torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()))
    ws = torch.empty(hip.easgd_mlp_round_workspace_bytes(wl.dims, wl.P, wl.batch), dtype=torch.uint8, device="cuda")

    def step(t, ev=None):
        X, y = batches[t % n_batches]
        if ev:
            ev[0].record()
        if one_call:
            hip.easgd_mlp_round(wl.dims, dW, dWc, X, y, wl.eta, wl.rho, V=dV, delta=wl.delta or 0.0, workspace=ws)
            if ev:
                ev[1].record()
                ev[2].record()
            return
        hip.easgd_grad(wl.dims, dW, X, y, dG, None, workspace=ws)
        if ev:
            ev[1].record()
        if g_bf16 and wl.momentum:
            hip.measgd_round_bf16(dW, dV, dG, dWc, wl.eta, wl.rho, wl.delta, N=wl.N)
        elif g_bf16:
            hip.easgd_sync_round_bf16(dW, dG, dWc, wl.eta, wl.rho, N=wl.N)
        elif v_bf16:
            hip.measgd_round_bf16v(dW, dV, dG, dWc, wl.eta, wl.rho, wl.delta, N=wl.N)
        elif wl.momentum:
            hip.measgd_round(dW, dV, dG, dWc, wl.eta, wl.rho, wl.delta, N=wl.N)
        else:
            hip.easgd_sync_round(dW, dG, dWc, wl.eta, wl.rho, N=wl.N)
        if ev:
            ev[2].record()

    done, pre = preroll(step, max(steps, 20))
    for t in range(warmup):
        step(done + t)
    # the timed region: exactly `steps` rounds, nothing but the library calls between the two synchronisations
    torch.cuda.synchronize()
    c0 = hip.launch_count()
    t0 = time.perf_counter()
    for t in range(steps):
        step(done + warmup + t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    launches = (hip.launch_count() - c0) / steps
    # a second, instrumented pass gives the duration of each phase from HIP events recorded on the launch stream
    # (recording them costs some microseconds per round, so it stays out of the timed region); at least 50 rounds,
    # so that the average does not hang on a handful of launches
    n_ev = max(steps, 50)
    e0, e1, e2 = _events(n_ev), _events(n_ev), _events(n_ev)
    for t in range(n_ev):
        step(done + warmup + steps + t, (e0[t], e1[t], e2[t]))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dWc).all()), "center weights diverged"
    grad_ms = _sum_ms(e0, e1) / n_ev
    upd_ms = _sum_ms(e1, e2) / n_ev
    return {"elapsed_s": elapsed, "ms_per_step": 1e3 * elapsed / steps, "grad_ms": grad_ms, "update_ms": upd_ms,
            "launches_per_round": launches, "event_rounds": n_ev, **pre}


def bench_host_fed(hip, wl, steps, warmup, group=1):
    """Whole rounds whose minibatches come from pinned host memory: the copy of round t+1 overlaps round t
    (the overlap of Sync EASGD3, Algorithm 3), two device buffers.  group = g > 1: one copy brings the minibatches
    of g rounds and overlaps the g rounds before them."""
    import torch
    steps, warmup = (steps + group - 1) // group * group, (warmup + group - 1) // group * group
    ld = workloads.round_up(wl.N, TRAINING_LD_ALIGN)
    w0 = workloads.init_packed_weights(wl)
    dW = torch.from_numpy(workloads.replicate(w0, wl.P, ld)).cuda()
    dWc = torch.from_numpy(w0.copy()).cuda()
    dV = torch.zeros_like(dW) if wl.momentum else None
    n_batches = min(wl.rounds, 16)
    n_batches = (n_batches + group - 1) // group * group
    new_feeder = lambda: hip.BatchFeeder(wl.P, wl.batch, wl.dims[0], rounds_per_copy=group)
    host = []
    layout = new_feeder()                # its host_batch(): samples and labels back to back, one copy
    for t0 in range(0, n_batches, group):
        hX, hy = layout.host_batch()
        for i in range(group):
            X, y = workloads.minibatch(wl, t0 + i)
            (hX[i] if group > 1 else hX).copy_(torch.from_numpy(X)); (hy[i] if group > 1 else hy).copy_(torch.from_numpy(y))
        host.append((hX, hy))
    del layout
    bytes_per_round = (host[0][0].numel() * 4 + host[0][1].numel() * 4) // group
    ws = torch.empty(hip.easgd_mlp_round_workspace_bytes(wl.dims, wl.P, wl.batch), dtype=torch.uint8, device="cuda")
    def run(feeder, first, count, primed=False):       # first and count are multiples of group
        # leaves the copy for the round after its last one in flight, so that a run that continues where this one
        # ended (primed=True) starts with a full pipeline: the timed region then holds no start-up copy that
        # nothing overlaps
        k0, kn = first // group, count // group
        if not primed:
            feeder.submit(k0 % 2, *host[k0 % len(host)])
        for k in range(k0, k0 + kn):
            feeder.submit((k + 1) % 2, *host[(k + 1) % len(host)])
            X, y = feeder.acquire(k % 2)
            for i in range(group):
                hip.easgd_mlp_round(wl.dims, dW, dWc, X[i] if group > 1 else X, y[i] if group > 1 else y, wl.eta, wl.rho,
                                    V=dV, delta=wl.delta or 0.0, workspace=ws)
            feeder.release(k % 2)

    # Measured on this device: the copy overlaps the round only when the round runs on a stream of its own
    # (not the default stream) and the library keeps to that one stream (the center rule on extra blocks of a
    # forward launch, never on the library's second stream); with three streams tied by events the copy and
    # the round serialise.  HIP also
    # multiplexes streams onto a few hardware queues (4 per process here), and a copy stream and a compute
    # stream that share a queue run one after the other: short trials pick a pair of streams that does not.
    old = hip.get_option(hip.OPT_ROUND_OVERLAP)
    hip.set_option(hip.OPT_ROUND_OVERLAP, 3)
    try:
        best, done = None, 0
        # the host link and its copy engines take a while to reach their rate after start-up: the first fed
        # loop of a process runs 25 % slower than any later one, so about a second of untimed fed rounds goes first
        feeder, cand = new_feeder(), torch.cuda.Stream()
        with torch.cuda.stream(cand):
            t_warm = time.perf_counter()
            while time.perf_counter() - t_warm < 1.0:
                run(feeder, done, 100)
                torch.cuda.synchronize()
                done += 100
        for _ in range(6):
            feeder, cand = new_feeder(), torch.cuda.Stream()
            with torch.cuda.stream(cand):
                run(feeder, done, warmup)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                run(feeder, done + warmup, 32, primed=True)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
            done += warmup + 32
            if best is None or dt < best[0]:
                best = (dt, feeder, cand)
        with torch.cuda.stream(best[2]):
            run(best[1], done, warmup)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(best[1], done + warmup, steps, primed=True)
            torch.cuda.synchronize()
            elapsed = time.perf_counter() - t0
    finally:
        hip.set_option(hip.OPT_ROUND_OVERLAP, old)
    assert bool(torch.isfinite(dWc).all()), "center weights diverged"
    return {"rounds_per_s": round(steps / elapsed, 2), "ms_per_step": round(1e3 * elapsed / steps, 4),
            "host_bytes_per_round": bytes_per_round,
            "host_GBs": round(bytes_per_round * steps / elapsed / 1e9, 2),
            "rounds_per_copy": group, "steps": steps,
            "note": "minibatches copied from pinned host memory, the copy of the next round(s) overlapping the "
                    "current one(s); rounds on a non-default stream, library on one stream"}


def bench_update_only(hip, wl, steps, warmup, pool=3, rule="elastic"):
    """rule = "elastic": the workload's EASGD / MEASGD update; "sync_sgd": the synchronous data-parallel SGD
    round on the same replicas and gradients (every replica moves by the gradient sum); "elastic_bf16": the
    workload's update with gradients and momentum buffers stored as bfloat16 (an extension); "async": the master
    serving the workers one at a time in rank order (Algorithm 1), one launch per sweep over the workers;
    "hogwild": all workers exchanging with the center at once, lock-free (Hogwild EASGD)."""
    import torch
    P, N = wl.P, wl.N
    # replica rows start on 1 KiB boundaries (ld = N rounded up to 256 elements; the padding is never touched): the
    # kernels' 1 KiB pieces then coincide with aligned KiB of every row, worth 2-4 % over ld = N
    ld = workloads.round_up(N, UPDATE_LD_ALIGN)
    dW = workloads.device_normal((P, ld), workloads.WEIGHT_STD, workloads.DEFAULT_SEED, 1)
    dWc = workloads.device_normal((N,), workloads.WEIGHT_STD, workloads.DEFAULT_SEED, 2)
    dV = torch.zeros_like(dW) if wl.momentum else None
    # gradients of consecutive rounds: a small pool of independent draws, cycled (footprint >> caches)
    Gs = [workloads.device_normal((P, ld), workloads.GRADIENT_STD, workloads.DEFAULT_SEED, 100 + t) for t in range(pool)]
    if rule == "elastic_bf16":
        Gs = [g.to(torch.bfloat16) for g in Gs]
        dV = torch.zeros((P, ld), dtype=torch.bfloat16, device="cuda") if wl.momentum else None

    rank_order = list(range(P))

    def step(t):
        if rule == "elastic_bf16" and wl.momentum:
            hip.measgd_round_bf16(dW, dV, Gs[t % pool], dWc, wl.eta, wl.rho, wl.delta, N=N)
        elif rule == "elastic_bf16":
            hip.easgd_sync_round_bf16(dW, Gs[t % pool], dWc, wl.eta, wl.rho, N=N)
        elif rule == "sync_sgd":
            hip.sync_sgd_round(dW, Gs[t % pool], wl.eta / P, V=dV, delta=wl.delta or 0.0, N=N)
        elif rule == "async":
            hip.async_easgd_round(dW, Gs[t % pool], dWc, rank_order, wl.eta, wl.rho, V=dV, delta=wl.delta or 0.0, N=N)
        elif rule == "hogwild":
            hip.hogwild_easgd_round(dW, Gs[t % pool], dWc, wl.eta, wl.rho, V=dV, delta=wl.delta or 0.0, N=N)
        elif wl.momentum:
            hip.measgd_round(dW, dV, Gs[t % pool], dWc, wl.eta, wl.rho, wl.delta, N=N)
        else:
            hip.easgd_sync_round(dW, Gs[t % pool], dWc, wl.eta, wl.rho, N=N)

    done, pre = preroll(step, 20)
    for t in range(warmup):
        step(done + t)
    e0, e1 = _events(steps), _events(steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        e0[t].record()
        step(done + warmup + t)
        e1[t].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert bool(torch.isfinite(dWc).all()) and bool(torch.isfinite(dW[0, :4096]).all())
    kernel_ms = _sum_ms(e0, e1) / steps
    return {"elapsed_s": elapsed, "ms_per_step": 1e3 * elapsed / steps, "update_ms": kernel_ms, **pre}


def triad_ceiling(hip, n=488_000_000, reps=20):
    """Attainable HBM bandwidth of this device for a 2-read/1-write stream (GB/s)."""
    import torch
    a = torch.empty(n, dtype=torch.float32, device="cuda")
    b = torch.ones_like(a)
    c = torch.ones_like(a)
    for _ in range(3):
        hip.stream_triad(a, b, c, 0.5)
    e0, e1 = _events(1)[0], _events(1)[0]
    e0.record()
    for _ in range(reps):
        hip.stream_triad(a, b, c, 0.5)
    e1.record()
    torch.cuda.synchronize()
    return 12.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9




# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by the reading
# of the same counter for the triad kernel of known traffic (x2.000 and x1.000).  They are counter readings of an
# earlier profiling session, not of this run: each entry names the summary under profiles/ it comes from, and all of
# them are dropped from the JSON line (traffic: null) when the running library reports another version than the one
# that was profiled, or non-default launch options.
TRAFFIC_PROFILES = {
    ("elastic", False, 8, 61_000_000): (2_025_433.1 * 1024 * 2.000 + 2_144_531.5 * 1024 * 1.000,
                                        "profiles/elastic_update_cfg4_cfg5_hbm_traffic.md"),
    ("elastic", True, 16, 61_000_000): (5_837_957.8 * 1024 * 2.000 + 7_863_310.1 * 1024 * 1.000,
                                        "profiles/elastic_update_cfg4_cfg5_hbm_traffic.md"),
    ("sync_sgd", False, 8, 61_000_000): (1_906_280.9 * 1024 * 2.000 + 1_906_253.1 * 1024 * 1.000,
                                         "profiles/elastic_update_cfg4_cfg5_hbm_traffic.md"),
    ("async", False, 8, 61_000_000): (2_025_431.3 * 1024 * 2.000 + 2_144_531.3 * 1024 * 1.000,
                                      "profiles/elastic_update_cfg4_cfg5_hbm_traffic.md"),
    ("hogwild", False, 8, 61_000_000): (2_868_972.1 * 1024 * 2.000 + 9_531_250.0 * 1024 * 1.000,
                                        "profiles/elastic_update_cfg4_cfg5_hbm_traffic.md"),
    ("elastic_bf16", False, 8, 61_000_000): (1_548_869.4 * 1024 * 2.000 + 2_144_531.7 * 1024 * 1.000,
                                             "profiles/elastic_update_cfg4_cfg5_hbm_traffic.md"),
    ("elastic_bf16", True, 16, 61_000_000): (3_931_724.0 * 1024 * 2.000 + 5_957_033.4 * 1024 * 1.000,
                                             "profiles/elastic_update_cfg4_cfg5_hbm_traffic.md"),
    ("grad", "cfg2"): (131_056.1 * 1024 * 2.000 + 149_337.0 * 1024 * 1.000, "profiles/easgd_grad_cfg2_hbm_traffic.md"),
}
TRAFFIC_PROFILED_VERSION = 500      # easgd_version() of the library the summaries above were taken with


def traffic_fields(hip, key):
    """`traffic` (bytes per launch) and its provenance for a roofline object; None when the profile is stale."""
    entry = TRAFFIC_PROFILES.get(key)
    default_opts = (hip.get_option(hip.OPT_UPDATE_GROUPS) == 0 and hip.get_option(hip.OPT_UPDATE_LAYOUT) == 2
                    and hip.get_option(hip.OPT_UPDATE_NONTEMPORAL) == 2
                    and hip.get_option(hip.OPT_UPDATE_BLOCKS_PER_CU) == 0 and hip.get_option(hip.OPT_GEMM_TILE) == 0)
    if entry is None or not default_opts or hip.version() != TRAFFIC_PROFILED_VERSION:
        return {"traffic": None}
    return {"traffic": entry[0],
            "traffic_from": {"profile": entry[1], "library_version": TRAFFIC_PROFILED_VERSION,
                             "note": "counter reading of an earlier rocprofv3 session with this library version, "
                                     "not of this run"}}


def hbm_roofline(hip, kernel, traffic_key, nbytes, update_ms, ceilings):
    """HBM roofline object of one streaming kernel: algorithmic bytes per launch / average launch duration."""
    achieved = nbytes / (update_ms * 1e-3) / 1e9
    out = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": round(achieved / HBM_PEAK_GBS, 4), **traffic_fields(hip, traffic_key),
           "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": round(update_ms, 4),
           "target_frac": 0.80, "meets_target": bool(achieved / HBM_PEAK_GBS >= 0.80)}
    for name, gbs in (ceilings or {}).items():
        out[f"measured_{name}_ceiling_GBs"] = round(gbs, 1)
        out[f"frac_of_{name}_ceiling"] = round(achieved / gbs, 4)
    return out


# ---------------------------------------------------------------------------
# CPU baseline: the oracle, as it stands, on the host cores
# ---------------------------------------------------------------------------

def cpu_baseline(wl, budget_s=12.0):
    """The oracle as it stands on this host.  Training workloads: whole rounds for about budget_s seconds.
    Update-only workloads: at least 3 rounds at FULL size (all P replicas x N parameters in host memory, inputs
    drawn by several threads) on all host cores, then the plain single-thread loop on a 1/16 slice."""
    import oracle
    F = np.float32
    cores = oracle.num_threads()
    if wl.has_grad:
        ld = workloads.round_up(wl.N, TRAINING_LD_ALIGN)
        w0 = workloads.init_packed_weights(wl)
        W = workloads.replicate(w0, wl.P, ld); Wc = w0.copy()
        V = np.zeros_like(W)
        X, y = workloads.minibatch(wl, 0)
        done, t0 = 0, time.perf_counter()
        while True:
            G, _ = oracle.mlp_grad_all_workers(wl.dims, W, X, y)
            if wl.momentum:
                oracle.measgd_round(W, V, G, Wc, F(wl.eta), F(wl.rho), F(wl.delta), N=wl.N)
            else:
                oracle.easgd_round(W, G, Wc, F(wl.eta), F(wl.rho), N=wl.N)
            done += 1
            el = time.perf_counter() - t0
            if el >= budget_s or done >= 200:
                break
        return {"value": round(done / el, 4), "unit": "rounds/s", "cores": cores, "kind": "oracle",
                "sample": f"{done} whole rounds (numpy fp64 gradient of all {wl.P} workers + C elastic update) "
                          f"of the same workload in {el:.1f} s"}
    t_gen = time.perf_counter()
    threads = min(16, os.cpu_count() or 8)
    W = workloads.host_normal_rows(wl.P, wl.N, workloads.WEIGHT_STD, 5, threads=threads)
    G = workloads.host_normal_rows(wl.P, wl.N, workloads.GRADIENT_STD, 6, threads=threads)
    Wc = workloads.host_normal_rows(1, wl.N, workloads.WEIGHT_STD, 7, threads=threads)[0]
    V = np.zeros_like(W) if wl.momentum else None
    t_gen = time.perf_counter() - t_gen

    def timed(W, V, G, Wc, budget, at_least, cap):
        done, t0 = 0, time.perf_counter()
        while True:
            if wl.momentum:
                oracle.measgd_round(W, V, G, Wc, F(wl.eta), F(wl.rho), F(wl.delta))
            else:
                oracle.easgd_round(W, G, Wc, F(wl.eta), F(wl.rho))
            done += 1
            el = time.perf_counter() - t0
            if done >= at_least and (el >= budget or done >= cap):
                return done, el

    timed(W, V, G, Wc, 0.0, 1, 1)                  # first touch of every page by the threads that will use it
    done, el = timed(W, V, G, Wc, budget_s, 3, 100)
    frac = 16
    n = wl.N // frac
    sW, sG, sWc = np.ascontiguousarray(W[:, :n]), np.ascontiguousarray(G[:, :n]), Wc[:n].copy()
    sV = np.zeros_like(sW) if wl.momentum else None
    oracle.set_num_threads(1)
    try:
        done1, el1 = timed(sW, sV, sG, sWc, 2.0, 1, 20)
    finally:
        oracle.set_num_threads(0)
    return {"value": round(done / el, 4), "unit": "rounds/s", "cores": cores, "kind": "oracle",
            "sample": f"{done} rounds at full size ({wl.P} replicas x {wl.N} parameters, "
                      f"{update_bytes(wl) / 1e9:.2f} GB streamed per round) in {el:.1f} s after one untimed round; "
                      f"inputs drawn in {t_gen:.1f} s",
            "GBs": round(update_bytes(wl) * done / el / 1e9, 2),
            "single_thread": {"value": round(done1 / el1 / frac, 4), "unit": "rounds/s",
                              "GBs": round(update_bytes(wl) / frac * done1 / el1 / 1e9, 2),
                              "sample": f"{done1} rounds on a 1/{frac} slice of the parameter index in {el1:.1f} s, "
                                        f"rate divided by {frac}"}}


# ---------------------------------------------------------------------------

def update_roofline(hip, wl, rule, update_ms, ceilings):
    """HBM roofline of one streaming update launch at the workload's size."""
    P, N = wl.P, wl.N
    if rule == "sync_sgd":
        return hbm_roofline(hip, "sync_sgd_vec4_dies_kernel", ("sync_sgd", wl.momentum, P, N), 12 * P * N, update_ms, ceilings)
    if rule == "elastic_bf16":
        return hbm_roofline(hip, "elastic_bf16_vec4_dies_kernel", ("elastic_bf16", wl.momentum, P, N),
                            N * ((14 if wl.momentum else 10) * P + 8), update_ms, ceilings)
    if rule == "async":      # P turns: W, g (V) read and W (V) written per turn, the center read and written once
        return hbm_roofline(hip, "async_vec4_dies_kernel", ("async", wl.momentum, P, N), update_bytes(wl), update_ms, ceilings)
    if rule == "hogwild":    # per worker: W, g read, W written, the center read and one read-modify-write added to it
        return hbm_roofline(hip, "hogwild_vec4_kernel", ("hogwild", wl.momentum, P, N),
                            N * P * ((32 if wl.momentum else 24)), update_ms, ceilings)
    return hbm_roofline(hip, "elastic_vec4_dies_kernel (measgd)" if wl.momentum else "elastic_vec4_dies_kernel (easgd)",
                        ("elastic", wl.momentum, P, N), update_bytes(wl), update_ms, ceilings)


MFMA_CEILINGS = {}      # filled by main(): what the bare matrix-instruction loops reach on this device in this run


def mfma_ceilings(hip, iters=2000, reps=5):
    """Attainable fp32 rate of the products' matrix instruction (TFLOP/s): the bare loop with operands in registers,
    and the same loop fetching every instruction's operands from LDS (two blocks of four wavefronts per compute
    unit, like a cfg2 forward launch; no global memory, barriers or epilogues)."""
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out = torch.empty(2 * cus * 4096, dtype=torch.float32, device="cuda")
    src = torch.randn(16 * 1024 * 1024, dtype=torch.float32, device="cuda")      # 64 MB: beyond the L2s, inside the last-level cache
    res = {}
    for name, fetch in (("registers", 0), ("lds_fetch", 1), ("lds_fetch_global_feed", 2)):
        for _ in range(5):                  # untimed: the clocks start slow
            flops = hip.mfma_probe(out, iters, fetch, 2, src=src)
        e0, e1 = _events(1)[0], _events(1)[0]
        e0.record()
        for _ in range(reps):
            hip.mfma_probe(out, iters, fetch, 2, src=src)
        e1.record()
        torch.cuda.synchronize()
        res[name] = flops * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12
    # the same loop in launches as short as a cfg2 forward product (25 passes = K 800), back to back on one stream:
    # what a kernel that did nothing but its matrix instructions would reach once launch boundaries are paid
    flops = hip.mfma_probe(out, 25, 1, 2)
    e0, e1 = _events(1)[0], _events(1)[0]
    e0.record()
    for _ in range(200):
        hip.mfma_probe(out, 25, 1, 2)
    e1.record()
    torch.cuda.synchronize()
    res["short_launch"] = flops * 200 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    res["short_launch_us"] = e0.elapsed_time(e1) * 1e3 / 200
    return res


def mfma_roofline(hip, kernel, traffic_key, flops, ms):
    tflops = flops / (ms * 1e-3) / 1e12
    out = {"bound": "mfma", "kernel": kernel, "achieved": round(tflops, 2), "peak": MFMA_FP32_PEAK_TFLOPS,
           "unit": "TFLOP/s", "frac": round(tflops / MFMA_FP32_PEAK_TFLOPS, 4), **traffic_fields(hip, traffic_key),
           "useful_flops_per_launch": flops, "avg_launch_ms": round(ms, 4)}
    if MFMA_CEILINGS:
        out["measured_mfma_loop_TFLOPs"] = round(MFMA_CEILINGS["registers"], 1)
        out["measured_mfma_loop_with_lds_fetch_TFLOPs"] = round(MFMA_CEILINGS["lds_fetch"], 1)
        out["frac_of_mfma_loop_with_lds_fetch"] = round(tflops / MFMA_CEILINGS["lds_fetch"], 4)
        out["measured_mfma_loop_with_lds_fetch_and_global_feed_TFLOPs"] = round(MFMA_CEILINGS["lds_fetch_global_feed"], 1)
        out["measured_mfma_loop_in_short_launches"] = {
            "TFLOPs": round(MFMA_CEILINGS["short_launch"], 1), "us_per_launch": round(MFMA_CEILINGS["short_launch_us"], 2),
            "note": "the LDS-fetch loop in back-to-back launches of 25 passes (3.36 GFLOP, the size of cfg2's first "
                    "forward product): the rate left once a launch boundary per product is paid"}
    return out


def training_report(hip, wl, steps, warmup, name, full):
    """One training workload through the one-call path (the headline) and the two-call path; full=True adds the
    bfloat16-storage extensions (the host-fed leg is timed by main(), last)."""
    r1 = bench_training(hip, wl, steps, warmup, one_call=True)
    r = bench_training(hip, wl, steps, warmup, one_call=False)
    out = {"value": round(steps / r1["elapsed_s"], 2), "ms_per_step": round(r1["ms_per_step"], 4),
           "path": "easgd_mlp_round: one call per round, elastic update fused into backward propagation",
           "round_call_ms": round(r1["grad_ms"], 4), "preroll_s": r1["preroll_s"],
           "preroll_stable": r1["preroll_stable"], "launches_per_round": r1["launches_per_round"],
           "two_call_path": {"rounds_per_s": round(steps / r["elapsed_s"], 2),
                             "ms_per_step": round(r["ms_per_step"], 4),
                             "launches_per_round": r["launches_per_round"],
                             "phases_ms": {"easgd_grad": round(r["grad_ms"], 4),
                                           "elastic_update": round(r["update_ms"], 4)}}}
    # the dominant kernels are the matrix products.  `roofline`: all products of one easgd_grad call of the two-call
    # path (matrix products, softmax and nothing else), useful flops over the call's duration from HIP events.
    # `roofline_one_call`: the same useful flops over the duration of the whole easgd_mlp_round call, whose
    # products also apply the elastic update in their epilogues -- the path `value` times.
    out["roofline"] = mfma_roofline(hip, "gemm_mfma_kernel (all products of easgd_grad, two-call path)",
                                    ("grad", name), grad_flops(wl), r["grad_ms"])
    out["roofline_one_call"] = mfma_roofline(hip, "gemm_mfma_kernel + elastic epilogues (all launches of easgd_mlp_round)",
                                             ("round", name), grad_flops(wl), r1["grad_ms"])
    out["update_in_round"] = {"GBs_algorithmic": round(update_bytes(wl) / (r["update_ms"] * 1e-3) / 1e9, 1),
                              "note": "elastic update of the two-call path; replicas of this size are served partly "
                                      "from the 256 MB last-level cache, so this is not an HBM figure"}
    if len(wl.dims) == 2 and hip.get_option(hip.OPT_ROUND_SINGLE_LAUNCH) == 0:
        # a single-layer network: the same round as ONE launch (both phases in one grid, a barrier over the grid
        # between them) instead of two dependent launches; opt-in in the library, timed here for comparison
        hip.set_option(hip.OPT_ROUND_SINGLE_LAUNCH, 1)
        try:
            s1 = bench_training(hip, wl, steps, warmup, one_call=True)
        finally:
            hip.set_option(hip.OPT_ROUND_SINGLE_LAUNCH, 0)
        out["single_launch_round"] = {
            "rounds_per_s": round(steps / s1["elapsed_s"], 2), "ms_per_step": round(s1["ms_per_step"], 4),
            "launches_per_round": s1["launches_per_round"],
            "note": "EASGD_OPT_ROUND_SINGLE_LAUNCH = 1 (not the default): forward and softmax, grid-wide barrier, "
                    "gradient and update in one launch"}
    if wl.momentum:
        # an extension (the paper names low precision only as future work): the same rounds with the momentum
        # buffers stored as bfloat16
        b1 = bench_training(hip, wl, steps, warmup, one_call=True, v_bf16=True)
        out["bf16_momentum_storage"] = {
            "rounds_per_s": round(steps / b1["elapsed_s"], 2), "ms_per_step": round(b1["ms_per_step"], 4),
            "note": "extension: easgd_mlp_round_bf16v, bfloat16 momentum buffers; fp32 replicas, center, gradients "
                    "and arithmetic"}
        if full:
            b2 = bench_training(hip, wl, steps, warmup, one_call=False, v_bf16=True)
            out["bf16_momentum_storage"]["two_call_path"] = {
                "rounds_per_s": round(steps / b2["elapsed_s"], 2), "ms_per_step": round(b2["ms_per_step"], 4),
                "phases_ms": {"easgd_grad": round(b2["grad_ms"], 4), "elastic_update": round(b2["update_ms"], 4)}}
    if full:
        # an extension: the two-call path with the gradients (and momentum buffers) stored as bfloat16
        g = bench_training(hip, wl, steps, warmup, one_call=False, v_bf16=wl.momentum, g_bf16=True)
        out["two_call_path"]["with_bf16_gradient_storage"] = {
            "rounds_per_s": round(steps / g["elapsed_s"], 2), "ms_per_step": round(g["ms_per_step"], 4),
            "phases_ms": {"easgd_grad": round(g["grad_ms"], 4), "elastic_update": round(g["update_ms"], 4)},
            "note": "extension: easgd_grad writes bfloat16 gradients, the update reads them"
                    + (" and keeps bfloat16 momentum buffers" if wl.momentum else "")}
    return out


def mix32_ceiling(hip, n=600_000_000, reps=12):
    """Attainable HBM bandwidth (GB/s) for a 3-read/2-write stream, the mix of the momentum update, over five
    arrays of 2.4 GB (12 GB in all, the footprint of cfg5)."""
    import torch
    bufs = [torch.ones(n, dtype=torch.float32, device="cuda") for _ in range(5)]
    for _ in range(3):
        hip.stream_mix32(*bufs, 0.5)
    e0, e1 = _events(1)[0], _events(1)[0]
    e0.record()
    for _ in range(reps):
        hip.stream_mix32(*bufs, 0.5)
    e1.record()
    torch.cuda.synchronize()
    return 20.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg2", choices=sorted(workloads.WORKLOADS))
    ap.add_argument("--no-extras", action="store_true", help="skip the cfg4/cfg5 elastic-update legs of the default run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--round-overlap", type=int, default=None, choices=(0, 1, 2, 3),
                    help="library option EASGD_OPT_ROUND_OVERLAP for the one-call path (default: the library's)")
    ap.add_argument("--gemm-pair", type=int, default=None, choices=(0, 1),
                    help="library option EASGD_OPT_GEMM_PAIR: 0 = one launch per matrix product (tells the products "
                         "apart in a profile), default: the library's (shared launches)")
    ap.add_argument("--gemm-xcd", type=int, default=None, choices=(0, 1, 2, 3),
                    help="library option EASGD_OPT_GEMM_XCD (block order of the matrix products), default: the library's")
    ap.add_argument("--mlp-head", type=int, default=None, choices=(0, 1),
                    help="library option EASGD_OPT_MLP_HEAD: 0 = the last layer as three launches, default: the "
                         "library's (one launch for a narrow last layer)")
    ap.add_argument("--update-layout", type=int, default=None, choices=(0, 1, 2),
                    help="library option EASGD_OPT_UPDATE_LAYOUT of the streaming update kernels: 0 = contiguous tiles, "
                         "1 = die-interleaved, default: the library's (chosen per call)")
    ap.add_argument("--update-groups", type=int, default=None, choices=(0, 1, 2, 4, 8),
                    help="library option EASGD_OPT_UPDATE_GROUPS, default: the library's (chosen per call)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all P replicas live in one HBM); --gpus must be 1. "
              "The design notes of this repository describe how the round would shard over several GPUs.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1708_02983_amd as hip      # raises if the HIP library is missing: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.round_overlap is not None:
        hip.set_option(hip.OPT_ROUND_OVERLAP, args.round_overlap)
    if args.gemm_pair is not None:
        hip.set_option(hip.OPT_GEMM_PAIR, args.gemm_pair)
    if args.gemm_xcd is not None:
        hip.set_option(hip.OPT_GEMM_XCD, args.gemm_xcd)
    if args.mlp_head is not None:
        hip.set_option(hip.OPT_MLP_HEAD, args.mlp_head)
    if args.update_layout is not None:
        hip.set_option(hip.OPT_UPDATE_LAYOUT, args.update_layout)
    if args.update_groups is not None:
        hip.set_option(hip.OPT_UPDATE_GROUPS, args.update_groups)
    wl = workloads.WORKLOADS[args.workload]
    steps = args.steps if args.steps is not None else (300 if wl.has_grad else 100)
    warmup = args.warmup if args.warmup is not None else (20 if wl.has_grad else 5)

    ceilings = {"triad": triad_ceiling(hip)}
    if wl.has_grad:
        MFMA_CEILINGS.update(mfma_ceilings(hip))
    mix = getattr(hip, "stream_mix32", None)
    if mix is not None:
        ceilings["3r2w"] = mix32_ceiling(hip)
    line = {"metric": "Sync EASGD rounds/sec", "unit": "rounds/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": DESCRIPTIONS[args.workload], "P": wl.P, "params_per_replica": wl.N,
                       "eta": wl.eta, "rho": wl.rho, "delta": wl.delta},
            "library_version": hip.version()}
    if wl.has_grad:
        line.update(training_report(hip, wl, steps, warmup, args.workload, full=True))
    else:
        r = bench_update_only(hip, wl, steps, warmup)
        line.update({"value": round(steps / r["elapsed_s"], 2), "ms_per_step": round(r["ms_per_step"], 4),
                     "preroll_s": r["preroll_s"]})
        line["roofline"] = update_roofline(hip, wl, "elastic", r["update_ms"], ceilings)

    if wl.has_grad and not args.no_extras:
        # the other two training workloads, at the same step counts (cfg3 is the one that exercises the momentum
        # rule Eq. (5),(6) and is large enough to matter for both rooflines; cfg1 is bound by launch latency)
        others = {}
        for name in ("cfg1", "cfg3"):
            if name != args.workload:
                others[name] = training_report(hip, workloads.WORKLOADS[name], steps, warmup, name, full=False)
                others[name]["workload"] = DESCRIPTIONS[name]
                torch.cuda.empty_cache()
        line["training_workloads"] = others
        extra = {}
        for name in ("cfg4", "cfg5"):
            w2 = workloads.WORKLOADS[name]
            r2 = bench_update_only(hip, w2, 100, 5)
            extra[name] = {"workload": DESCRIPTIONS[name], "rounds_per_s": round(100 / r2["elapsed_s"], 2),
                           "ms_per_step": round(r2["ms_per_step"], 4), "preroll_s": r2["preroll_s"],
                           "roofline": update_roofline(hip, w2, "elastic", r2["update_ms"], ceilings)}
            torch.cuda.empty_cache()
        # the method's point of comparison on the same replicas: synchronous data-parallel SGD (gradient sum
        # applied to every copy); per parameter and worker it reads g and W and writes W
        w4 = workloads.WORKLOADS["cfg4"]
        r3 = bench_update_only(hip, w4, 100, 5, rule="sync_sgd")
        extra["sync_sgd_cfg4_shape"] = {
            "workload": "synchronous data-parallel SGD round, P=8 replicas x 61M fp32 parameters (sync_sgd_round)",
            "rounds_per_s": round(100 / r3["elapsed_s"], 2), "ms_per_step": round(r3["ms_per_step"], 4),
            "roofline": update_roofline(hip, w4, "sync_sgd", r3["update_ms"], ceilings)}
        torch.cuda.empty_cache()
        # the asynchronous exchanges the paper compares the synchronous round with, on cfg4's replicas: the master
        # serving one worker at a time (one sweep over the workers in rank order per launch; deterministic), and the
        # lock-free exchange of all workers at once (not reproducible from run to run)
        for rule, label in (("async", "one worker at a time in rank order (Original / Async EASGD; async_easgd_round)"),
                            ("hogwild", "all workers at once, lock-free (Hogwild EASGD; hogwild_easgd_round)")):
            r4 = bench_update_only(hip, w4, 100, 5, rule=rule)
            extra[rule + "_easgd_cfg4_shape"] = {
                "workload": "P=8 replicas x 61M fp32 parameters, " + label,
                "rounds_per_s": round(100 / r4["elapsed_s"], 2), "ms_per_step": round(r4["ms_per_step"], 4),
                "roofline": update_roofline(hip, w4, rule, r4["update_ms"], ceilings)}
            torch.cuda.empty_cache()
        # an extension (the paper names low precision only as future work): the same updates with gradients and
        # momentum buffers stored as bfloat16, fp32 replicas, center and arithmetic
        for name in ("cfg4", "cfg5"):
            w5 = workloads.WORKLOADS[name]
            r5 = bench_update_only(hip, w5, 100, 5, rule="elastic_bf16")
            extra[name + "_bf16_storage"] = {
                "workload": DESCRIPTIONS[name] + "; gradients" + (" and momentum buffers" if w5.momentum else "")
                            + " stored as bfloat16 (extension)",
                "rounds_per_s": round(100 / r5["elapsed_s"], 2), "ms_per_step": round(r5["ms_per_step"], 4),
                "roofline": update_roofline(hip, w5, "elastic_bf16", r5["update_ms"], ceilings)}
            torch.cuda.empty_cache()
        line["elastic_update"] = extra

    if wl.has_grad:
        # last of the GPU legs: it creates a dozen streams, and HIP maps streams onto a few hardware queues in turn --
        # a stream that the library creates afterwards (the second stream of a large whole-round call) can then land
        # on the caller's queue, and the center rule no longer runs beside forward propagation (cfg3: 2.6 ms per
        # round instead of 2.4 ms when this leg ran first)
        line["host_fed"] = bench_host_fed(hip, wl, steps, warmup)
        # the same with one copy per four rounds: a wait and a release between two streams cost the rounds' stream
        # about 13 us a pair whatever the copy's size, which is 6 % of a cfg2 round
        line["host_fed"]["four_rounds_per_copy"] = bench_host_fed(hip, wl, steps, warmup, group=4)

    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, budget_s=8.0 if wl.has_grad else 4.0)
        if "elastic_update" in line:
            for name in ("cfg4", "cfg5"):
                line["elastic_update"][name]["cpu_baseline"] = cpu_baseline(workloads.WORKLOADS[name], budget_s=2.0)
        for name, sub in line.get("training_workloads", {}).items():
            sub["cpu_baseline"] = cpu_baseline(workloads.WORKLOADS[name], budget_s=1.0 if name == "cfg1" else 6.0)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
