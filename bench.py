#!/usr/bin/env python3
"""Benchmark of the IMPACT learner hot path on one MI355X.

A step is one pass of the whole path over one batch: the circular buffer's host-side sampling
(slots and replay counts, written into page-locked host memory that the kernel reads in place:
64 KB per step) and the fused gather + loss + gradient kernel reading the sampled trajectories in
place from the HBM-resident ring.  The ring, the learner's distribution tensors, values and outputs are resident in HBM
before the timed region starts.

Every fourth launch of the timed region is bracketed by HIP events on its stream, for the kernel's
average duration.

Prints one JSON line: trajectory-steps per second, the HBM roofline of the dominant kernel and
the CPU oracle's rate on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, AMD's published peak
# HBM bytes per launch of the fused loss kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by what the
# same counters read for copy kernels of known size (profiles/loss_static_gauss17_C5_fused.md).  Each figure
# is tied to the kernel sources it was taken on (kernel_sources_digest below): once any of them changes, the
# benchmark reports null until the counters are taken again.
MEASURED_TRAFFIC = {       # workload -> (bytes per launch, digest of the kernel sources at that time)
    "C5": (2.0 * 344974 * 1024 + 311038 * 1024, "b97e71b7737558d7"),     # FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, KiB per dispatch
    "C4": (2.0 * 97567 * 1024 + 69744 * 1024, "b97e71b7737558d7"),
}


# The sources that make up the fused loss kernels' device code (the kernels the counters were taken on): the
# pipeline, the policy classes, the device helpers, the argument structure and the instantiation units.
LOSS_KERNEL_SOURCES = ("impact_internal.h", "loss_device.h", "loss_pipeline.h", "policy_cat.h", "policy_gauss.h",
                       "loss_cat.hip", "loss_gauss.hip")


def kernel_sources_digest() -> str:
    """A digest of the loss kernels' sources (what the counters were measured on)."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_1912_00167_amd", "csrc")
    h = hashlib.sha256()
    for name in LOSS_KERNEL_SOURCES:
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str):
    entry = MEASURED_TRAFFIC.get(workload)
    return entry[0] if entry and entry[1] == kernel_sources_digest() else None


def algorithmic_bytes_per_step(wl, cached=None, learner_bf16=False, actions_u8=False) -> int:
    """Each input read once, each output written once (single pass), per (t, b) step.
    cached: None (both distributions in the batch), or "with_target" / "no_target": the buffer keeps
    log pi_worker(a), log pi_target(a) as two doubles in place of the worker's distribution (and of the
    target's, which only the KL term needs)."""
    es = 4 if wl.storage == "f32" else 2
    W = wl.A if wl.dist == workloads.CATEGORICAL else 2 * wl.A
    action = (1 if actions_u8 else 4) if wl.dist == workloads.CATEGORICAL else wl.A * es
    behaviour = {None: 2 * W * es, "with_target": 16 + W * es, "no_target": 16}[cached]
    reads = (2 if learner_bf16 else 4) * W + behaviour + action + es + 1 + 4      # learner, behaviour side, action, reward, done, value
    writes = 4 * W + 12                                  # gradient of the distribution, of the value, vs, adv
    return reads + writes


def refill(binding, buf) -> None:
    """The workers' side of the ring, as bookkeeping only (the records are in place): once fewer live slots
    than a batch remain, free the places of what has been replayed K times (its loss has been enqueued by now)
    and mark every empty slot live again."""
    binding.impact_buffer_release_discarded(buf)
    binding.impact_buffer_reserve(buf, binding.impact_buffer_num_empty(buf))


def fill_ring(torch, binding, wl, buf, block: int):
    """Fill all num_slots slots block by block; return the learner-side tensors (learner dist, values,
    bootstrap) per batch-sized group of consecutive slots.  One batch worth of distinct synthetic
    trajectories is generated and inserted once per batch-sized quarter of the ring (generation on the
    host is the slow part); every quarter has its own slots and its own learner-side tensors in HBM, so
    successive steps touch disjoint memory."""
    per_batch = wl.B // block
    parts = [workloads.make_trajectories(wl, block, stream=1000 + i) for i in range(per_batch)]
    learner, values, boot = [], [], []
    for q in range(wl.num_slots // wl.B):
        cur = dict(learner=[], values=[], bootstrap=[])
        for i, x in enumerate(parts):
            d = {k: torch.from_numpy(v).cuda() for k, v in x.items()}
            if wl.dist == workloads.CATEGORICAL:                # (a buffer may keep action indices as bytes)
                d["actions"] = d["actions"].to(buf.action_dtype)
            slots = binding.impact_buffer_insert(buf, d)
            first = (q * per_batch + i) * block
            assert slots[0] == first and slots[-1] == first + block - 1
            for k in cur:
                cur[k].append(d[k])
            del d
        learner.append(torch.cat(cur["learner"], dim=1).contiguous())
        values.append(torch.cat(cur["values"], dim=1).contiguous())
        boot.append(torch.cat(cur["bootstrap"], dim=0).contiguous())
    torch.cuda.synchronize()
    return learner, values, boot


def cpu_model_string() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl, sample_B: int, min_wall_s: float = 8.0, single_B: int = 256, single_wall_s: float = 4.0):
    """Time the oracle (as it is) on a bounded sample of the workload: whole passes (sample, gather, loss with
    gradients) over sample_B trajectories on all host threads until min_wall_s has elapsed, then the same on
    single_B trajectories with one thread."""
    import oracle
    from oracle.buffer import BufferOracle, bf16_bits_to_f32

    def leg(n_traj, threads, wall_s):
        x = workloads.make_trajectories(wl, n_traj, stream=77)
        ob = BufferOracle(wl.dist, wl.T, wl.A, n_traj, max(wl.K, 1 << 20), wl.storage)
        ob.insert_records(x["worker"], x["actions"], x["rewards"], x["dones"], target=x["target"])
        cfg = oracle.config_from_hyper(wl.hyper)
        passes = 0
        t0 = time.perf_counter()
        while True:
            slots, _ = ob.sample(n_traj)
            g = ob.gather(slots)
            if wl.storage == "bf16":
                g = {k: (bf16_bits_to_f32(v) if v.dtype == np.uint16 else v) for k, v in g.items()}
            oracle.impact_loss(wl.dist, x["learner"], g["target"], g["worker"], g["actions"], g["rewards"], g["dones"],
                               x["values"], x["bootstrap"], cfg, n_threads=threads)
            passes += 1
            dt = time.perf_counter() - t0
            if dt >= wall_s:
                break
        return passes, dt

    threads = min(oracle.max_threads(), os.cpu_count() or 1)
    passes, dt = leg(sample_B, threads, min_wall_s)
    p1, dt1 = leg(single_B, 1, single_wall_s)
    return dict(value=passes * wl.T * sample_B / dt, unit="trajectory-steps/s", cores=threads, kind="oracle",
                sample=f"{passes} passes over {sample_B} of {wl.B} trajectories of {wl.name} (T={wl.T}): sample + gather + "
                       f"loss with gradients, {dt:.2f} s wall on {threads} threads ({dt * threads:.0f} core-seconds); "
                       f"single thread: {p1} passes over {single_B} trajectories in {dt1:.2f} s",
                single_thread_value=p1 * wl.T * single_B / dt1, nproc=os.cpu_count(), cpu_model=cpu_model_string())


def device_copy_ceiling(torch, nbytes: int = 1 << 30, repeats: int = 20):
    """The box's device-to-device copy rate (read + written bytes per second), timed in this process: a
    torch copy of nbytes between two resident tensors, HIP events around `repeats` back-to-back copies."""
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    a.zero_()
    for _ in range(5):
        b.copy_(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(repeats):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / repeats
    del a, b
    return 2 * nbytes / (ms * 1e-3) / 1e9


def branch_fractions(wl, n: int = 256):
    """Clip and truncation fractions of the synthetic workload (oracle, small sample): the share of steps
    whose surrogate sits on the clipped branch and whose importance weight exceeds rho_bar."""
    import oracle

    x = workloads.make_trajectories(wl, min(n, wl.B), stream=78)
    if wl.storage == "bf16":
        x = dict(x)
        for k in ("target", "worker", "rewards") + (("actions",) if wl.dist == workloads.GAUSSIAN else ()):
            x[k] = oracle.quantize_bf16(x[k])[1]
    h = wl.hyper
    o = oracle.impact_loss(wl.dist, x["learner"], x["target"], x["worker"], x["actions"], x["rewards"], x["dones"],
                           x["values"], x["bootstrap"], oracle.config_from_hyper(h))
    R, adv, lp = np.asarray(o["ratio"]), np.asarray(o["adv"]), np.asarray(o["logp3"])
    clipped = ((adv > 0) & (R > 1 + h.eps)) | ((adv < 0) & (R < 1 - h.eps))
    w = np.exp(lp[..., 1] - lp[..., 2])
    return float(clipped.mean()), float((w > h.rho_bar).mean())


def table(torch, binding, names, repeats: int = 5) -> None:
    """Three lines per workload, as markdown on stdout: the loss on a pre-gathered time-major batch, the
    gather alone, and the fused gather + loss.  HIP events around back-to-back calls, median of repeats."""
    def timed(call, n_calls):
        for i in range(max(10, n_calls)):            # past the clock transient that follows idle
            call(i)
        torch.cuda.synchronize()
        us = []
        for _ in range(repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(n_calls):
                call(i)
            e1.record()
            torch.cuda.synchronize()
            us.append(e0.elapsed_time(e1) * 1e3 / n_calls)
        return float(np.median(us))

    def timed_wall(call, n_calls):
        for i in range(max(10, n_calls)):
            call(i)
        torch.cuda.synchronize()
        us = []
        for _ in range(repeats):
            t0 = time.perf_counter()
            for i in range(n_calls):
                call(i)
            torch.cuda.synchronize()
            us.append((time.perf_counter() - t0) * 1e6 / n_calls)
        return float(np.median(us))

    gc.collect()
    gc.disable()       # a full collection (about 30 ms with torch loaded) would land in one of the timing loops
    print("| workload | line | us/call | steps/s | algorithmic GB/s | % of 8 TB/s | clipped | truncated |")
    print("|---|---|---|---|---|---|---|---|")
    for name in names:
        wl = workloads.WORKLOADS[name]
        T, B, W = wl.T, wl.B, wl.W
        buf = binding.Buffer(wl.dist, T, wl.A, wl.num_slots, wl.K, wl.storage)
        learner, values, boot = fill_ring(torch, binding, wl, buf, min(B, 4096))
        nq = len(learner)
        slots = [torch.arange(q * B, (q + 1) * B, dtype=torch.int32, device="cuda") for q in range(nq)]
        outs2 = [binding.alloc_loss_out(T, B, W) for _ in range(2)]      # alternate: no call overwrites what the last one wrote
        out = outs2[0]
        ws = torch.empty(binding.impact_loss_workspace_bytes(wl.dist, T, B, wl.A), dtype=torch.uint8, device="cuda")
        cfg = binding.config_from_hyper(wl.hyper)
        gathered = [binding.impact_buffer_gather(buf, slots[q]) for q in range(min(nq, 2))]
        dst = binding.alloc_batch(buf, B)
        n_calls = 100
        t_tm = timed(lambda i: binding.impact_loss_fwd_bwd(wl.dist, learner[i % len(gathered)], values[i % len(gathered)],
                                                           boot[i % len(gathered)], gathered[i % len(gathered)], cfg,
                                                           out=outs2[i % 2], workspace=ws), n_calls)
        out_tp = [binding.alloc_loss_out(T, B, W, packed=True) for _ in range(2)]
        t_tp = timed(lambda i: binding.impact_loss_fwd_bwd(wl.dist, learner[i % len(gathered)], values[i % len(gathered)],
                                                            boot[i % len(gathered)], gathered[i % len(gathered)], cfg,
                                                            out=out_tp[i % 2], workspace=ws), n_calls)
        del out_tp
        t_g = timed(lambda i: binding.impact_buffer_gather(buf, slots[i % nq], dst), n_calls)
        t_f = timed(lambda i: binding.impact_loss_fwd_bwd_from_buffer(buf, slots[i % nq], learner[i % nq], values[i % nq],
                                                                      boot[i % nq], cfg, out=outs2[i % 2], workspace=ws), n_calls)
        out_p = [binding.alloc_loss_out(T, B, W, packed=True) for _ in range(2)]
        t_p = timed(lambda i: binding.impact_loss_fwd_bwd_from_buffer(buf, slots[i % nq], learner[i % nq], values[i % nq],
                                                                      boot[i % nq], cfg, out=out_p[i % 2], workspace=ws), n_calls)
        del out_p
        # successive calls alternating between two streams and two lanes (wall clock: no stream sees both)
        lanes = [dict(stream=torch.cuda.Stream(), cfg=binding.config_from_hyper(wl.hyper, binding.IMPACT_FLAG_LANE(n + 1)),
                      ws=torch.empty_like(ws), outs=[binding.alloc_loss_out(T, B, W) for _ in range(2)]) for n in range(2)]

        def two(i):
            ln = lanes[i % 2]
            binding.impact_loss_fwd_bwd_from_buffer(buf, slots[i % nq], learner[i % nq], values[i % nq], boot[i % nq], ln["cfg"],
                                                    out=ln["outs"][(i // 2) % 2], workspace=ln["ws"], stream=ln["stream"])
        t_2 = timed_wall(two, n_calls)
        del lanes
        t_b = None
        if wl.storage == "bf16":                     # the learner's distribution in bf16 as well (a dtype variant)
            lb = [x.to(torch.bfloat16) for x in learner]
            t_b = timed(lambda i: binding.impact_loss_fwd_bwd_from_buffer(buf, slots[i % nq], lb[i % nq], values[i % nq],
                                                                          boot[i % nq], cfg, out=outs2[i % 2], workspace=ws), n_calls)
            del lb
        # host bookkeeping of one sample call (ring walk, counts), timed on its own
        s_np, c_np = np.empty(B, np.int32), np.empty(B, np.int32)
        n_samples = 200
        for k in range(20 + n_samples):
            if k == 20:                             # after a warm-up
                t0 = time.perf_counter()
            if binding.impact_buffer_num_live(buf) < B:
                refill(binding, buf)
            binding.impact_buffer_sample(buf, B, s_np, c_np)
        t_s = (time.perf_counter() - t0) * 1e6 / n_samples
        clip, trunc = branch_fractions(wl)
        es = 4 if wl.storage == "f32" else 2
        resident = (2 * W * es + (4 if wl.dist == workloads.CATEGORICAL else wl.A * es) + es + 1)   # buffer bytes per step
        steps = T * B
        for line, us, bps in (("loss, time-major batch", t_tm, algorithmic_bytes_per_step(wl)),
                              ("loss, time-major batch, per-step scalars as packed records", t_tp, algorithmic_bytes_per_step(wl)),
                              ("gather alone", t_g, 2 * resident),
                              ("fused gather + loss", t_f, algorithmic_bytes_per_step(wl)),
                              ("fused, per-step scalars as packed records", t_p, algorithmic_bytes_per_step(wl)),
                              ("fused, successive calls alternating between two streams", t_2, algorithmic_bytes_per_step(wl))):
            gbs = bps * steps / us / 1e3
            print(f"| {wl.name} | {line} | {us:.1f} | {steps / us * 1e6:.3e} | {gbs:.0f} | {gbs / 80:.1f} | "
                  f"{clip * 100:.1f} % | {trunc * 100:.1f} % |", flush=True)
        if t_b is not None:
            bps = algorithmic_bytes_per_step(wl, learner_bf16=True)
            gbs = bps * steps / t_b / 1e3
            print(f"| {wl.name} | fused, learner distribution in bf16 ({bps} B/step) | {t_b:.1f} | {steps / t_b * 1e6:.3e} | "
                  f"{gbs:.0f} | {gbs / 80:.1f} | {clip * 100:.1f} % | {trunc * 100:.1f} % |", flush=True)
        print(f"| {wl.name} | sample (host bookkeeping, incl. refill) | {t_s:.1f} | {steps / t_s * 1e6:.3e} | - | - | - | - |", flush=True)
        buf.close()
        del gathered, dst
        # the same step on a buffer that keeps the two log-probabilities per step instead of the worker's
        # distribution, and the target's distribution only if the workload has a KL term
        cached = "with_target" if wl.hyper.kl_coeff != 0 else "no_target"
        flags = binding.IMPACT_BUFFER_CACHE_LOGP | (0 if cached == "with_target" else binding.IMPACT_BUFFER_NO_TARGET_DIST)
        buf = binding.Buffer(wl.dist, T, wl.A, wl.num_slots, wl.K, wl.storage, flags=flags)
        del learner, values, boot
        learner, values, boot = fill_ring(torch, binding, wl, buf, min(B, 4096))
        t_c = timed(lambda i: binding.impact_loss_fwd_bwd_from_buffer(buf, slots[i % nq], learner[i % nq], values[i % nq],
                                                                      boot[i % nq], cfg, out=outs2[i % 2], workspace=ws), n_calls)
        bps = algorithmic_bytes_per_step(wl, cached)
        gbs = bps * steps / t_c / 1e3
        what = "kept for the KL term" if cached == "with_target" else "not kept"
        print(f"| {wl.name} | fused, cached log pi(a) pair ({bps} B/step; target distribution {what}) | {t_c:.1f} | "
              f"{steps / t_c * 1e6:.3e} | {gbs:.0f} | {gbs / 80:.1f} | {clip * 100:.1f} % | {trunc * 100:.1f} % |", flush=True)
        buf.close()
        if wl.dist == workloads.CATEGORICAL and wl.A <= 256:
            # the same step on a buffer that keeps the index of the action taken as one byte (a storage variant)
            buf = binding.Buffer(wl.dist, T, wl.A, wl.num_slots, wl.K, wl.storage, flags=binding.IMPACT_BUFFER_ACTIONS_U8)
            del learner, values, boot
            learner, values, boot = fill_ring(torch, binding, wl, buf, min(B, 4096))
            t_u = timed(lambda i: binding.impact_loss_fwd_bwd_from_buffer(buf, slots[i % nq], learner[i % nq], values[i % nq],
                                                                          boot[i % nq], cfg, out=outs2[i % 2], workspace=ws), n_calls)
            bps = algorithmic_bytes_per_step(wl, actions_u8=True)
            gbs = bps * steps / t_u / 1e3
            print(f"| {wl.name} | fused, action indices as bytes ({bps} B/step) | {t_u:.1f} | {steps / t_u * 1e6:.3e} | "
                  f"{gbs:.0f} | {gbs / 80:.1f} | {clip * 100:.1f} % | {trunc * 100:.1f} % |", flush=True)
            buf.close()
        del learner, values, boot, out, outs2
        gc.collect()
    gc.enable()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=128)
    # After idle the chip runs its first 12-30 ms of sustained load with launches up to 35 % longer than in the
    # steady state that follows (kernel trace in profiles/).  Whatever --warmup says, the run therefore starts
    # with an untimed settle phase of this many steps of the same fused launch (reported as config.settle_steps).
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed settle phase before the warm-up: at least this much device time of fused steps (default 100)")
    ap.add_argument("--workload", default="C5", choices=sorted(workloads.WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--packed-outputs", action="store_true",
                    help="per-step scalars as one 16-byte record per step (a layout variant; not the default)")
    ap.add_argument("--no-variants", action="store_true",
                    help="time the headline configuration only (for profiler runs: one kind of launch in the trace)")
    ap.add_argument("--event-every", type=int, default=4, choices=(1, 2, 4, 8, 16),
                    help="in the bracketed phase that follows the timed region: a pair of HIP events around every N-th launch (default 4)")
    ap.add_argument("--series", metavar="FILE", help="also write the bracketed launches' durations (step, ms, ...; one per line) to FILE")
    ap.add_argument("--table", action="store_true",
                    help="instead of the JSON line: a markdown table of all workloads (loss, gather, fused)")
    ap.add_argument("--table-workloads", default=",".join(sorted(workloads.WORKLOADS)),
                    help="with --table: the workloads to include (comma-separated; default all)")
    ap.add_argument("--table-repeats", type=int, default=5, help="with --table: timing repeats per line (median reported)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch
    from paper_1912_00167_amd import binding

    binding.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.table:
        table(torch, binding, [w for w in args.table_workloads.split(",") if w], repeats=args.table_repeats)
        return 0
    wl = workloads.WORKLOADS[args.workload]
    T, B, W = wl.T, wl.B, wl.W

    buf = binding.Buffer(wl.dist, T, wl.A, wl.num_slots, wl.K, wl.storage)
    block = min(B, 4096)
    learner, values, boot = fill_ring(torch, binding, wl, buf, block)
    n_batches = len(learner)                       # distinct batches per pass over the ring
    outs = [binding.alloc_loss_out(T, B, W, packed=args.packed_outputs) for _ in range(2)]
    workspace = torch.empty(binding.impact_loss_workspace_bytes(wl.dist, T, B, wl.A), dtype=torch.uint8, device="cuda")
    cfg = binding.config_from_hyper(wl.hyper)
    stream = torch.cuda.current_stream()

    # Page-locked buffers for the slot indices, read by the kernel in place; the host may run this many
    # steps ahead of the device.
    depth = 16
    pinned = [torch.empty(B, dtype=torch.int32).pin_memory() for _ in range(depth)]
    pinned_np = [p.numpy() for p in pinned]
    counts_np = np.empty(B, dtype=np.int32)
    # A staging buffer is free again once the launch that read it has finished: the stream gets one marker event
    # per `mark_every` launches (two in rotation), and a step waits for the marker that covers the launch which
    # last used its buffer (16 steps back, so that marker was recorded at least 9 launches ago).
    mark_every = 8
    marks = [torch.cuda.Event() for _ in range(depth // mark_every)]
    # The bracketed phase (after the timed region): a pair of timing events around every `every`-th launch, one
    # pair per staging buffer.  The two records between back-to-back launches cost the stream about 2.5 us each,
    # which is why the timed region carries none.
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(depth)]
    every = args.event_every
    assert depth % every == 0 and depth % mark_every == 0
    in_flight = [0] * depth                        # 1 + the step that holds the buffer
    bracketed = [False] * depth
    kept_steps = []
    state = dict(step=0, outs=outs)
    kernel_times = []
    host_marks = {}                                # step -> host clock before and after its records and launch

    def retire(j):
        if in_flight[j]:
            m = in_flight[j] - 1
            marks[(m // mark_every) % len(marks)].synchronize()    # the kernel has read pinned[j]: the buffer is free again
            if bracketed[j]:
                kernel_times.append(pairs[j][0].elapsed_time(pairs[j][1]))
                kept_steps.append(m)
                bracketed[j] = False
            in_flight[j] = 0

    def drain():
        """Wait for everything issued; collect the bracketed launches' times."""
        torch.cuda.synchronize()
        for j in range(depth):
            if bracketed[j]:
                kernel_times.append(pairs[j][0].elapsed_time(pairs[j][1]))
                kept_steps.append(in_flight[j] - 1)
                bracketed[j] = False
            in_flight[j] = 0

    def one_step(bracket=False, mark=None):
        """mark: an event to record on the stream right before this step's launch."""
        i = state["step"]
        j = i % depth
        retire(j)
        if binding.impact_buffer_num_live(buf) < B:
            refill(binding, buf)
        binding.impact_buffer_sample(buf, B, pinned_np[j], counts_np)
        q = int(pinned_np[j][0]) // B              # ring order: batch q holds slots [qB, (q+1)B)
        t_host = time.perf_counter()
        bracket = bracket and j % every == 0
        if mark is not None:
            mark.record(stream)
        if bracket:
            pairs[j][0].record(stream)
        binding.impact_loss_fwd_bwd_from_buffer(buf, pinned[j], learner[q % n_batches], values[q % n_batches],
                                                boot[q % n_batches], cfg, out=state["outs"][i % 2], workspace=workspace,
                                                stream=stream)
        if bracket:
            pairs[j][1].record(stream)
            bracketed[j] = True
        if i % mark_every == mark_every - 1:
            marks[(i // mark_every) % len(marks)].record(stream)
        host_marks[i] = (t_host, time.perf_counter())
        in_flight[j] = i + 1
        state["step"] = i + 1

    # The interpreter's cyclic collector, set off by the small objects every call allocates, takes about
    # 30 ms per full pass over torch's object graph: more than a hundred steps.  It stays off while steps run.
    gc.collect()
    gc.disable()
    # settle phase: fused steps until the device has been busy for --settle-ms (clock steady state); the host
    # runs at most `depth` steps ahead of the device (it waits for each staging buffer), so wall time is device time
    settle_steps = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms or settle_steps < depth:
        one_step()
        settle_steps += 1
    for _ in range(args.warmup):
        one_step()
    drain()

    # The timed region: K steps between two readings of the host clock, and their K launches between two events
    # on the launch stream (the kernel's average duration per launch, dispatch included, is their distance over K;
    # the first is recorded right before the first launch: the device is idle while the host samples for it).
    region = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(mark=region[0] if k == 0 else None)
    region[1].record(stream)
    issued = time.perf_counter() - t0              # host side done; the device may still be working
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    drain()
    kernel_ms = region[0].elapsed_time(region[1]) / args.steps

    # The bracketed phase: the same steps with a pair of events around every `every`-th launch, for the
    # launch-by-launch series and as a cross-check of the figure above (it runs a little higher: the records
    # themselves take stream time).
    n_br = max(every, min(args.steps, 128) // every * every)
    for _ in range(n_br):
        one_step(bracket=True)
    drain()
    assert len(kernel_times) == len(kept_steps) == n_br // every
    main_times, main_steps = list(kernel_times), list(kept_steps)

    # The same step with the per-step scalars written as packed records (a layout variant of the outputs,
    # not the default): a shorter run on the warm device, reported next to the headline figure.
    variant = None
    if not args.packed_outputs and not args.no_variants:
        state["outs"] = [binding.alloc_loss_out(T, B, W, packed=True) for _ in range(2)]
        n_var = min(args.steps, 256)
        for _ in range(32):
            one_step()
        drain()
        ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        ev[0].record(stream)
        for _ in range(n_var):
            one_step()
        ev[1].record(stream)
        drain()
        variant = ev[0].elapsed_time(ev[1]) / n_var
        state["outs"] = outs

    # Successive steps alternating between two streams (a lane of the buffer's completion counters, a
    # workspace and output tensors each): one launch starts while the other drains.  Whole-step throughput
    # only; a launch's own duration is not meaningful while two share the chip.
    two_streams = None
    if not args.packed_outputs and not args.no_variants:
        n_var, n_warm = min(args.steps, 256), min(args.warmup, 128)      # (the device idled while the buffers below were made)
        lanes = [dict(stream=torch.cuda.Stream(), cfg=binding.config_from_hyper(wl.hyper, binding.IMPACT_FLAG_LANE(n + 1)),
                      workspace=torch.empty_like(workspace),
                      outs=[binding.alloc_loss_out(T, B, W) for _ in range(2)]) for n in range(2)]
        staging = [torch.empty(B, dtype=torch.int32).pin_memory() for _ in range(n_var + n_warm)]   # one per step: nothing to wait for
        staging_np = [p.numpy() for p in staging]
        torch.cuda.synchronize()

        def lane_step(i):
            if binding.impact_buffer_num_live(buf) < B:
                refill(binding, buf)
            binding.impact_buffer_sample(buf, B, staging_np[i], counts_np)
            q = int(staging_np[i][0]) // B
            ln = lanes[i % 2]
            binding.impact_loss_fwd_bwd_from_buffer(buf, staging[i], learner[q % n_batches], values[q % n_batches],
                                                    boot[q % n_batches], ln["cfg"], out=ln["outs"][(i // 2) % 2],
                                                    workspace=ln["workspace"], stream=ln["stream"])
        for i in range(n_warm):
            lane_step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(n_warm, n_warm + n_var):
            lane_step(i)
        two_issued = (time.perf_counter() - t1) * 1e3 / n_var
        torch.cuda.synchronize()
        two_ms = (time.perf_counter() - t1) * 1e3 / n_var
        for ln in lanes:
            for o in ln["outs"]:
                assert np.all(np.isfinite(o["loss5"].cpu().numpy()))
        two_streams = {"ms_per_step": two_ms, "value": T * B / (two_ms * 1e-3), "host_issue_ms_per_step": two_issued,
                       "algorithmic_GBps": algorithmic_bytes_per_step(wl) * T * B / (two_ms * 1e-3) / 1e9,
                       "what": "successive steps alternate between two streams and two lanes of the buffer's completion "
                               "counters, so that one launch starts while the other drains; whole-step throughput"}
    # The headline samples in ring order, which yields runs of consecutive slots (the kernel is then given the
    # first slot and reads no index array).  The same step on a batch whose slots lie scattered over the ring
    # (a shuffled quarter of it; the index array in page-locked host memory, read by the kernel): kernel time only.
    scattered = None
    if not args.packed_outputs and not args.no_variants:
        rng = np.random.default_rng(12)
        n_var = min(args.steps, 128)
        perms = []
        for q in range(n_batches):
            perm = torch.from_numpy((q * B + rng.permutation(B)).astype(np.int32))
            order = (perm.long() - q * B).cuda()
            perms.append((perm.pin_memory(), learner[q].index_select(1, order).contiguous(),
                          values[q].index_select(1, order).contiguous(), boot[q].index_select(0, order).contiguous()))
        torch.cuda.synchronize()
        ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        for i in range(32 + n_var):
            sl, ln, va, bo = perms[i % n_batches]
            if i == 32:
                ev[0].record(stream)
            binding.impact_loss_fwd_bwd_from_buffer(buf, sl, ln, va, bo, cfg, out=outs[i % 2], workspace=workspace, stream=stream)
        ev[1].record(stream)
        torch.cuda.synchronize()
        sc_ms = ev[0].elapsed_time(ev[1]) / n_var
        scattered = {"kernel_ms": sc_ms, "frac": algorithmic_bytes_per_step(wl) * T * B / (sc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "what": "the batch's slots scattered over a quarter of the ring (shuffled), index array in page-locked "
                             "host memory read by the kernel; two HIP events around the launches, their distance per launch"}
        del perms
    copy_ceiling = device_copy_ceiling(torch)
    gc.enable()
    if args.series:
        with open(args.series, "w") as f:
            for x, k in zip(main_times, main_steps):       # step, kernel ms, host ms in the launch, host ms since the previous launch
                since = (host_marks[k][0] - host_marks[k - 1][1]) * 1e3 if k - 1 in host_marks else 0.0
                f.write(f"{k} {x:.4f} {(host_marks[k][1] - host_marks[k][0]) * 1e3:.4f} {since:.4f}\n")

    loss = outs[(args.warmup + args.steps - 1) % 2]["loss5"].cpu().numpy()
    assert np.all(np.isfinite(loss)), f"non-finite loss {loss}"
    steps_per_call = T * B
    ms_per_step = wall * 1e3 / args.steps
    bytes_per_call = algorithmic_bytes_per_step(wl) * steps_per_call
    achieved = bytes_per_call / (kernel_ms * 1e-3) / 1e9

    result = {
        "metric": "trajectory-steps/sec for IMPACT loss fwd+bwd (+gather); % of HBM peak",
        "value": steps_per_call / (ms_per_step * 1e-3),
        "unit": "trajectory-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if wl.dist == workloads.GAUSSIAN else "f32+f64",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: T={T} B={B} A={wl.A} {wl.dist}, {wl.storage} buffer fields, "
                               f"ring {wl.num_slots} slots K={wl.K}, fused gather+loss+grad"
                               + (", per-step scalars as packed records" if args.packed_outputs else ""),
                   "algorithmic_bytes_per_step": algorithmic_bytes_per_step(wl),
                   "settle_steps": settle_steps,
                   "host_issue_ms_per_step": issued * 1e3 / args.steps,
                   "loss5": [float(v) for v in loss]},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None if args.packed_outputs else measured_traffic(args.workload),
                     "kernel_ms": kernel_ms, "kernel": "fused loss kernel (the last workgroup sums the loss terms)",
                     "kernel_launches_timed": args.steps,
                     "kernel_ms_bracketed": float(np.mean(main_times)), "kernel_launches_bracketed": len(main_times),
                     "device_copy_ceiling_GBps": copy_ceiling,
                     "frac_of_copy_ceiling": achieved / copy_ceiling},
    }
    if two_streams is not None:
        result.setdefault("variants", {})["two_streams"] = two_streams
    if scattered is not None:
        result.setdefault("variants", {})["scattered_slots"] = scattered
    if variant is not None:
        result.setdefault("variants", {})["packed_step_outputs"] = {
            "kernel_ms": variant, "frac": bytes_per_call / (variant * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "what": "grad_values, vs, adv written as one 16-byte record per step (whole lines per wavefront) "
                    "instead of three [T][B] tensors; same algorithmic bytes"}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, max(8, min(B, 4096)))
    print(json.dumps(result))
    buf.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
