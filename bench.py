#!/usr/bin/env python3
"""Benchmark of the compact-prefill path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 8b] [--sets R] [--layers N] [--no-cpu]

A step is one pass of the whole path over one batch of synthetic input already resident in HBM:
civic_score_visual (the visual rows scored where they lie in the dense sequence) -> civic_select (on
the scores just written) -> civic_compact -> civic_prefill_attn_kv (attention and the KV-cache write
of the same K/V as one call; --unfused runs civic_prefill_attn -> civic_kv_write instead), back to
back on one stream, for one transformer layer.  The timed step issues the first three through
civic_compact_prefill, the library's one-call front (the same three kernels, one crossing from Python;
--separate-calls issues them one by one).  Buffers rotate over R independent sets so that
consecutive steps do not find their inputs in the last-level cache.

Order of a run: an untimed pre-warm of full steps for --prewarm-ms of wall time (the chip's clock
governor needs tens of milliseconds of load before the clocks settle; reported as `prewarm_ms`), W
untimed warm-up steps, then exactly K timed steps between device synchronisations: `value` is
compact-prefill tokens/s = batch * S_c * K / time.

A second pass of the same K steps brackets every stage with HIP events (recorded on the stream the
kernels run on: `us_in_step`, which carries the 2-3 us an event between two short dependent launches
costs).  Another pass of the same K steps arms the library's one-shot kernel timer before every
stage, so that the stage's kernel carries its own pair of HIP events and their difference is the
kernel's duration inside the step (`us_kernel_in_step`, the figure a kernel trace reports);
`roofline` describes the dominant kernel (the attention) against the MI355X bf16 MFMA peak from that
duration.  A third pass times every stage alone as a GPU number: a
spin kernel holds the stream while --stage-launches launches of the stage are queued behind it, and
two events bracket them, so the figure under `stages` (`us`) is the kernels' own back-to-back time
and carries no host launch cost.  `decode` reports the decode-step attention
over the cache the step has just written (one query per sequence, HBM-bound).  `cpu_baseline` times
the CPU oracle, as it stands, on a bounded sample of the same workload on this machine's host cores.
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

from paper_2605_28115_amd import workloads as wl

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
STAGES_FUSED = ("score", "select", "compact", "attn_kv")
STAGES_UNFUSED = ("score", "select", "compact", "attn", "kv_write")


def measured_traffic(workload: str, stage: str):
    """HBM bytes per launch of a stage as the profiler's FETCH_SIZE / WRITE_SIZE counters gave them (scaled by
    what the same counters read for a copy of known size): the line `traffic_bytes_per_launch <stage> <bytes>`
    of profiles/bench_<workload>_hbm_traffic.txt, written by the profiled run.  None when no profile says."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == stage:
                return float(f[2])
    except OSError:
        pass
    return None


def dev(storage: np.ndarray) -> torch.Tensor:
    if storage.dtype == np.uint16:
        return torch.from_numpy(storage.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(storage).cuda()


class BufferSet:
    """Device inputs and outputs of one step (one independent copy per rotation slot)."""

    def __init__(self, bd, w: wl.Workload, trial: int):
        hid, _ = wl.hidden(w, trial)
        self.hidden = dev(hid)
        self.pos = torch.from_numpy(wl.position_ids(w)).cuda()
        (q, _), (k, _), (v, _) = wl.qkv(w, trial)
        self.q, self.k, self.v = dev(q), dev(k), dev(v)
        self.anchor_q = torch.from_numpy(bd.civic_anchor_normalize(wl.anchor(w, trial))).cuda()
        b, sc = w.batch, w.seq_compact
        dt = self.hidden.dtype
        # in a step civic_select reads what civic_score_visual has just written; the workload's own score
        # distribution (scores_in) is what the selection is timed on when it runs alone
        self.scores_in = torch.from_numpy(wl.scores(w, trial)).cuda()
        self.scores = torch.empty((b, w.n_visual), dtype=torch.float32, device="cuda")
        self.kept = torch.empty((b, w.kept), dtype=torch.int32, device="cuda")
        self.hidden_c = torch.empty((b, sc, w.dim), dtype=dt, device="cuda")
        self.pos_c = torch.empty((3, b, sc), dtype=torch.int32, device="cuda")
        self.src_idx = torch.empty((b, sc), dtype=torch.int32, device="cuda")
        self.out = torch.empty((b, sc, w.n_q_heads, w.head_dim), dtype=dt, device="cuda")
        self.k_cache = torch.empty((b, w.n_kv_heads, sc, w.head_dim), dtype=dt, device="cuda")
        self.v_cache = torch.empty_like(self.k_cache)


def make_stage_calls(bd, w: wl.Workload, fs):
    grid = bd.make_grid(w.grid_tuple())

    def score(s):
        bd.civic_score_visual(s.hidden, grid, fs, s.anchor_q, 1.0, scores=s.scores)

    def select(s):
        bd.civic_select(s.scores, grid, kept_idx=s.kept)

    def select_dist(s):
        bd.civic_select(s.scores_in, grid, kept_idx=s.kept)

    def compact(s):
        bd.civic_compact(s.hidden, s.pos, grid, fs, s.kept, hidden_c=s.hidden_c, pos_c=s.pos_c, src_idx=s.src_idx)

    def front(s):
        bd.civic_compact_prefill(s.hidden, s.pos, grid, fs, s.anchor_q, 1.0, scores=s.scores, kept_idx=s.kept,
                                 hidden_c=s.hidden_c, pos_c=s.pos_c, src_idx=s.src_idx)

    def attn(s):
        bd.civic_prefill_attn(s.q, s.k, s.v, w.causal, 0.0, out=s.out)

    def kv_write(s):
        bd.civic_kv_write(s.k, s.v, s.k_cache, s.v_cache, 0)

    def attn_kv(s):
        bd.civic_prefill_attn_kv(s.q, s.k, s.v, s.k_cache, s.v_cache, 0, w.causal, 0.0, out=s.out)

    return dict(score=score, select=select, select_dist=select_dist, compact=compact, front=front, attn=attn,
                kv_write=kv_write, attn_kv=attn_kv)


def algorithmic_work(w: wl.Workload) -> dict:
    """Bytes (or flops) the method itself must move per step, per stage."""
    e = 2 if w.dtype == "bf16" else 4
    b, sc, k = w.batch, w.seq_compact, w.kept
    attn_flops = 4 * w.n_q_heads * w.head_dim * (sc * (sc + 1) // 2 if w.causal else sc * sc) * b
    return dict(
        score=b * w.n_visual * (w.dim * e + 4),
        select=b * (4 * w.n_visual + 4 * k),
        compact=b * sc * (2 * w.dim * e + 24 + 4),
        kv_write=b * sc * 4 * w.n_kv_heads * w.head_dim * e,
        attn_flops=attn_flops,
        attn_bytes=b * sc * (2 * w.n_q_heads + 2 * w.n_kv_heads) * w.head_dim * e,
    )


def cpu_baseline(w: wl.Workload, target_seconds: float = 20.0) -> dict:
    """Times the oracle on a bounded sample of the workload: every stage in full except the
    attention, which computes every `row_step`-th query row and is scaled by row_step."""
    import oracle
    oracle.build()
    fs, grid = wl.frame_starts(w), w.grid_tuple()
    hw = w.height * w.width
    hid, hid32 = wl.hidden(w, 0)
    vis32 = np.ascontiguousarray(np.concatenate([hid32[:, s:s + hw] for s in fs], axis=1).reshape(-1, w.dim))
    q_anchor = oracle.anchor_normalize(wl.anchor(w, 0)).astype(np.float32)
    pos = wl.position_ids(w)
    (q, q32), (k, k32), (v, v32) = wl.qkv(w, 0)
    t = {}
    t0 = time.perf_counter(); sc = oracle.score(vis32, q_anchor, 1.0); t["score"] = time.perf_counter() - t0
    sc = sc.reshape(w.batch, w.n_visual)                   # the selection reads the scores just computed, as on the GPU
    t0 = time.perf_counter(); kept, _ = oracle.select(sc, grid); t["select"] = time.perf_counter() - t0
    t0 = time.perf_counter(); oracle.compact(hid, pos, grid, fs, kept); t["compact"] = time.perf_counter() - t0
    # choose the attention sample from a short probe so the whole leg stays near target_seconds
    t0 = time.perf_counter(); oracle.attention(q32, k32, v32, w.causal, row_step=256); probe = time.perf_counter() - t0
    full_est = probe * 256
    row_step = max(1, int(np.ceil(full_est / target_seconds)))
    t0 = time.perf_counter(); oracle.attention(q32, k32, v32, w.causal, row_step=row_step)
    t["attn"] = (time.perf_counter() - t0) * row_step
    kc = np.zeros((w.batch, w.n_kv_heads, w.seq_compact, w.head_dim), dtype=k.dtype)
    vc = np.zeros_like(kc)
    t0 = time.perf_counter(); oracle.kv_write(k, v, kc, vc, 0); t["kv_write"] = time.perf_counter() - t0
    total = sum(t.values())
    model = next((l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name")), "unknown")
    return {"value": w.batch * w.seq_compact / total, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "cpu_model": model,
            "sample": (f"workload {w.name}: every stage in full, one pass" if row_step == 1 else
                       f"workload {w.name}: score, select, compact and kv_write in full; attention on every "
                       f"{row_step}-th query row, its time scaled by {row_step}"),
            "stage_ms": {s: round(1e3 * x, 3) for s, x in t.items()}}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="8b", choices=list(wl.WORKLOADS))
    ap.add_argument("--sets", type=int, default=4, help="independent buffer sets rotated through (1 = warm cache)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--layers", type=int, default=28,
                    help="transformer layers N_l of the amortised figure: score, select and compact once, attention and "
                         "KV write per layer (28 = the layer count the paper's Table 1 KV sizes imply for its 2B model)")
    ap.add_argument("--unfused", action="store_true", help="attention and KV write as two calls")
    ap.add_argument("--batch", type=int, default=0,
                    help="scale-up run: the same shapes at this batch size instead of the workload's own (labelled in the "
                         "JSON line; shows the stages at steady state, does not replace the workload)")
    ap.add_argument("--path-only", action="store_true",
                    help="skip the decode, rotary and encoder figures (counter runs: every launch then belongs to the path)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="the timed step calls score_visual, select and compact one by one instead of civic_compact_prefill")
    ap.add_argument("--prewarm-ms", type=float, default=150.0,
                    help="untimed full steps for this much wall time ahead of --warmup (0 = none)")
    ap.add_argument("--stage-launches", type=int, default=200,
                    help="launches per stage of the stage-alone pass (queued behind a spin kernel, bracketed by two events)")
    ap.add_argument("--calibrate", action="store_true",
                    help="run only a device-to-device copy of 256 MiB (the known-size kernel the HBM byte counters "
                         "of a profiler run are scaled by) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures the one-GPU path only: run it with --gpus 1 (this build has no collective or "
              "sharded path, so no multi-GPU figure exists)", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py needs the MI355X: no GPU visible", file=sys.stderr)
        return 2

    torch.cuda.set_device(0)
    if args.calibrate:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate": "copy", "bytes_read": 256 << 20, "bytes_written": 256 << 20, "launches": 10}))
        return 0
    from paper_2605_28115_amd import binding as bd     # raises if libcivic.so is not built
    w = wl.WORKLOADS[args.workload]
    if args.batch > 0 and args.batch != w.batch:
        import dataclasses
        w = dataclasses.replace(w, batch=args.batch)
    assert bd.civic_kept_count(w.grid_tuple()) == w.kept
    fs = wl.frame_starts(w)
    sets = [BufferSet(bd, w, trial) for trial in range(max(1, args.sets))]
    calls = make_stage_calls(bd, w, fs)
    STAGES = STAGES_UNFUSED if args.unfused else STAGES_FUSED
    order = [calls[s] for s in STAGES]

    # the timed step: the front of the path as one library call (the same three kernels; one crossing from Python
    # instead of three), then attention and the KV write
    step_calls = order if args.separate_calls else [calls["front"]] + order[3:]

    def step(i):
        s = sets[i % len(sets)]
        for c in step_calls:
            c(s)

    # untimed pre-warm by wall time: the clocks settle under load, whatever --warmup and --steps are
    prewarm_steps, t_pre = 0, time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for _ in range(20):
            step(prewarm_steps)
            prewarm_steps += 1
        torch.cuda.synchronize()
    prewarm_ms = (time.perf_counter() - t_pre) * 1e3
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    tokens = w.batch * w.seq_compact

    def rewarm():
        # ~30 ms of untimed steps queued right ahead of a measuring pass (no synchronisation in between), so that a
        # short pass does not start on a chip that idled while the host prepared it
        for i in range(max(20, int(30.0 / ms_per_step)) if args.prewarm_ms > 0 else 0):
            step(i)

    # second pass: the same steps with an event between stages (torch's current stream is the launch stream)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(STAGES) + 1)] for _ in range(args.steps)]
    rewarm()
    for i in range(args.steps):
        s = sets[i % len(sets)]
        ev[i][0].record()
        for j, c in enumerate(order):
            c(s)
            ev[i][j + 1].record()
    torch.cuda.synchronize()
    stage_us = {}
    for j, name in enumerate(STAGES):
        d = np.asarray([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(args.steps)]) * 1e3
        stage_us[name] = {"mean": float(d.mean()), "median": float(np.median(d)), "min": float(d.min())}

    # the same steps once more, every stage's kernel carrying its own pair of events (the library's one-shot kernel
    # timer): the kernel's duration inside the step, without the gap to the launch before it
    kev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in STAGES]
           for _ in range(args.steps)]
    for per_step in kev:
        for a, b in per_step:
            a.record(); b.record()                  # torch creates an event's handle at its first record
    torch.cuda.synchronize()
    rewarm()
    for i in range(args.steps):
        s = sets[i % len(sets)]
        for j, c in enumerate(order):
            bd.civic_time_next_kernel(*kev[i][j])
            c(s)
    torch.cuda.synchronize()
    for j, name in enumerate(STAGES):
        d = np.asarray([kev[i][j][0].elapsed_time(kev[i][j][1]) for i in range(args.steps)]) * 1e3
        stage_us[name]["kernel"] = float(d.mean())

    # third pass: every stage alone as a GPU number.  A spin kernel occupies the stream while the host queues
    # the launches behind it, so that the two events bracket kernels that start back to back, without the
    # ~8 us of host time a launch from Python costs; the average is the kernel's duration plus the gap the
    # hardware leaves between two dependent launches.
    spin_cycles = 1_000_000
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); torch.cuda._sleep(spin_cycles); e1.record(); torch.cuda.synchronize()
    spin_ms = max(e0.elapsed_time(e1), 1e-3)
    n_alone = max(1, args.stage_launches)
    hold_cycles = int(spin_cycles * (n_alone * 0.012 + 1.0) / spin_ms)     # 12 us of host time per launch, and 1 ms

    def alone(call, cost=1):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        torch.cuda._sleep(hold_cycles * cost)            # (cost: library calls per invocation, so the hold covers the queueing)
        a.record()
        for i in range(n_alone):
            call(sets[i % len(sets)])
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / n_alone

    for name in STAGES:
        if name in ("attn", "attn_kv"):
            # attention launches back to back run slower than in a step (the chip holds a lower clock under
            # sustained MFMA load): the kernel's own duration inside the step is its figure
            stage_us[name]["alone"] = stage_us[name]["kernel"]
            stage_us[name]["back_to_back"] = alone(calls[name])
            continue
        stage_us[name]["alone"] = alone(calls[name])
    select_dist_us = alone(calls["select_dist"])

    work = algorithmic_work(w)
    stages = {}
    for name in STAGES:
        us = stage_us[name]["alone"]
        entry = {"us": round(us, 2), "us_in_step": round(stage_us[name]["mean"], 2),
                 "us_in_step_median": round(stage_us[name]["median"], 2),
                 "us_kernel_in_step": round(stage_us[name]["kernel"], 2)}
        if "back_to_back" in stage_us[name]:
            entry["us_back_to_back"] = round(stage_us[name]["back_to_back"], 2)
        if name in ("attn", "attn_kv"):
            tf = work["attn_flops"] / (us * 1e-6) / 1e12
            entry.update(tflops=round(tf, 1), frac_mfma_peak=round(tf / MFMA_BF16_PEAK_TFLOPS, 4))
            if name == "attn_kv":
                entry["kv_write_bytes"] = work["kv_write"]     # copied inside the attention launch
        else:
            gbs = work[name] / (us * 1e-6) / 1e9
            entry.update(gbs=round(gbs, 1), frac_hbm_peak=round(gbs / HBM_PEAK_GBS, 4))
        stages[name] = entry
    stages["select"]["us_on_workload_scores"] = round(select_dist_us, 2)   # the configuration's own score distribution
    sg = (work["select"] + work["compact"]) / ((stage_us["select"]["alone"] + stage_us["compact"]["alone"]) * 1e-6) / 1e9
    stages["select+compact"] = {"gbs": round(sg, 1), "frac_hbm_peak": round(sg / HBM_PEAK_GBS, 4)}

    attn_name = "attn" if args.unfused else "attn_kv"
    attn_us = stage_us[attn_name]["kernel"]          # the events ride on the kernel's own dispatch, inside the step
    attn_tf = work["attn_flops"] / (attn_us * 1e-6) / 1e12
    if w.dtype == "bf16":
        roofline = {"bound": "mfma", "kernel": f"attn_mfma_kernel (civic_prefill_{attn_name})", "achieved": round(attn_tf, 2),
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(attn_tf / MFMA_BF16_PEAK_TFLOPS, 4),
                    "traffic": measured_traffic(w.name, attn_name) if w.batch == wl.WORKLOADS[w.name].batch else None, "launch_us": round(attn_us, 2),
                    "launch_us_between_events": round(stage_us[attn_name]["mean"], 2), "flops_per_launch": work["attn_flops"]}
    else:
        roofline = {"bound": "alu", "kernel": f"attn_plain_kernel (civic_prefill_{attn_name})", "achieved": round(attn_tf, 3),
                    "peak": 157.3, "unit": "TFLOP/s", "frac": round(attn_tf / 157.3, 5), "traffic": None,
                    "launch_us": round(attn_us, 2), "flops_per_launch": work["attn_flops"]}

    result = {
        "metric": "compact-prefill tokens/s", "value": round(tokens / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "prewarm_ms": round(prewarm_ms, 1),
        "prewarm_steps": prewarm_steps, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": (f"Qwen3-VL-{w.name}-shaped" if w.name in ("2b", "8b") else w.name) +
                               (f", scale-up to batch {w.batch}" if w.batch != wl.WORKLOADS[w.name].batch else ""),
                   "batch": w.batch, "seq_dense": w.seq_len, "seq_compact": w.seq_compact, "visual_tokens": w.n_visual,
                   "kept_visual": w.kept, "hidden": w.dim, "heads": f"{w.n_q_heads}q/{w.n_kv_heads}kv x {w.head_dim}",
                   "causal": w.causal, "layers_timed": 1, "buffer_sets": len(sets),
                   "calls": ("+".join(STAGES).replace("score", "score_visual") if args.separate_calls
                             else "compact_prefill(score_visual,select,compact)+" + "+".join(STAGES[3:])),
                   "stage_launches": n_alone},
        "dense_equivalent_tokens_per_s": round(w.batch * w.seq_len / (ms_per_step * 1e-3), 1),
        "stages": stages,
        "roofline": roofline,
    }
    # Decode-step attention over the cache the step has just written (n_ctx = S_c, one query per sequence): the
    # per-token work of the decoding phase.  The workload's own batch is a launch of a few microseconds; the
    # same shape at batch 64 (labelled) shows the bandwidth the kernel reaches once the chip is covered.
    def decode_figures(batch):
        e = 2 if w.dtype == "bf16" else 4
        dt = sets[0].hidden.dtype
        sc = w.seq_compact
        reps = max(1, min(len(sets), 1 + (1 << 30) // max(1, batch * w.n_kv_heads * sc * w.head_dim * e * 2)))
        kcs = [torch.randn((batch, w.n_kv_heads, sc, w.head_dim), device="cuda").to(dt) for _ in range(reps)]
        vcs = [torch.randn((batch, w.n_kv_heads, sc, w.head_dim), device="cuda").to(dt) for _ in range(reps)]
        qd = torch.randn((batch, w.n_q_heads, w.head_dim), device="cuda").to(dt)
        od = torch.empty_like(qd)
        need = bd.civic_decode_attn_workspace_bytes(dt, batch, w.n_q_heads, w.n_kv_heads, w.head_dim, sc)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        def call(i):
            bd.civic_decode_attn(qd, kcs[i % reps], vcs[i % reps], sc, 0.0, out=od, workspace=ws)
        for i in range(20):
            call(i)
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        torch.cuda._sleep(hold_cycles)
        a.record()
        for i in range(n_alone):
            call(i)
        b_.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b_) * 1e3 / n_alone
        nbytes = batch * (2 * w.n_kv_heads * sc * w.head_dim * e + 2 * w.n_q_heads * w.head_dim * e)
        gbs = nbytes / (us * 1e-6) / 1e9
        return {"batch": batch, "n_ctx": sc, "us": round(us, 2), "bytes": nbytes, "gbs": round(gbs, 1),
                "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "workspace_bytes": need, "cache_sets": reps}

    decode = None
    if not args.path_only and (w.n_kv_heads != w.n_q_heads or w.causal):   # the encoder-side workload keeps no cache
        decode = {"kernel": "decode_partial_kernel + decode_merge_kernel (civic_decode_attn)", "bound": "hbm",
                  "unit": "GB/s", "peak": HBM_PEAK_GBS, "workload": decode_figures(w.batch), "batch_64": decode_figures(64)}

    # Rotary embedding from the carried ids: the table once per prompt; per layer K rotated on its way into the
    # cache (civic_kv_write_rope) and Q rotated inside the attention launch (civic_prefill_attn_rope reading K and
    # V from the cache).  civic_mrope_apply on Q is what the fused attention saves.
    rope = None
    if not args.path_only and w.head_dim % 32 == 0 and w.dtype == "bf16":
        n_pairs = w.head_dim // 2
        inv_freq = (1.0e6 ** (-np.arange(n_pairs, dtype=np.float64) / n_pairs)).astype(np.float32)
        axis = (np.arange(n_pairs) % 3).astype(np.int32)
        e = 2
        for s_ in sets:
            s_.cos_sin = torch.empty((w.batch, w.seq_compact, n_pairs, 2), dtype=torch.float32, device="cuda")
            s_.q_rot = torch.empty_like(s_.q)
        def rope_table(s_):
            bd.civic_mrope_table(s_.pos_c, axis, inv_freq, cos_sin=s_.cos_sin)
        def kv_rope(s_):
            bd.civic_kv_write_rope(s_.k, s_.v, s_.cos_sin, s_.k_cache, s_.v_cache, 0)
        def attn_rope(s_):
            bd.civic_prefill_attn_rope(s_.q, s_.k_cache.permute(0, 2, 1, 3), s_.v_cache.permute(0, 2, 1, 3), s_.cos_sin, w.causal,
                                       0.0, out=s_.out)
        def attn_cache(s_):
            bd.civic_prefill_attn(s_.q, s_.k_cache.permute(0, 2, 1, 3), s_.v_cache.permute(0, 2, 1, 3), w.causal, 0.0, out=s_.out)
        def apply_q(s_):
            bd.civic_mrope_apply(s_.q, s_.cos_sin, out=s_.q_rot)
        for s_ in sets:
            compact_call = calls["compact"]; compact_call(s_); rope_table(s_); kv_rope(s_)
        torch.cuda.synchronize()
        table_bytes = w.batch * w.seq_compact * n_pairs * 8
        t_table, t_kv, t_attn_rope, t_attn_cache, t_apply = (alone(f) for f in (rope_table, kv_rope, attn_rope, attn_cache, apply_q))
        kv_bytes = work["kv_write"] + table_bytes
        q_bytes = 2 * w.batch * w.seq_compact * w.n_q_heads * w.head_dim * e + table_bytes
        rope = {"table_us": round(t_table, 2),
                "kv_write_rope": {"us": round(t_kv, 2), "bytes": kv_bytes, "gbs": round(kv_bytes / t_kv / 1e3, 1),
                                  "frac_hbm_peak": round(kv_bytes / t_kv / 1e3 / HBM_PEAK_GBS, 4)},
                "prefill_attn_rope_us_back_to_back": round(t_attn_rope, 2),
                "prefill_attn_on_cache_us_back_to_back": round(t_attn_cache, 2),
                "mrope_apply_q": {"us": round(t_apply, 2), "bytes": q_bytes, "gbs": round(q_bytes / t_apply / 1e3, 1),
                                  "frac_hbm_peak": round(q_bytes / t_apply / 1e3 / HBM_PEAK_GBS, 4)}}

    # The path on a ragged batch (images of different grid sizes in one batch, packed along the token axis), on the
    # 8b-shaped workload's widths: eight samples from one 16 x 16 image to two 32 x 32 images.  The front runs its three
    # kernels sample by sample; the attention (with the KV write) is one launch, timed against one call per sample.
    ragged = None
    if not args.path_only and w.name == "8b":
        from paper_2605_28115_amd import workloads as wl_
        rgrids = [(1, 16, 16, 4, 4, 1, 0, 85), (1, 32, 32, 4, 4, 1, 0, 341), (2, 32, 32, 4, 4, 1, 0, 682), (1, 24, 24, 4, 4, 1, 0, 192),
                  (1, 32, 32, 4, 4, 1, 0, 341), (2, 24, 24, 4, 4, 1, 0, 384), (1, 16, 16, 4, 4, 1, 0, 85), (2, 32, 32, 4, 4, 1, 0, 682)]
        text = [32, 128, 256, 64, 96, 128, 16, 200]
        rstarts, rlens = [], []
        for g_, t_ in zip(rgrids, text):
            hw_ = g_[1] * g_[2]
            rstarts.append([t_ // 2 + f_ * hw_ for f_ in range(g_[0])]); rlens.append(t_ + g_[0] * hw_)
        rseq, rvis, rkept, rcomp = bd.civic_ragged_offsets(rlens, rgrids)
        rh = torch.randn((int(rseq[-1]), w.dim), device="cuda").to(sets[0].hidden.dtype)
        rp = torch.randint(0, 4096, (3, int(rseq[-1])), dtype=torch.int32, device="cuda")
        t_front = alone(lambda s_: bd.civic_compact_prefill_ragged(rh, rp, rlens, rgrids, rstarts, sets[0].anchor_q, 1.0), cost=3 * len(rgrids))
        tc = int(rcomp[-1])
        rq = torch.randn((tc, w.n_q_heads, w.head_dim), device="cuda").to(rh.dtype)
        rk = torch.randn((tc, w.n_kv_heads, w.head_dim), device="cuda").to(rh.dtype); rv = torch.randn_like(rk)
        ro = torch.empty_like(rq)
        smax_r = int(max(np.diff(rcomp)))
        rkc = torch.empty((len(rgrids), w.n_kv_heads, smax_r, w.head_dim), dtype=rh.dtype, device="cuda"); rvc = torch.empty_like(rkc)
        t_rattn = alone(lambda s_: bd.civic_prefill_attn_ragged(rq, rk, rv, rcomp, True, 0.0, rkc, rvc, 0, out=ro))
        def attn_per_sample(s_):
            for i_ in range(len(rgrids)):
                a_, b_ = int(rcomp[i_]), int(rcomp[i_ + 1])
                bd.civic_prefill_attn_kv(rq[a_:b_][None], rk[a_:b_][None], rv[a_:b_][None], rkc[i_:i_ + 1], rvc[i_:i_ + 1], 0, True, 0.0, out=ro[a_:b_][None])
        t_rattn_items = alone(attn_per_sample, cost=len(rgrids))
        # the decode step over the caches the ragged prefill has left: one context length per sample
        rctx = [int(n_) for n_ in np.diff(rcomp)]
        rdq = torch.randn((len(rgrids), w.n_q_heads, w.head_dim), device="cuda").to(rh.dtype)
        rdo = torch.empty_like(rdq)
        rws = torch.empty(max(16, int(bd.lib.civic_decode_attn_ragged_workspace_bytes(1, len(rctx), np.asarray(rctx, dtype=np.int32).ctypes.data,
                                                                                      w.n_q_heads, w.n_kv_heads, w.head_dim))), dtype=torch.uint8, device="cuda")
        t_rdec = alone(lambda s_: bd.civic_decode_attn_ragged(rdq, rkc, rvc, rctx, out=rdo, workspace=rws), cost=2)
        f_r = sum(4.0 * w.n_q_heads * w.head_dim * (n_ * (n_ + 1) / 2) for n_ in np.diff(rcomp))
        ragged = {"samples": len(rgrids), "dense_rows": int(rseq[-1]), "compact_rows": tc,
                  "compact_prefill_ragged_us": round(t_front, 2),
                  # scores 64 frame spans per launch, selection 16 samples per launch, merge 24 samples per launch (all have few frames)
                  "launches_front": -(-sum(g_[0] for g_ in rgrids) // 64) + -(-len(rgrids) // 16) + -(-len(rgrids) // 24),
                  "prefill_attn_ragged": {"us": round(t_rattn, 2), "us_one_call_per_sample": round(t_rattn_items, 2), "flops": f_r,
                                          "tflops": round(f_r / t_rattn / 1e6, 1)},
                  "decode_attn_ragged_us": round(t_rdec, 2)}

    # Encoder-side compaction (the paper's own soft route), timed on the encoder-shaped workload: Eq. 8 from the
    # dense patch grid to K anchors, and Eq. 9 (KV compression to S memory anchors + attention over them).
    encoder = None
    if not args.path_only and w.name == "vit":
        t_e, m_e, d_v, s_mem = w.n_visual, w.kept, w.dim, 256
        x0 = sets[0].hidden[:, :t_e].contiguous()
        anchors = torch.randn((m_e, d_v), device="cuda").to(x0.dtype)
        z0 = torch.empty((w.batch, m_e, d_v), dtype=x0.dtype, device="cuda")
        ws_a = torch.empty(int(bd.lib.civic_anchor_aggregate_workspace_bytes(w.batch, t_e, m_e, d_v)), dtype=torch.uint8, device="cuda")
        kq = sets[0].k[:, :m_e].contiguous(); vq = sets[0].v[:, :m_e].contiguous(); qq = sets[0].q[:, :m_e].contiguous()
        r = torch.rand((m_e, s_mem), device="cuda") ** 4
        kc = torch.empty((w.batch, s_mem, w.n_kv_heads, w.head_dim), dtype=x0.dtype, device="cuda"); vc = torch.empty_like(kc)
        ws_c = torch.empty(int(bd.lib.civic_kv_compress_workspace_bytes(w.batch, m_e, s_mem, w.n_kv_heads * w.head_dim)), dtype=torch.uint8, device="cuda")
        oc = torch.empty_like(qq)
        t_agg = alone(lambda s_: bd.civic_anchor_aggregate(x0, anchors, 14.0, z0=z0, workspace=ws_a))
        t_cmp = alone(lambda s_: bd.civic_kv_compress(kq, vq, r, k_c=kc, v_c=vc, workspace=ws_c))
        t_x = alone(lambda s_: bd.civic_cross_attn(qq, kc, vc, out=oc))
        t_full = alone(lambda s_: bd.civic_prefill_attn(qq, kq, vq, False, out=oc))
        # images of different grid sizes in one batch (packed rows): the Eq. 9 attention as one launch over all items,
        # against one rectangular call per item; the compression runs item by item either way
        sizes = [1365, 341, 85, 1024, 600, 341, 1365, 85]
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        qr = torch.randn((int(off[-1]), w.n_q_heads, w.head_dim), device="cuda").to(x0.dtype)
        kr = torch.randn((len(sizes), s_mem, w.n_kv_heads, w.head_dim), device="cuda").to(x0.dtype); vr = torch.randn_like(kr)
        outr = torch.empty_like(qr)
        t_rag = alone(lambda s_: bd.civic_cross_attn_ragged(qr, kr, vr, off, out=outr))
        def per_item(s_):
            for i in range(len(sizes)):
                bd.civic_cross_attn(qr[off[i]:off[i + 1]][None], kr[i:i + 1], vr[i:i + 1], out=outr[off[i]:off[i + 1]][None])
        t_items = alone(per_item, cost=len(sizes))
        width = w.n_kv_heads * w.head_dim
        kp = torch.randn((int(off[-1]), width), device="cuda").to(x0.dtype); vp = torch.randn_like(kp)
        rp = torch.rand((int(off[-1]), s_mem), device="cuda") ** 4
        kcr = torch.empty((len(sizes), s_mem, width), dtype=x0.dtype, device="cuda"); vcr = torch.empty_like(kcr)
        ws_r = torch.empty(int(bd.lib.civic_kv_compress_ragged_workspace_bytes(len(sizes), off.ctypes.data, s_mem, width)),
                           dtype=torch.uint8, device="cuda")
        t_cmp_rag = alone(lambda s_: bd.civic_kv_compress_ragged(kp, vp, rp, off, k_c=kcr, v_c=vcr, workspace=ws_r), cost=len(sizes))
        f_agg = 4.0 * m_e * t_e * d_v * w.batch
        f_cmp = 4.0 * s_mem * m_e * w.n_kv_heads * w.head_dim * w.batch
        f_x = 4.0 * w.n_q_heads * w.head_dim * m_e * s_mem * w.batch
        encoder = {"tokens": t_e, "anchors": m_e, "dim": d_v, "memory_anchors": s_mem,
                   "anchor_aggregate": {"us": round(t_agg, 2), "flops": f_agg, "tflops": round(f_agg / t_agg / 1e6, 1),
                                        "frac_mfma_peak": round(f_agg / t_agg / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
                                        "workspace_bytes": ws_a.numel(), "launches": 4},
                   "kv_compress": {"us": round(t_cmp, 2), "flops": f_cmp, "tflops": round(f_cmp / t_cmp / 1e6, 1)},
                   "cross_attn": {"us": round(t_x, 2), "flops": f_x, "tflops": round(f_x / t_x / 1e6, 1)},
                   "uncompressed_attn_us": round(t_full, 2),
                   "cross_attn_ragged": {"items": sizes, "us": round(t_rag, 2), "us_one_call_per_item": round(t_items, 2),
                                         "flops": 4.0 * w.n_q_heads * w.head_dim * float(off[-1]) * s_mem},
                   "kv_compress_ragged": {"items": sizes, "us": round(t_cmp_rag, 2), "flops": 4.0 * s_mem * float(off[-1]) * width}}

    # the selection runs once per prompt, the attention and the KV write once per layer: one measured step plus
    # layers - 1 further attention launches (in-step duration)
    per_layer_us = attn_us + (stage_us["kv_write"]["mean"] if args.unfused else 0.0)
    amortised_us = 1e3 * ms_per_step + (args.layers - 1) * per_layer_us
    result["amortised"] = {"layers": args.layers, "us": round(amortised_us, 2),
                           "tokens_per_s": round(tokens / (amortised_us * 1e-6), 1)}
    if decode is not None:
        result["decode"] = decode
    if rope is not None:
        result["rope"] = rope
    if ragged is not None:
        result["ragged"] = ragged
    if encoder is not None:
        result["encoder"] = encoder
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
