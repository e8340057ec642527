#!/usr/bin/env python3
"""Benchmark of the SPA hot path on one MI355X.

A step is one pass of the whole forward path (gate score + selection, index-only packing,
per-image attention on the selected tokens fetched through the index, scatter back - the last
two in one launch) over one seeded synthetic batch that is already resident in HBM.  The
headline workload is the detection-shaped batch, the largest single-GPU configuration (8
images x 4200 tokens, dim 256, 8 heads of 32, bf16, 5-40 % of the tokens selected per image):
it is the one whose attention sits above the ridge of the roofline, so its matrix-pipe fraction
means something.

Prints ONE JSON line: whole-path throughput in selected tokens/s (median over R repeats of the
timed K-step region), the roofline of the dominant kernel (durations measured live with events
on the launch stream), the CPU oracle timed on this machine's host cores, and a `configs` block
with the same measurements for every configuration: ViT-S-shaped forward, detection-shaped
forward, ViT-B-shaped forward + backward, four-stage hierarchy forward + backward.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
FP32_VECTOR_PEAK_TFLOPS = 157.3
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.txt")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--repeats", type=int, default=15,
                    help="the K-step region is timed this many times; median and min are reported")
    ap.add_argument("--workload", default="det", choices=["tiny", "vit_s", "det"], help="headline forward workload")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--streams", type=int, default=0,
                    help="independent batches in flight, one HIP stream each (1 = one stream, steps back to back; "
                         "0 = 2 or 4, whichever is faster on regions of --steps steps)")
    ap.add_argument("--only", default=None, choices=["forward", "vit_s", "det", "vit_b_train", "hierarchy"],
                    help="measure one chain only (profiling runs): forward = the headline workload's forward chain")
    ap.add_argument("--form", default="auto", choices=["auto", "selected", "fused", "gathered", "packed"],
                    help="forward step.  gathered: gate, index-only pack, attention on gathered rows (3 launches); "
                         "selected: gate, attention that takes the packing order from the mask itself (2 launches; "
                         "images of at most 256 tokens); auto (default): selected where it applies, else gathered; "
                         "fused: gate + packing index in one launch, attention on gathered rows (2 launches); packed: "
                         "gate, pack of the rows, attention on the packed rows (3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the four-call form, graph replay, padded baseline, widened rows")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--kernel-launches", type=int, default=200,
                    help="launches per kernel of the per-kernel timing passes (independent of --steps)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


# ------------------------------------------------------------------------------- timing
def timed(fn, steps, torch, streams=None):
    """K calls bracketed by synchronize on both sides -> seconds.  Where the calls went to several
    streams the closing bracket first waits for each of them in turn and then synchronizes the
    device: the same state when the clock is read, but a device-wide synchronize that finds four
    streams with work it has not yet waited for takes ~40 us longer to notice that they are done
    (measured on a 20-step region of the detection workload: 697 against 655 us)."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    for s in streams or ():
        s.synchronize()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def timed_polled(fn, steps, torch, streams):
    """The same K calls; the clock is stopped when events recorded behind the last launch of every
    stream read complete (polled), before the closing synchronize.  The blocking calls of the closing
    bracket of timed() put markers of their own behind the work and wait for those, ~40-60 us on this
    stack whatever the work was: a fixed cost that a 20-step region of a short step does not amortise.
    Reported beside the bracketed figure, never instead of it."""
    evs = [torch.cuda.Event() for _ in streams]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    for e, s in zip(evs, streams):
        e.record(s)
    for e in evs:
        while not e.query():
            pass
    dt = time.perf_counter() - t0
    torch.cuda.synchronize()
    return dt


def timed_regions(fn, steps, repeats, torch, streams=None):
    """The K-step region, timed `repeats` times (a 20-step region of a 20 us step lasts 0.4 ms
    and one reading of it carries the host's jitter): seconds per step, median and min."""
    per = [timed(fn, steps, torch, streams) / steps for _ in range(max(1, repeats))]
    return float(np.median(per)), float(np.min(per))


def per_stage_us(stage_sets, steps, torch):
    """Average duration of every stage, from event pairs recorded on the launch stream around
    each launch of the timed steps.  stage_sets: one list of (name, launch) per independent copy
    of the inputs and buffers; step i runs on copy i % len(stage_sets), so with enough copies every
    launch finds its inputs out of the last-level cache."""
    names = [n for n, _ in stage_sets[0]]
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in names]
          for _ in range(steps)]
    torch.cuda.synchronize()
    for s in range(steps):
        for i, (_, fn) in enumerate(stage_sets[s % len(stage_sets)]):
            a, b = ev[s][i]
            a.record()
            fn()
            b.record()
    torch.cuda.synchronize()
    return {n: 1e3 * float(np.mean([ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(steps)]))
            for i, n in enumerate(names)}


def back_to_back_us(fn, steps, torch):
    """Average duration of one launch when the same kernel is enqueued `steps` times between two
    events (no per-launch event overhead).  fn may be a list of launches of the same kernel on
    independent copies of its data, used round-robin."""
    fns = fn if isinstance(fn, (list, tuple)) else [fn]
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    for i in range(min(8, steps)):      # untimed: the first launches after an idle stretch read up to 2x slower
        fns[i % len(fns)]()
    a.record()
    for i in range(steps):
        fns[i % len(fns)]()
    b.record()
    torch.cuda.synchronize()
    return 1e3 * a.elapsed_time(b) / steps


def kernel_times_us(stage_sets, launches, torch):
    """Per launch, the kernel running alone on one stream: two live readings with HIP events on the
    launch stream, both upper bounds of the kernel's duration (an event pair around each launch
    inside steps of the whole chain, and back-to-back launches between one pair); the smaller."""
    steps = max(1, launches)     # (not the K of the timed region: a pair of events around 20 launches still reads the start-up)
    ev = per_stage_us(stage_sets, steps, torch)
    out = {}
    for i, (name, _) in enumerate(stage_sets[0]):
        b2b = back_to_back_us([cs[i][1] for cs in stage_sets], steps, torch)
        out[name] = {"event_us": round(ev[name], 2), "back_to_back_us": round(b2b, 2),
                     "kernel_us": round(min(ev[name], b2b), 2)}
    return out


def ceilings(spa, torch):
    """Achievable ceilings measured on this machine with the library's yardstick kernels: a plain
    streaming copy whose buffers rotate through 1 GiB (every launch misses the last-level cache)
    and an MFMA-only loop."""
    nbuf, nbytes = 8, 64 << 20
    src = [torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1) for _ in range(nbuf)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(nbuf)]
    copies = [spa.spa_ceiling_copy(a, b, prepare=True) for a, b in zip(src, dst)]
    for c in copies:
        c()
    us = back_to_back_us(copies, 64, torch)
    copy_gbs = 2.0 * nbytes / us / 1e3
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    best = 0.0
    for wps in (1, 2):
        flops = spa.spa_ceiling_mfma(sink, wps, 4096)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            spa.spa_ceiling_mfma(sink, wps, 4096)
        b.record()
        torch.cuda.synchronize()
        best = max(best, 5 * flops / (a.elapsed_time(b) * 1e-3) / 1e12)
    del src, dst
    return {"copy_GBs": round(copy_gbs, 1), "copy": "64 MiB read + 64 MiB written per launch, 8 buffer pairs in rotation",
            "mfma_bf16_TFLOPs": round(best, 1),
            "mfma": "v_mfma_f32_32x32x16_bf16 only, 4 chains per wave, best of 1 and 2 waves per SIMD"}


def graph_replay_s(make_step, steps, torch):
    """Capture one step (prepared on the capture stream) into a hipGraph and time replays."""
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run = make_step()
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        run()
    for _ in range(3):
        g.replay()
    return timed(g.replay, steps, torch)


# ----------------------------------------------------------------------------- rooflines
def load_traffic_table():
    """HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs, as the committed table
    under profiles/ holds them (written by `python -m paper_2410_23608_amd.profiling`)."""
    table = {}
    if os.path.exists(TRAFFIC_TABLE):
        for line in open(TRAFFIC_TABLE):
            f = line.split()
            if len(f) >= 3 and not line.startswith("#"):
                table[(f[0], f[1])] = float(f[2])
    return table


def roofline_entry(name, us, flops, nbytes, dtype, traffic):
    """The roof that bounds a launch, chosen by operational intensity: below the ridge (peak flop
    rate / peak bandwidth) the HBM roof is the lower one."""
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if dtype == "bf16" else FP32_VECTOR_PEAK_TFLOPS
    ridge = mfma_peak * 1e12 / (HBM_PEAK_GBS * 1e9)
    intensity = flops / nbytes
    if intensity < ridge:
        bound, ach, peak, unit = "hbm", nbytes / us / 1e3, HBM_PEAK_GBS, "GB/s"
    else:
        bound, ach, peak, unit = ("mfma" if dtype == "bf16" else "alu"), flops / us / 1e6, mfma_peak, "TFLOP/s"
    r = {"kernel": name, "bound": bound, "achieved": round(ach, 2), "peak": peak, "unit": unit,
         "frac": round(ach / peak, 4), "avg_launch_us": us, "algorithmic_bytes": int(nbytes),
         "algorithmic_flops": flops, "flop_per_byte": round(intensity, 1), "ridge_flop_per_byte": round(ridge, 1),
         "traffic": traffic,
         "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated; from "
                         "profiles/hbm_traffic_table.txt)"}
    if flops > 0:
        r["tflops"] = round(flops / us / 1e6, 2)
        r["mfma_frac"] = round(flops / us / 1e6 / mfma_peak, 4)
        r["hbm_frac"] = round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)
    return r


def kernels_block(times, work, dtype, wl_name, traffic_table, seed):
    """times: name -> {kernel_us, ...}; work: name -> (flops, bytes).  Returns the per-kernel table
    and the roofline of the dominant (longest) kernel."""
    out = {}
    for name, t in times.items():
        if name not in work:
            out[name] = t
            continue
        fl, by = work[name]
        traffic = traffic_table.get((wl_name, name)) if seed == 0 else None
        r = roofline_entry(name, t["kernel_us"], fl, by, dtype, traffic)
        r.update(t)
        out[name] = r
    scored = [n for n in out if "frac" in out[n]]
    dom = max(scored, key=lambda n: out[n]["kernel_us"])
    return out, dict(out[dom])


# ------------------------------------------------------------------------ forward chain
def forward_work(wl, T, sum_n2, keep_out=False):
    """Algorithmic (flops, bytes) per launch of the forward kernels."""
    B, N, C, H = wl.B, wl.N, wl.C, wl.H
    e = 2 if wl.dtype == "bf16" else 4
    attn = (4.0 * C * sum_n2, T * 3 * C * e + B * N * C * e + 4 * T + 4 * B * N + 4 * (B + 1)
            + (T * C * e + 4 * H * T if keep_out else 0))
    return {
        "gate_select": (0.0, B * N * (C * e + 5)),
        "gate_select_index": (0.0, B * N * (C * e + 5) + 4 * T + 5 * B * N + 4 * (B + 1)),
        "pack": (0.0, 2 * T * 3 * C * e + 4 * T + 5 * B * N + 4 * (B + 1)),
        "pack_indices": (0.0, 4 * T + 5 * B * N + 4 * (B + 1)),
        "packed_attention_unpack": attn, "gathered_attention_unpack": attn,
        # no index arrays: the mask bytes are read instead (once per query block and head; counted once)
        "selected_attention_unpack": (attn[0], attn[1] - 4 * T - 4 * B * N - 4 * (B + 1) + B * N),
        "packed_attention": (4.0 * C * sum_n2, T * 3 * C * e + T * C * e + 4 * H * T + 4 * (B + 1)),
        "unpack": (0.0, T * C * e + 4 * B * N + B * N * C * e),
    }


def forward_form(requested, wl):
    """The form a forward workload is timed in: `selected` needs images of at most 256 tokens."""
    fits = wl.N <= 256
    if requested == "auto":
        return "selected" if fits else "gathered"
    if requested == "selected" and not fits:
        return "gathered"
    return requested


def measure_forward(wl, args, torch, workloads, ForwardPass, traffic_table, streams_cache):
    """Forward chain of one workload: S batches in flight (cold rotation), one stream, per kernel."""
    td = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    e = 2 if wl.dtype == "bf16" else 4
    bun = workloads.generate(wl, args.seed)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(td).contiguous()
    x, w, qkv = up(bun["x"]), up(bun["w"]), up(bun["qkv"])
    form = forward_form(args.form, wl)
    gathered = form in ("gathered", "fused", "selected")
    mk = lambda: ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, wl.bias, keep_packed_out=False,
                             gathered=gathered, fused_index=form == "fused", from_mask=form == "selected")
    fp = mk()
    stages = fp.stages(x, w, qkv)

    def step():
        for _, fn in stages:
            fn()

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    n = fp.mask.sum(dim=1).cpu().numpy().astype(np.float64)      # (the selected form writes no cu_seqlens / total)
    T = int(n.sum())
    sum_n2 = float((n * n).sum())

    # one stream, steps back to back on ONE copy of the batch (warm last-level cache): the latency of a step
    s_med, s_min = timed_regions(step, args.steps, args.repeats, torch)
    single = {"ms_per_step": 1e3 * s_med, "ms_per_step_min": 1e3 * s_min, "value": T / s_med,
              "unit": "selected tokens/s", "cache": "warm (one copy of the batch, reused every step)"}

    # S independent batches in flight: S HIP streams (default priority), steps dealt round-robin, the
    # launches of a step in order on their stream; every step works on its own copy of the inputs and
    # buffers, enough copies (> 512 MB in total) that no step finds anything in the last-level cache
    set_bytes = (x.numel() + qkv.numel() + (0 if gathered else fp.packed_qkv.numel()) + fp.y.numel()) * e
    cfg = {"S": 1, "n_sets": 2}
    turn = [0]
    holder = {}

    def configure(S_):
        cfg["S"] = S_
        cfg["n_sets"] = S_ * max(2, -(-(512 << 20) // (S_ * set_bytes)))

    def build_sets(streams_):
        made = []
        for i in range(cfg["n_sets"]):
            with torch.cuda.stream(streams_[i % cfg["S"]]):
                fp_s = mk()
                ins = (x.clone(), w.clone(), qkv.clone())
                made.append((fp_s, fp_s.stages(*ins), ins))
        torch.cuda.synchronize()
        return made

    def sstep():   # step i -> copy i % n_sets, which lives on stream i % S
        for _, fn in holder["sets"][turn[0] % cfg["n_sets"]][1]:
            fn()
        turn[0] += 1

    # Which HIP streams end up sharing one of the process's hardware queues (4 here) is the runtime's
    # business, and two batches on one queue run one after the other: three groups of S streams are
    # tried for a few hundred untimed steps each and the fastest group is kept (once per process and S).
    calib = {}

    def streams_for(S_):
        if S_ == 1:
            return [torch.cuda.current_stream()]
        if ("streams", S_) not in streams_cache:
            best = None
            for gi_ in range(3):
                cand = [torch.cuda.Stream() for _ in range(S_)]
                holder["sets"] = build_sets(cand)
                for _ in range(cfg["n_sets"]):
                    sstep()
                torch.cuda.synchronize()
                turn[0] = 0
                probe = timed(sstep, 300, torch, cand) / 300
                calib[f"S{S_}_group_{gi_}_us_per_step"] = round(1e6 * probe, 2)
                if best is None or probe < best[0]:
                    best = (probe, cand)
                holder["sets"] = None
            streams_cache[("streams", S_)] = best[1]
        return streams_cache[("streams", S_)]

    def ready(S_):
        """Copies built on the chosen streams of S_ batches in flight, warmed up; returns the streams."""
        configure(S_)
        streams_ = streams_for(S_)
        holder["sets"] = build_sets(streams_)
        for _ in range(max(args.warmup, cfg["n_sets"])):
            sstep()
        torch.cuda.synchronize()
        turn[0] = 0
        return streams_

    # How many batches to keep in flight depends on the length of the timed region: a region of K steps
    # starts and ends with the streams' pipelines filling and draining, which costs more the more
    # streams there are (200-step regions of the detection workload: 4 streams 31.5 us per step, 2
    # streams 33.3; 20-step regions: 36.9 and 35.1).  --streams 0 (the default) times a few regions
    # of the K steps asked for with 2 and with 4 batches in flight and keeps the better.
    if args.streams > 0:
        S = args.streams
    else:
        probes = {}
        for S_ in (2, 4):
            streams_ = ready(S_)
            probes[S_] = timed_regions(sstep, args.steps, 7, torch, streams_)[0]
            calib[f"S{S_}_us_per_step_at_{args.steps}_steps"] = round(1e6 * probes[S_], 2)
            holder["sets"] = None
        S = min(probes, key=probes.get)
    streams = ready(S)
    sets, n_sets = holder["sets"], cfg["n_sets"]
    med, mn = timed_regions(sstep, args.steps, args.repeats, torch, streams)
    if not all(torch.equal(fs.y, fp.y) and int(fs.mask.sum().item()) == T for fs, _, _ in sets):
        print("bench.py: a copy's result differs from the single-stream result", file=sys.stderr)
        sys.exit(1)

    polled = [timed_polled(sstep, args.steps, torch, streams) / args.steps for _ in range(max(1, args.repeats))]

    # per-kernel durations: the copies of the timed region on ONE stream, in rotation (cold)
    cold_sets = [fs.stages(*ins) for fs, _, ins in sets]
    times = kernel_times_us(cold_sets, args.kernel_launches, torch)
    warm = {nme: back_to_back_us(fn, args.kernel_launches, torch) for nme, fn in stages}
    for nme in times:
        times[nme]["warm_cache_us"] = round(warm[nme], 2)
    kernels, roof = kernels_block(times, forward_work(wl, T, sum_n2), wl.dtype, wl.name, traffic_table, args.seed)
    roof["cache"] = f"cold: {n_sets} copies of the batch and its buffers in rotation ({n_sets * set_bytes >> 20} MB)"
    # context beside `achieved` (the launch alone on one stream): the same algorithmic work over the
    # whole step of the timed region, where the launches of S batches share the GPU
    if roof.get("algorithmic_flops", 0) > 0:
        peak = MFMA_BF16_PEAK_TFLOPS if wl.dtype == "bf16" else FP32_VECTOR_PEAK_TFLOPS
        roof["tflops_over_step"] = round(roof["algorithmic_flops"] / med / 1e12, 2)
        roof["mfma_frac_over_step"] = round(roof["algorithmic_flops"] / med / 1e12 / peak, 4)
    res = {
        "workload": f"{wl.name}: B={wl.B} N={wl.N} C={wl.C} H={wl.H} Dh={wl.Dh} {wl.dtype}, selected fraction "
                    f"U[{wl.frac[0]},{wl.frac[1]}] per image, forward select+pack+attention+unpack",
        "selected_tokens": T, "sum_n2": sum_n2, "value": T / med, "unit": "selected tokens/s",
        "ms_per_step": 1e3 * med, "ms_per_step_min": 1e3 * mn, "regions": args.repeats,
        "ms_per_step_until_last_event": 1e3 * float(np.median(polled)),
        "launch": f"eager, {len(stages)} launches per step ({' + '.join(n_ for n_, _ in stages)}); {S} independent "
                  f"batches in flight on {S} HIP stream(s); {n_sets} copies of the inputs and buffers in rotation "
                  f"({n_sets * set_bytes >> 20} MB, cold last-level cache)",
        "streams": S, "copies": n_sets, "single_stream": single, "kernels": kernels, "roofline": roof,
    }
    if calib:
        res["stream_group_calibration"] = calib
    del sets, cold_sets
    holder["sets"] = None
    return res, dict(bun=bun, x=x, w=w, qkv=qkv, fp=fp, stages=stages, T=T, n=n, sum_n2=sum_n2, streams=streams)


# ------------------------------------------------------------------- forward + backward
def train_work(B, N, C, H, T, sum_n2, prefix="", bwd_executed_over_algorithmic=1.0):
    e = 2
    return {
        prefix + "gate_select": (0.0, B * N * (C * e + 5)),
        prefix + "gate_select_pooled": (0.0, B * N * (C * e + 5 + 16)),
        prefix + "pack_qk_rg": (0.0, 2 * T * 3 * C * e + 8 * T + 5 * B * N + 4 * (B + 1)),
        prefix + "packed_attention_unpack": (4.0 * C * sum_n2, T * 3 * C * e + B * N * C * e + 4 * T + 4 * B * N
                                             + 4 * (B + 1) + T * C * e + 4 * H * T),
        # reads q, k, v, out rows and dy at the selected positions; writes dq | dk and d_rg at ALL token positions
        prefix + "packed_attention_bwd_tokens": (10.0 * C * sum_n2, 5 * T * C * e + 3 * B * N * C * e + 4 * H * T
                                                 + 8 * B * N),
        prefix + "gate_bwd": (0.0, B * N * (3 * C * e + 9) + 8 * C),
    }


def measure_train(args, torch, workloads, TrainPass, traffic_table, streams):
    """ViT-B-shaped training step: forward + backward with the selection loss, 5 calls."""
    wl = workloads.WORKLOADS["vit_b_train"]
    B, N, C, H = wl.B, wl.N, wl.C, wl.H
    td = torch.bfloat16
    tb = workloads.generate(wl, args.seed)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(td).contiguous()
    tx, tw, tqk, tdy = up(tb["x"]), up(tb["w"]), up(tb["qkv"][:, :, :2 * C]), up(tb["dy"])
    tlab = torch.from_numpy(tb["labels"]).cuda()
    tp = TrainPass(B, N, C, H, wl.dtype, wl.tau, wl.bias)
    stages = tp.stages(tx, tw, tqk, tlab, tdy)

    def step():
        for _, fn in stages:
            fn()

    for _ in range(max(5, args.warmup // 4)):
        step()
    torch.cuda.synchronize()
    T = int(tp.total.item())
    n = np.diff(tp.cu_seqlens.cpu().numpy()).astype(np.float64)
    sum_n2 = float((n * n).sum())
    med, mn = timed_regions(step, args.steps, args.repeats, torch)
    times = kernel_times_us([stages], args.kernel_launches, torch)
    kernels, roof = kernels_block(times, train_work(B, N, C, H, T, sum_n2), wl.dtype, wl.name, traffic_table, args.seed)
    res = {"workload": f"vit_b_train: B={B} N={N} C={C} H={H} Dh={wl.Dh} bf16, selected fraction "
                       f"U[{wl.frac[0]},{wl.frac[1]}] per image, forward + backward with the selection loss",
           "selected_tokens": T, "sum_n2": sum_n2, "value": T / med, "unit": "selected tokens/s",
           "ms_per_step": 1e3 * med, "ms_per_step_min": 1e3 * mn, "regions": args.repeats,
           "launch": f"eager, one stream, {len(stages)} calls per step ({' + '.join(n_ for n_, _ in stages)}), warm cache",
           "kernels": kernels, "roofline": roof,
           "attention_bwd_tflops": kernels["packed_attention_bwd_tokens"].get("tflops")}
    S = len(streams)
    if S > 1:   # the training step with S batches in flight, like the forward headline
        tsets = []
        for s_ in streams:
            with torch.cuda.stream(s_):
                tp_s = TrainPass(B, N, C, H, wl.dtype, wl.tau, wl.bias)
                tsets.append((tp_s, tp_s.stages(tx.clone(), tw.clone(), tqk.clone(), tlab.clone(), tdy.clone())))
        torch.cuda.synchronize()
        turn = [0]

        def tsstep():
            for _, fn in tsets[turn[0] % S][1]:
                fn()
            turn[0] += 1

        for _ in range(2 * S):
            tsstep()
        torch.cuda.synchronize()
        turn[0] = 0
        smed, smin = timed_regions(tsstep, args.steps, args.repeats, torch, streams)
        same = all(torch.equal(ts.dx, tp.dx) and torch.equal(ts.dw, tp.dw) for ts, _ in tsets)
        res["batches_in_flight"] = {"streams": S, "value": T / smed, "ms_per_step": 1e3 * smed,
                                    "ms_per_step_min": 1e3 * smin, "gradients_equal_single_stream": bool(same)}
    return res


def measure_hierarchy(args, torch, workloads, HierarchyPass, HierarchyTrainPass, traffic_table):
    """Four-stage hierarchy (batch 16, 56^2 .. 7^2 tokens, C 96 .. 768): forward chain (12 launches)
    and forward + backward chain (20 calls); per-kernel rooflines, dominant = the finest stage's."""
    hb = workloads.generate_hierarchy(args.seed)
    td = torch.bfloat16
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(td).contiguous()
    hcfg = [(b_["workload"].B, *b_["workload"].grid, b_["workload"].C, b_["workload"].H, b_["workload"].dtype,
             b_["workload"].tau, b_["bias"]) for b_ in hb]
    hx, hw, hq = [up(b_["x"]) for b_ in hb], [up(b_["w"]) for b_ in hb], [up(b_["qkv"]) for b_ in hb]
    hp = HierarchyPass(hcfg, lean=True)
    hstages = hp.stages(hx, hw, hq)

    def hstep():
        for _, fn in hstages:
            fn()

    for _ in range(5):
        hstep()
    torch.cuda.synchronize()
    hT = [int(p_.mask.sum().item()) for p_ in hp.passes]
    fmed, fmin = timed_regions(hstep, args.steps, args.repeats, torch)
    res = {"workload": "hierarchy: B=16, stages of 56^2/28^2/14^2/7^2 tokens, C=96/192/384/768, heads 3/6/12/24 of 32, "
                       "bf16, every stage's gate takes the finer stage's score map (max-pooled in the gate kernel)",
           "stages": [b_["workload"].name for b_ in hb], "tokens": [c_[0] * c_[1] * c_[2] for c_ in hcfg],
           "forward": {"launches": len(hstages), "selected_tokens": hT, "value": sum(hT) / fmed,
                       "unit": "selected tokens/s", "ms_per_step": 1e3 * fmed, "ms_per_step_min": 1e3 * fmin,
                       "stage_us": {nme: round(back_to_back_us(fn, args.kernel_launches, torch), 2)
                                    for nme, fn in hstages}}}
    htp = HierarchyTrainPass(hcfg)
    hqk = [up(b_["qkv"][:, :, :2 * b_["workload"].C]) for b_ in hb]
    hlab = [torch.from_numpy(b_["labels"]).cuda() for b_ in hb]
    hdy = [up(b_["dy"]) for b_ in hb]
    htstages = htp.stages(hx, hw, hqk, hlab, hdy)

    def htstep():
        for _, fn in htstages:
            fn()

    for _ in range(5):
        htstep()
    torch.cuda.synchronize()
    htT = [int(p_.total.item()) for p_ in htp.passes]
    med, mn = timed_regions(htstep, args.steps, args.repeats, torch)
    times = kernel_times_us([htstages], args.kernel_launches, torch)
    work, sum_n2s = {}, []
    for i, (b_, tp_) in enumerate(zip(hb, htp.passes)):
        wl_ = b_["workload"]
        n = np.diff(tp_.cu_seqlens.cpu().numpy()).astype(np.float64)
        sum_n2s.append(float((n * n).sum()))
        work.update(train_work(wl_.B, wl_.N, wl_.C, wl_.H, htT[i], sum_n2s[-1], prefix=f"s{i + 1}."))
    kernels, roof = kernels_block(times, work, "bf16", "hierarchy", traffic_table, args.seed)
    res.update({"selected_tokens": htT, "sum_n2": sum_n2s, "value": sum(htT) / med, "unit": "selected tokens/s",
                "ms_per_step": 1e3 * med, "ms_per_step_min": 1e3 * mn, "regions": args.repeats,
                "launch": f"eager, one stream, {len(htstages)} calls per forward + backward chain, warm cache",
                "kernels": kernels, "roofline": roof})
    htpc = HierarchyTrainPass(hcfg, concurrent=True)
    htcstages = htpc.stages(hx, hw, hqk, hlab, hdy)

    def htcstep():
        for _, fn in htcstages:
            fn()

    for _ in range(5):
        htcstep()
    torch.cuda.synchronize()
    cmed, cmin = timed_regions(htcstep, args.steps, args.repeats, torch)
    res["stream_per_stage"] = {
        "ms_per_step": 1e3 * cmed, "ms_per_step_min": 1e3 * cmin, "value": sum(htT) / cmed,
        "gradients_equal_one_stream": bool(all(torch.equal(a_.dx, b_.dx) and torch.equal(a_.dw, b_.dw)
                                               for a_, b_ in zip(htpc.passes, htp.passes)))}
    return res


# ------------------------------------------------------------------------------- extras
def measure_extras(wl, ctx, args, torch, spa, workloads, pipeline):
    """On the headline workload: the four-call form of the boundary, the other forward form, hipGraph
    replay, the padded-to-max baseline; on the ViT-S-shaped batch the widened rows (block with
    projections forward and forward + backward, container-local attention)."""
    out = {}
    td = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    B, N, C, H = wl.B, wl.N, wl.C, wl.H
    x, w, qkv, fp, T, n, sum_n2 = ctx["x"], ctx["w"], ctx["qkv"], ctx["fp"], ctx["T"], ctx["n"], ctx["sum_n2"]
    steps = max(20, min(args.steps, 200))
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if wl.dtype == "bf16" else FP32_VECTOR_PEAK_TFLOPS

    def run_chain(stages_):
        def go():
            for _, fn in stages_:
                fn()
        for _ in range(5):
            go()
        torch.cuda.synchronize()
        return timed_regions(go, steps, 5, torch)[0]

    # the hot path as its four calls (gate_select, pack of the rows, packed_attention, unpack), nothing fused
    fp4 = pipeline.ForwardPass(B, N, C, H, wl.dtype, wl.tau, wl.bias, fused_unpack=False)
    st4 = fp4.stages(x, w, qkv)
    med4 = run_chain(st4)
    work4 = forward_work(wl, T, sum_n2)
    four = {}
    for nme, fn in st4:
        us_ = back_to_back_us(fn, steps, torch)
        fl, by = work4[nme]
        four[nme] = {"us": round(us_, 2), "GB/s": round(by / us_ / 1e3, 1),
                     "hbm_frac": round(by / us_ / 1e3 / HBM_PEAK_GBS, 4)}
        if fl > 0:
            four[nme].update({"tflops": round(fl / us_ / 1e6, 2), "mfma_frac": round(fl / us_ / 1e6 / mfma_peak, 4)})
    out["four_call_form"] = {"ms_per_step": 1e3 * med4, "value": T / med4,
                             "cache": "warm (one copy of the batch, one stream)",
                             "y_equals_headline_form": bool(torch.equal(fp4.y, fp.y)), "kernels": four}
    # the other forward forms (rows copied by the pack launch / fetched through the index / index built by the gate launch)
    timed_form = forward_form(args.form, wl)
    for other in ("selected", "fused", "gathered", "packed"):
        if other == timed_form or forward_form(other, wl) != other:
            continue
        fpo = pipeline.ForwardPass(B, N, C, H, wl.dtype, wl.tau, wl.bias, keep_packed_out=False,
                                   gathered=other != "packed", fused_index=other == "fused",
                                   from_mask=other == "selected")
        sto = fpo.stages(x, w, qkv)
        medo = run_chain(sto)
        out[f"{other}_form"] = {"ms_per_step": 1e3 * medo, "value": T / medo, "cache": "warm, one stream",
                                "launches": [n_ for n_, _ in sto], "y_equals_headline_form": bool(torch.equal(fpo.y, fp.y)),
                                "stage_us": {nme: round(back_to_back_us(fn, steps, torch), 2) for nme, fn in sto}}
    # the headline step replayed as a hipGraph
    try:
        def make_step():
            st = fp.stages(x, w, qkv)
            return lambda: [fn() for _, fn in st]
        gdt = graph_replay_s(make_step, steps, torch)
        out["graph_replay"] = {"ms_per_step": 1e3 * gdt / steps, "value": T * steps / gdt}
    except Exception as ex:  # capture refused: report, do not hide
        out["graph_replay"] = {"error": str(ex)[:200]}
    # padded-to-max masked attention on the same selected tokens
    n_max = int(n.max())
    cu = fp4.cu_seqlens.cpu().numpy()                     # (the four-call pass above always builds the index)
    gidx = fp4.gather_idx.cpu().numpy()
    flat_qkv = qkv.view(B * N, 3 * C)
    packed = flat_qkv[torch.from_numpy(gidx[:T].astype(np.int64)).cuda()].contiguous()   # setup of the padded inputs only
    pad = torch.zeros(B, n_max, 3 * C, dtype=td, device="cuda")
    for b in range(B):
        pad[b, :cu[b + 1] - cu[b]] = packed[cu[b]:cu[b + 1]]
    lens = torch.from_numpy(np.diff(cu).astype(np.int32)).cuda()
    pout = torch.empty(B, n_max, C, dtype=td, device="cuda")
    flat = pad.view(B * n_max, 3 * C)
    pfn = spa.spa_padded_attention(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], lens, B, n_max, H, wl.Dh, pout,
                                   prepare=True)
    lens_full = torch.full((B,), n_max, dtype=torch.int32, device="cuda")
    dfn = spa.spa_padded_attention(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], lens_full, B, n_max, H, wl.Dh, pout,
                                   prepare=True)
    aout = torch.empty(B * N, C, dtype=td, device="cuda")
    afn = spa.spa_packed_attention(packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:], fp4.cu_seqlens, B, N, H, wl.Dh,
                                   aout, None, prepare=True)
    for f_ in (pfn, dfn, afn):
        f_()
    pus, dus, aus = (back_to_back_us(f_, steps, torch) for f_ in (pfn, dfn, afn))
    out["padded_baseline"] = {
        "n_max": n_max, "packed_attention_us": round(aus, 2),
        "padded_dense_us": round(dus, 2), "speedup_over_padded_dense": round(dus / aus, 3),
        "padded_dense": "every image padded to n_max queries AND n_max keys (B n_max^2 scores): what padding to the "
                        "batch maximum costs",
        "work_ratio_B_nmax2_over_sum_n2": round(B * n_max * n_max / sum_n2, 3),
        "padded_skipping_masked_keys_us": round(pus, 2), "speedup_over_padded_skipping": round(pus / aus, 3),
        "padded_skipping_masked_keys": "n_max queries per image, but keys past the image's length are skipped instead "
                                       "of masked (sum n_max n_b scores): a length-aware padded kernel",
        "work_ratio_nmax_sum_n_over_sum_n2": round(n_max * float(n.sum()) / sum_n2, 3)}
    if wl.dtype != "bf16":
        return out

    # widened rows, on the ViT-S-shaped batch (their shapes are the classification ones)
    vwl = workloads.WORKLOADS["vit_s"]
    vb = workloads.generate(vwl, args.seed)
    vup = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(torch.bfloat16).contiguous()
    vx, vw, vqkv = vup(vb["x"]), vup(vb["w"]), vup(vb["qkv"])
    VB, VN, VC, VH = vwl.B, vwl.N, vwl.C, vwl.H
    g = torch.Generator(device="cpu").manual_seed(args.seed + 17)
    mkw = lambda r, c: (torch.randn(r, c, generator=g) / c ** 0.5).cuda().to(torch.bfloat16)
    W_qkv, b_qkv, W_o, b_o = mkw(3 * VC, VC), mkw(1, 3 * VC).view(-1), mkw(VC, VC), mkw(1, VC).view(-1)
    bp = pipeline.BlockPass(VB, VN, VC, VH, "bf16", vwl.tau, vwl.bias)
    bstages = bp.stages(vx, vw, W_qkv, b_qkv, W_o, b_o)
    bmed = run_chain(bstages)
    vT = int(bp.total.item())
    bus = {nme: back_to_back_us(fn, steps, torch) for nme, fn in bstages}
    out["block_with_projections"] = {
        "workload": "vit_s", "launches": [n_ for n_, _ in bstages], "value": vT / bmed, "unit": "selected tokens/s",
        "ms_per_step": 1e3 * bmed, "stage_us": {k_: round(v_, 2) for k_, v_ in bus.items()},
        "qkv_projection_tflops": round(2.0 * vT * VC * 3 * VC / bus["qkv_projection"] / 1e6, 1),
        "out_projection_tflops": round(2.0 * vT * VC * VC / bus["out_projection"] / 1e6, 1),
        "dense_projection_flops_saved": round(1.0 - vT / (VB * VN), 3)}
    dy_blk = torch.randn(VB, VN, VC, generator=g).cuda().to(torch.bfloat16)
    lab_blk = torch.from_numpy(vb["labels"]).cuda()
    blk_train = {}
    for key, ov in (("two_streams", True), ("one_stream", False)):
        btp = pipeline.BlockTrainPass(VB, VN, VC, VH, "bf16", vwl.tau, vwl.bias, overlap_weight_grads=ov)
        tst = btp.stages(vx, vw, W_qkv, b_qkv, W_o, b_o, lab_blk, dy_blk)
        tmed = run_chain(tst)
        blk_train[key] = {"ms_per_step": 1e3 * tmed, "value": vT / tmed, "unit": "selected tokens/s"}
        if not ov:
            blk_train[key]["launches"] = [n_ for n_, _ in tst]
            blk_train[key]["stage_us"] = {nme: round(back_to_back_us(fn, steps, torch), 2) for nme, fn in tst}
    out["block_with_projections"]["fwd_bwd"] = blk_train
    # the paper's container mask: containers of L = 7^2 tokens, map shifted by (3, 3)
    side = int(round(VN ** 0.5))
    cp = pipeline.ContainerForwardPass(VB, side, side, VC, VH, "bf16", 49, (3, 3), vwl.tau, vwl.bias)
    cstages = cp.stages(vx, vw, vqkv)
    cmed = run_chain(cstages)
    cus = {nme: back_to_back_us(fn, steps, torch) for nme, fn in cstages}
    seg = cp.seg_cu_seqlens.cpu().numpy().astype(np.float64)
    seg_n2 = float((np.diff(seg) ** 2).sum())
    out["container_local"] = {
        "workload": "vit_s", "container_len": 49, "shift": [3, 3], "segments": int(cp.n_segments.item()),
        "segment_capacity": cp.seg_cap, "sum_n2": seg_n2, "value": vT / cmed, "unit": "selected tokens/s",
        "ms_per_step": 1e3 * cmed, "stage_us": {k_: round(v_, 2) for k_, v_ in cus.items()},
        "attention_tflops": round(4.0 * VC * seg_n2 / cus["segment_attention_unpack"] / 1e6, 2)}
    return out


def cpu_oracle_baseline(wl, bundle, seconds):
    """The oracle as it stands, timed on this machine's host cores on the same batch."""
    from oracle import spa_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    reps, tokens = 0, 0
    t0 = time.perf_counter()
    while True:
        r = orc.spa_forward(bundle["x"], bundle["w"], bundle["bias"], bundle["qkv"], wl.H, wl.tau, wl.dtype)
        reps += 1
        tokens += r["total"]
        dt = time.perf_counter() - t0
        if dt >= seconds:
            break
    return {"value": tokens / dt, "unit": "selected tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{reps} full forward passes of the {wl.name} batch (NumPy fp64, {dt:.1f} s)"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2410_23608_amd import pipeline, spa, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.calibration_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    traffic_table = load_traffic_table()
    streams_cache = {}
    fwd = lambda name: measure_forward(workloads.WORKLOADS[name], args, torch, workloads, pipeline.ForwardPass,
                                       traffic_table, streams_cache)
    if args.only is not None:      # one chain only (profiling runs): a short line, same fields
        if args.only in ("forward", "vit_s", "det"):
            res, _ = fwd(args.workload if args.only == "forward" else args.only)
        elif args.only == "vit_b_train":
            res = measure_train(args, torch, workloads, pipeline.TrainPass, traffic_table, [torch.cuda.current_stream()])
        else:
            res = measure_hierarchy(args, torch, workloads, pipeline.HierarchyPass, pipeline.HierarchyTrainPass,
                                    traffic_table)
        print(json.dumps({"only": args.only, **res}))
        return

    wl = workloads.WORKLOADS[args.workload]
    head, ctx = fwd(args.workload)
    configs = {args.workload: head}
    if wl.dtype == "bf16":
        for name in ("tiny", "vit_s", "det"):
            if name not in configs:
                configs[name], _ = fwd(name)
        configs["vit_b_train"] = measure_train(args, torch, workloads, pipeline.TrainPass, traffic_table, ctx["streams"])
        configs["hierarchy"] = measure_hierarchy(args, torch, workloads, pipeline.HierarchyPass,
                                                 pipeline.HierarchyTrainPass, traffic_table)
    ceil_ = ceilings(spa, torch)
    roof = dict(head["roofline"])
    measured = ceil_["copy_GBs"] if roof["bound"] == "hbm" else ceil_["mfma_bf16_TFLOPs"]
    roof["measured_ceiling"] = measured
    roof["frac_of_measured_ceiling"] = round(roof["achieved"] / measured, 4) if roof["bound"] != "alu" else None

    result = {
        "metric": "selected tokens/sec (SPA fwd) at 1 GPU", "value": head["value"], "unit": "selected tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": head["workload"], "selected_tokens": head["selected_tokens"], "sum_n2": head["sum_n2"],
                   "seed": args.seed, "launch": head["launch"], "streams": head["streams"], "copies": head["copies"],
                   "timing": f"median over {args.repeats} repeats of the {args.steps}-step region (min: "
                             f"{head['ms_per_step_min'] * 1e3:.2f} us per step)"},
        "ms_per_step_min": head["ms_per_step_min"],
        "ms_per_step_until_last_event": head["ms_per_step_until_last_event"], "single_stream": head["single_stream"],
        "roofline": roof, "ceilings": ceil_, "kernels": head["kernels"], "configs": configs,
    }
    if not args.no_extras:
        result["extras"] = measure_extras(wl, ctx, args, torch, spa, workloads, pipeline)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_oracle_baseline(wl, ctx["bun"], args.cpu_seconds)
        result["cpu_baseline"]["gpu_over_cpu"] = round(head["value"] / result["cpu_baseline"]["value"], 1)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
