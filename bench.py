#!/usr/bin/env python3
"""Benchmark of the SPA hot path on one MI355X.

A step is one pass of the whole forward path (gate score + selection, pack, per-image
attention on the packed tokens, scatter back — the last two in one launch) over one seeded
synthetic batch that is already resident in HBM.  The default workload is the ViT-S-shaped classification batch
(64 images x 196 tokens, dim 384, 6 heads, bf16, per-image selected fraction U[0.1, 0.9]).

Prints ONE JSON line: whole-path throughput in selected tokens/s, the roofline of the
dominant kernel (durations measured live with events on the launch stream), the CPU
oracle timed on this machine's host cores, and secondary measurements (per-kernel table,
hipGraph replay, the padded-to-max attention baseline, the forward+backward training
step of the ViT-B-shaped workload).
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak

# HBM bytes per launch (fetch + write) of each stage, seed 0, from two `rocprofv3 --pmc` runs of
# this script (FETCH_SIZE, then WRITE_SIZE; `--calibration-copy --steps 20 --warmup 5`), each
# counter scaled by what it reads for the plain 256 MiB device copy of the same run
# (factors 2.000 and 1.000).  Re-measure after any change to a kernel's access pattern.
MEASURED_TRAFFIC_BYTES = {
    ("vit_s", "gate_select"): 9.76e6, ("vit_s", "pack"): 29.45e6, ("vit_s", "packed_attention_unpack"): 24.86e6,
    ("det", "gate_select"): 17.46e6, ("det", "pack"): 26.64e6, ("det", "packed_attention_unpack"): 44.85e6,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="vit_s", choices=["tiny", "vit_s", "vit_b_train", "det"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--streams", type=int, default=4,
                    help="independent batches in flight, one HIP stream each (1 = one stream, steps back to back)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip graph / padded / training measurements")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def timed(fn, steps, torch):
    """K calls bracketed by synchronize on both sides -> seconds."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def per_stage_us(stage_sets, steps, torch):
    """Average duration of every stage, from event pairs recorded on the launch stream
    around each launch of the timed steps.  stage_sets: one list of (name, launch) per
    independent copy of the inputs and buffers; step i runs on copy i % len(stage_sets), so
    with enough copies every launch finds its inputs out of the last-level cache."""
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
    out = {}
    for i, n in enumerate(names):
        out[n] = 1e3 * float(np.mean([ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(steps)]))
    return out


def empty_pair_us(stages, steps, torch):  # noqa: D401
    """What an event pair reads with NO launch between its two records, measured in the same
    position (inside steps of the whole path): the part of a per-launch reading that is not
    kernel time."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for s in range(steps):
        for i, (_, fn) in enumerate(stages):
            fn()
            if i == 1:
                ev[s][0].record()
                ev[s][1].record()
    torch.cuda.synchronize()
    return 1e3 * float(np.mean([a.elapsed_time(b) for a, b in ev]))


def back_to_back_us(fn, steps, torch):
    """Average duration of one launch when the same kernel is enqueued `steps` times between
    two events (no per-launch event overhead).  fn may be a list of launches of the same kernel
    on independent copies of its data, used round-robin."""
    fns = fn if isinstance(fn, (list, tuple)) else [fn]
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for i in range(steps):
        fns[i % len(fns)]()
    b.record()
    torch.cuda.synchronize()
    return 1e3 * a.elapsed_time(b) / steps


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
            "mfma_bf16_TFLOPs": round(best, 1), "mfma": "v_mfma_f32_32x32x16_bf16 only, 4 chains per wave, best of 1 and 2 waves per SIMD"}


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
    from paper_2410_23608_amd import spa, workloads
    from paper_2410_23608_amd.pipeline import ForwardPass, TrainPass

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    wl = workloads.WORKLOADS[args.workload]
    e = 2 if wl.dtype == "bf16" else 4
    td = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    bun = workloads.generate(wl, args.seed)

    def up(a, dtype=None):
        """Host array -> device tensor in the dtype of the workload it is uploaded FOR (the
        headline workload's unless another one is named)."""
        t_ = td if dtype is None else (torch.bfloat16 if dtype == "bf16" else torch.float32)
        return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(t_).contiguous()

    if args.calibration_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    x, w, qkv = up(bun["x"]), up(bun["w"]), up(bun["qkv"])
    # forward only: y is the result; the packed attention output and lse (inputs of a backward
    # pass) are not written
    fp = ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, wl.bias, keep_packed_out=False)
    stages = fp.stages(x, w, qkv)

    def step():
        for _, fn in stages:
            fn()

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    T = int(fp.total.item())
    n = np.diff(fp.cu_seqlens.cpu().numpy()).astype(np.float64)
    sum_n2 = float((n * n).sum())

    # ---- one stream, steps back to back on ONE copy of the batch (everything stays in the
    # 256 MB last-level cache): the latency of a step
    dt1 = timed(step, args.steps, torch)
    single = {"ms_per_step": 1e3 * dt1 / args.steps, "value": T * args.steps / dt1, "unit": "selected tokens/s",
              "cache": "warm (one copy of the batch, reused every step)"}

    # ---- the timed region: exactly K steps.  The batches of a data-parallel job are independent,
    # so S of them are kept in flight: S HIP streams (default priority), steps dealt round-robin,
    # the launches of a step in order on their stream.  Every step works on its own copy of the
    # inputs and its own buffers, and there are enough copies (> 512 MB in total) that no step
    # finds its inputs or a previous step's buffers in the last-level cache.
    S = max(1, args.streams)
    set_bytes = (x.numel() + qkv.numel() + fp.packed_qkv.numel() + fp.y.numel()) * e
    n_sets = S * max(2, -(-(512 << 20) // (S * set_bytes)))
    turn = [0]

    def build_sets(streams_):
        made = []
        for i in range(n_sets):
            with torch.cuda.stream(streams_[i % S]):
                fp_s = ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, wl.bias, keep_packed_out=False)
                ins = (x.clone(), w.clone(), qkv.clone())
                made.append((fp_s, fp_s.stages(*ins), ins))
        torch.cuda.synchronize()
        return made

    def sstep():   # step i -> copy i % n_sets, which lives on stream i % S
        for _, fn in sets[turn[0] % n_sets][1]:
            fn()
        turn[0] += 1

    # Which HIP streams end up sharing one of the process's hardware queues (4 here) is the
    # runtime's business, and two batches on one queue run one after the other.  So three groups of
    # S streams are tried for a few hundred untimed steps each and the fastest group is kept.
    stream_groups = {}
    if S > 1:
        best = None
        for gi_ in range(3):
            cand = [torch.cuda.Stream() for _ in range(S)]
            sets = build_sets(cand)
            for _ in range(n_sets):
                sstep()
            torch.cuda.synchronize()
            turn[0] = 0
            probe = timed(sstep, 300, torch) / 300
            stream_groups[f"group_{gi_}_us_per_step"] = round(1e6 * probe, 2)
            if best is None or probe < best[0]:
                best = (probe, cand, sets)
            del sets
        _, streams, sets = best
        del best
    else:
        streams = [torch.cuda.current_stream()]
        sets = build_sets(streams)

    for _ in range(max(args.warmup, n_sets)):
        sstep()
    torch.cuda.synchronize()
    turn[0] = 0
    dt = timed(sstep, args.steps, torch)
    if not all(torch.equal(fs.y, fp.y) and int(fs.total.item()) == T for fs, _, _ in sets):
        print("bench.py: a copy's result differs from the single-stream result", file=sys.stderr)
        sys.exit(1)
    ms_per_step = 1e3 * dt / args.steps
    value = T * args.steps / dt

    # ---- per-kernel durations, live, events on the launch stream, the kernel running alone.
    # cold: the copies of the timed region on ONE stream, in rotation; warm: one copy reused.
    cold_sets = [fs.stages(*ins) for fs, _, ins in sets]   # the same launches, prepared on this stream
    st_us = per_stage_us(cold_sets, args.steps, torch)
    b2b_us = {nme: back_to_back_us([cs[i][1] for cs in cold_sets], args.steps, torch)
              for i, (nme, _) in enumerate(stages)}
    warm_us = {nme: min(v_, back_to_back_us(fn, args.steps, torch))
               for (nme, fn), v_ in zip(stages, per_stage_us([stages], args.steps, torch).values())}
    ev_overhead = empty_pair_us(stages, args.steps, torch)
    B, N, C, H = wl.B, wl.N, wl.C, wl.H
    attn_flops = 4.0 * C * sum_n2
    work = {  # algorithmic (flops, bytes) per launch
        "gate_select": (0.0, B * N * (C * e + 5)),
        "pack": (0.0, 2 * T * 3 * C * e + 4 * T + 5 * B * N + 4 * (B + 1)),
        "packed_attention": (attn_flops, T * 3 * C * e + T * C * e + 4 * H * T + 4 * (B + 1)),
        # attention + scatter back in one launch: q|k|v rows in, every row of y out, the index arrays
        "packed_attention_unpack": (attn_flops, T * 3 * C * e + B * N * C * e + 4 * T + 4 * B * N + 4 * (B + 1)
                                    + (T * C * e + 4 * H * T if fp.keep_packed_out else 0)),
        "unpack": (0.0, T * C * e + 4 * B * N + B * N * C * e),
    }
    work = {k_: v_ for k_, v_ in work.items() if k_ in st_us}
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if wl.dtype == "bf16" else 157.3
    ridge = mfma_peak * 1e12 / (HBM_PEAK_GBS * 1e9)     # flop per byte at which the two roofs meet
    kernels = {}
    for nme, (flops, nbytes) in work.items():
        # Two live readings, both with HIP events on the launch stream and both upper bounds of
        # the kernel's duration: an event pair around each launch inside K steps of the whole
        # path (includes the cost of the two markers; an empty pair reads ev_overhead) and K
        # back-to-back launches of the kernel between one pair (includes the dispatch gap).
        # The smaller one is used; rocprofv3's kernel-trace average sits a little below it.
        us = min(st_us[nme], b2b_us[nme])
        intensity = flops / nbytes
        # the roof that bounds the kernel: below the ridge the HBM roof is the lower one
        if intensity < ridge:
            bound, ach, peak, unit = "hbm", nbytes / us / 1e3, HBM_PEAK_GBS, "GB/s"
        else:
            bound, ach, peak, unit = "mfma" if wl.dtype == "bf16" else "alu", flops / us / 1e6, mfma_peak, "TFLOP/s"
        kernels[nme] = {"bound": bound, "cache": "cold", "event_us": round(st_us[nme], 2), "kernel_us": round(us, 2),
                        "back_to_back_us": round(b2b_us[nme], 2), "warm_cache_us": round(warm_us[nme], 2),
                        "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4),
                        "algorithmic_bytes": int(nbytes), "algorithmic_flops": flops,
                        "flop_per_byte": round(intensity, 1), "ridge_flop_per_byte": round(ridge, 1)}
        if flops > 0:
            kernels[nme]["tflops"] = round(flops / us / 1e6, 2)
            kernels[nme]["mfma_frac"] = round(flops / us / 1e6 / mfma_peak, 4)
    dom = max(kernels, key=lambda k_: kernels[k_]["kernel_us"])
    kd = kernels[dom]
    ceil_ = ceilings(spa, torch)
    measured_ceiling = ceil_["copy_GBs"] if kd["bound"] == "hbm" else ceil_["mfma_bf16_TFLOPs"]
    roofline = {"kernel": dom, "bound": kd["bound"], "achieved": kd["achieved"], "peak": kd["peak"],
                "unit": kd["unit"], "frac": kd["frac"],
                "cache": f"cold: {n_sets} copies of the batch and its buffers in rotation ({n_sets * set_bytes >> 20} MB)",
                "warm_cache_frac": round(kd["frac"] * kd["kernel_us"] / kd["warm_cache_us"], 4),
                "measured_ceiling": measured_ceiling,
                "frac_of_measured_ceiling": round(kd["achieved"] / measured_ceiling, 4) if kd["bound"] != "alu" else None,
                "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, dom)) if args.seed == 0 else None,
                "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated)",
                "avg_launch_us": kd["kernel_us"],
                "event_pair_overhead_us": round(ev_overhead, 2)}
    if "tflops" in kd:
        roofline.update({"flop_per_byte": kd["flop_per_byte"], "ridge_flop_per_byte": kd["ridge_flop_per_byte"],
                         "tflops": kd["tflops"], "mfma_frac": kd["mfma_frac"]})

    result = {
        "metric": "selected tokens/sec (SPA fwd) at 1 GPU", "value": value, "unit": "selected tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={B} N={N} C={C} H={H} Dh={wl.Dh} {wl.dtype}, selected fraction "
                               f"U[{wl.frac[0]},{wl.frac[1]}] per image, forward select+pack+attention+unpack",
                   "selected_tokens": T, "sum_n2": sum_n2, "seed": args.seed,
                   "launch": f"eager, {len(stages)} launches per step ({' + '.join(n_ for n_, _ in stages)}); "
                             f"{S} independent batches in flight on {S} HIP stream(s); {n_sets} copies of the "
                             f"inputs and buffers in rotation ({n_sets * set_bytes >> 20} MB, cold last-level cache)",
                   "streams": S, "copies": n_sets, "stream_group_calibration": stream_groups},
        "single_stream": single,
        "roofline": roofline, "ceilings": ceil_, "kernels": kernels,
    }

    if not args.no_extras:
        # the hot path as its four calls (gate_select, pack, packed_attention, unpack), the last two NOT
        # fused: warm back-to-back launch times and the roofline fraction of each kernel on its own
        fp4 = ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, wl.bias, fused_unpack=False)
        st4 = fp4.stages(x, w, qkv)

        def step4():
            for _, fn in st4:
                fn()

        for _ in range(5):
            step4()
        torch.cuda.synchronize()
        dt4 = timed(step4, args.steps, torch)
        us4 = {nme: back_to_back_us(fn, args.steps, torch) for nme, fn in st4}
        all_work = {"gate_select": (0.0, B * N * (C * e + 5)),
                    "pack": (0.0, 2 * T * 3 * C * e + 4 * T + 5 * B * N + 4 * (B + 1)),
                    "packed_attention": (attn_flops, T * 3 * C * e + T * C * e + 4 * H * T + 4 * (B + 1)),
                    "unpack": (0.0, T * C * e + 4 * B * N + B * N * C * e)}
        four = {}
        for nme, us_ in us4.items():
            fl, by = all_work[nme]
            four[nme] = {"us": round(us_, 2), "GB/s": round(by / us_ / 1e3, 1), "hbm_frac": round(by / us_ / 1e3 / HBM_PEAK_GBS, 4)}
            if fl > 0:
                four[nme].update({"tflops": round(fl / us_ / 1e6, 2), "mfma_frac": round(fl / us_ / 1e6 / mfma_peak, 4)})
        result["four_call_form"] = {"ms_per_step": 1e3 * dt4 / args.steps, "value": T * args.steps / dt4,
                                    "cache": "warm (one copy of the batch, one stream)",
                                    "y_equals_fused_form": bool(torch.equal(fp4.y, fp.y)), "kernels": four}

        # the same step replayed as a hipGraph
        try:
            def make_step():
                st = fp.stages(x, w, qkv)
                return lambda: [fn() for _, fn in st]
            gdt = graph_replay_s(make_step, args.steps, torch)
            result["graph_replay"] = {"ms_per_step": 1e3 * gdt / args.steps, "value": T * args.steps / gdt}
        except Exception as ex:  # capture refused: report, do not hide
            result["graph_replay"] = {"error": str(ex)[:200]}
        # padded-to-max masked attention on the same selected tokens
        n_max = int(n.max())
        pad = torch.zeros(B, n_max, 3 * C, dtype=td, device="cuda")
        cu = fp.cu_seqlens.cpu().numpy()
        for b in range(B):
            pad[b, :cu[b + 1] - cu[b]] = fp.packed_qkv[cu[b]:cu[b + 1]]
        lens = torch.from_numpy(np.diff(cu).astype(np.int32)).cuda()
        pout = torch.empty(B, n_max, C, dtype=td, device="cuda")
        flat = pad.view(B * n_max, 3 * C)
        pfn = spa.spa_padded_attention(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], lens, B, n_max, H, wl.Dh, pout,
                                       prepare=True)
        # the cost of padding itself: every image carries n_max keys (timing only: the mask of a
        # dense masked kernel adds a compare/select per score on top of this)
        lens_full = torch.full((B,), n_max, dtype=torch.int32, device="cuda")
        dfn = spa.spa_padded_attention(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], lens_full, B, n_max, H, wl.Dh,
                                       pout, prepare=True)
        pfn()
        dfn()
        pus = back_to_back_us(pfn, args.steps, torch)
        dus = back_to_back_us(dfn, args.steps, torch)
        afn = spa.spa_packed_attention(fp.packed_qkv[:, :C], fp.packed_qkv[:, C:2 * C], fp.packed_qkv[:, 2 * C:],
                                       fp.cu_seqlens, B, N, H, wl.Dh, fp.out, None, prepare=True)
        aus = back_to_back_us(afn, args.steps, torch)
        result["padded_baseline"] = {
            "n_max": n_max, "packed_attention_us": round(aus, 2),
            "padded_dense_us": round(dus, 2), "speedup_over_padded_dense": round(dus / aus, 3),
            "padded_dense": "every image padded to n_max queries AND n_max keys (B n_max^2 scores): what padding to "
                            "the batch maximum costs",
            "work_ratio_B_nmax2_over_sum_n2": round(B * n_max * n_max / sum_n2, 3),
            "padded_skipping_masked_keys_us": round(pus, 2), "speedup_over_padded_skipping": round(pus / aus, 3),
            "padded_skipping_masked_keys": "n_max queries per image, but keys past the image's length are skipped "
                                           "instead of masked (sum n_max n_b scores): a length-aware padded kernel",
            "work_ratio_nmax_sum_n_over_sum_n2": round(n_max * float(n.sum()) / sum_n2, 3)}
        # forward + backward training step, ViT-B-shaped
        twl = workloads.WORKLOADS["vit_b_train"]
        tb = workloads.generate(twl, args.seed)
        tp = TrainPass(twl.B, twl.N, twl.C, twl.H, twl.dtype, twl.tau, twl.bias)
        tx, tw = up(tb["x"], twl.dtype), up(tb["w"], twl.dtype)
        tqk = up(tb["qkv"][:, :, :2 * twl.C], twl.dtype)
        tdy = up(tb["dy"], twl.dtype)
        tlab = torch.from_numpy(tb["labels"]).cuda()
        tstages = tp.stages(tx, tw, tqk, tlab, tdy)

        def tstep():
            for _, fn in tstages:
                fn()

        for _ in range(5):
            tstep()
        torch.cuda.synchronize()
        tT = int(tp.total.item())
        tn = np.diff(tp.cu_seqlens.cpu().numpy()).astype(np.float64)
        tdt = timed(tstep, args.steps, torch)
        tus = {nme: back_to_back_us(fn, args.steps, torch) for nme, fn in tstages}
        bwd_flops = 10.0 * twl.C * float((tn * tn).sum())
        result["fwd_bwd"] = {"workload": "vit_b_train: B=64 N=196 C=768 H=12 bf16, fwd+bwd with selection loss",
                             "value": tT * args.steps / tdt, "unit": "selected tokens/s",
                             "ms_per_step": 1e3 * tdt / args.steps, "selected_tokens": tT,
                             "stage_us": {k_: round(v_, 2) for k_, v_ in tus.items()},
                             "attention_bwd_tflops": round(bwd_flops / tus["packed_attention_bwd_tokens"] / 1e6, 2)}
        # the same step with the gather of dy and the scatters of dq, dk, dv as separate launches (9 launches)
        tp9 = TrainPass(twl.B, twl.N, twl.C, twl.H, twl.dtype, twl.tau, twl.bias, fused_bwd=False, pack_pair=False)
        t9 = tp9.stages(tx, tw, tqk, tlab, tdy)

        def t9step():
            for _, fn in t9:
                fn()

        for _ in range(5):
            t9step()
        torch.cuda.synchronize()
        t9dt = timed(t9step, args.steps, torch)
        t9us = {nme: back_to_back_us(fn, args.steps, torch) for nme, fn in t9}
        result["fwd_bwd"]["separate_gather_scatter"] = {
            "ms_per_step": 1e3 * t9dt / args.steps, "launches": len(t9),
            "gradients_equal": bool(torch.equal(tp9.dx, tp.dx) and torch.equal(tp9.dqk, tp.dqk) and torch.equal(tp9.dw, tp.dw)),
            "stage_us": {k_: round(t9us[k_], 2) for k_ in ("unpack_bwd", "packed_attention_bwd", "pack_bwd_v", "pack_bwd_qk")}}
        if S > 1:   # the training step with S batches in flight, like the forward headline
            tsets = []
            for s_ in streams:
                with torch.cuda.stream(s_):
                    tp_s = TrainPass(twl.B, twl.N, twl.C, twl.H, twl.dtype, twl.tau, twl.bias)
                    tsets.append((tp_s, tp_s.stages(tx.clone(), tw.clone(), tqk.clone(), tlab.clone(), tdy.clone())))
            torch.cuda.synchronize()
            turn[0] = 0

            def tsstep():
                for _, fn in tsets[turn[0] % S][1]:
                    fn()
                turn[0] += 1

            for _ in range(2 * S):
                tsstep()
            torch.cuda.synchronize()
            turn[0] = 0
            tsdt = timed(tsstep, args.steps, torch)
            same = all(torch.equal(ts.dx, tp.dx) and torch.equal(ts.dw, tp.dw) for ts, _ in tsets)
            result["fwd_bwd"]["batches_in_flight"] = {"streams": S, "value": tT * args.steps / tsdt,
                                                      "ms_per_step": 1e3 * tsdt / args.steps,
                                                      "gradients_equal_single_stream": bool(same)}
        # the same step with stochastic Gumbel-Softmax selection and the straight-through backward
        gn = torch.from_numpy(np.random.default_rng(args.seed + 5).logistic(size=(twl.B, twl.N)).astype(np.float32)).cuda()
        gstages = tp.stages(tx, tw, tqk, tlab, tdy, noise=gn, temperature=1.0)

        def gstep():
            for _, fn in gstages:
                fn()

        for _ in range(5):
            gstep()
        torch.cuda.synchronize()
        gT = int(tp.total.item())
        gdt2 = timed(gstep, args.steps, torch)
        result["fwd_bwd_gumbel"] = {"selected_tokens": gT, "value": gT * args.steps / gdt2, "unit": "selected tokens/s",
                                    "ms_per_step": 1e3 * gdt2 / args.steps,
                                    "stage_us": {nme: round(back_to_back_us(fn, args.steps, torch), 2)
                                                 for nme, fn in (gstages[0], gstages[-1])}}

        # the block with its projections: only selected tokens are projected
        from paper_2410_23608_amd.pipeline import BlockPass
        g = torch.Generator(device="cpu").manual_seed(args.seed + 17)
        mkw = lambda r, c: (torch.randn(r, c, generator=g) / c ** 0.5).cuda().to(td)
        W_qkv, b_qkv, W_o, b_o = mkw(3 * C, C), mkw(1, 3 * C).view(-1), mkw(C, C), mkw(1, C).view(-1)
        bp = BlockPass(B, N, C, H, wl.dtype, wl.tau, wl.bias)
        bstages = bp.stages(x, w, W_qkv, b_qkv, W_o, b_o)

        def bstep():
            for _, fn in bstages:
                fn()

        for _ in range(5):
            bstep()
        torch.cuda.synchronize()
        bdt = timed(bstep, args.steps, torch)
        bus = {nme: back_to_back_us(fn, args.steps, torch) for nme, fn in bstages}
        result["block_with_projections"] = {
            "launches": [n_ for n_, _ in bstages], "value": T * args.steps / bdt, "unit": "selected tokens/s",
            "ms_per_step": 1e3 * bdt / args.steps, "stage_us": {k_: round(v_, 2) for k_, v_ in bus.items()},
            "qkv_projection_tflops": round(2.0 * T * C * 3 * C / bus["qkv_projection"] / 1e6, 1),
            "out_projection_tflops": round(2.0 * T * C * C / bus["out_projection"] / 1e6, 1),
            "dense_projection_flops_saved": round(1.0 - T / (B * N), 3)}
        # the block forward + backward with its projections (input-side and weight-side GEMMs of both
        # projections, attention backward, gate backward with the selection loss)
        from paper_2410_23608_amd.pipeline import BlockTrainPass
        dy_blk = torch.randn(B, N, C, generator=g).cuda().to(td)
        lab_blk = torch.from_numpy(bun["labels"]).cuda()
        blk_train = {}
        for key, ov in (("two_streams", True), ("one_stream", False)):
            btp = BlockTrainPass(B, N, C, H, wl.dtype, wl.tau, wl.bias, overlap_weight_grads=ov)
            tst = btp.stages(x, w, W_qkv, b_qkv, W_o, b_o, lab_blk, dy_blk)

            def tstep():
                for _, fn in tst:
                    fn()

            for _ in range(5):
                tstep()
            torch.cuda.synchronize()
            tdt = timed(tstep, args.steps, torch)
            blk_train[key] = {"ms_per_step": 1e3 * tdt / args.steps, "value": T * args.steps / tdt,
                              "unit": "selected tokens/s"}
            if not ov:
                tus = {nme: back_to_back_us(fn, args.steps, torch) for nme, fn in tst}
                gemm = {"qkv_projection_bwd_input": 3, "qkv_projection_bwd_weight": 3, "out_projection_bwd_input": 1,
                        "out_projection_bwd_weight": 1}
                blk_train[key]["launches"] = [n_ for n_, _ in tst]
                blk_train[key]["stage_us"] = {k_: round(v_, 2) for k_, v_ in tus.items()}
                blk_train[key]["gemm_tflops"] = {k_: round(2.0 * T * C * m_ * C / tus[k_] / 1e6, 1) for k_, m_ in gemm.items()}
        if S > 1:   # independent batches in flight, one stream each, like the forward headline
            bsets = []
            for s_ in streams:
                with torch.cuda.stream(s_):
                    b_s = BlockTrainPass(B, N, C, H, wl.dtype, wl.tau, wl.bias, overlap_weight_grads=False)
                    bsets.append((b_s, b_s.stages(x.clone(), w.clone(), W_qkv.clone(), b_qkv.clone(), W_o.clone(),
                                                  b_o.clone(), lab_blk.clone(), dy_blk.clone())))
            torch.cuda.synchronize()
            turn[0] = 0

            def bsstep():
                for _, fn in bsets[turn[0] % S][1]:
                    fn()
                turn[0] += 1

            for _ in range(2 * S):
                bsstep()
            torch.cuda.synchronize()
            turn[0] = 0
            bsdt = timed(bsstep, args.steps, torch)
            blk_train["batches_in_flight"] = {
                "streams": S, "ms_per_step": 1e3 * bsdt / args.steps, "value": T * args.steps / bsdt,
                "gradients_equal_single_stream": bool(all(torch.equal(b_.dW_qkv, btp.dW_qkv) and torch.equal(b_.dx, btp.dx)
                                                          for b_, _ in bsets))}
        result["block_with_projections"]["fwd_bwd"] = blk_train

        # the paper's container mask: containers of L = 7^2 tokens, map shifted by (3, 3)
        side = int(round(N ** 0.5))
        if side * side == N:
            from paper_2410_23608_amd.pipeline import ContainerForwardPass
            cp = ContainerForwardPass(B, side, side, C, H, wl.dtype, 49, (3, 3), wl.tau, wl.bias)
            cstages = cp.stages(x, w, qkv)

            def cstep():
                for _, fn in cstages:
                    fn()

            for _ in range(5):
                cstep()
            torch.cuda.synchronize()
            cdt = timed(cstep, args.steps, torch)
            cus = {nme: back_to_back_us(fn, args.steps, torch) for nme, fn in cstages}
            seg = cp.seg_cu_seqlens.cpu().numpy().astype(np.float64)
            seg_n2 = float((np.diff(seg) ** 2).sum())
            result["container_local"] = {
                "container_len": 49, "shift": [3, 3], "segments": int(cp.n_segments.item()),
                "segment_capacity": cp.seg_cap, "sum_n2": seg_n2, "value": T * args.steps / cdt,
                "unit": "selected tokens/s", "ms_per_step": 1e3 * cdt / args.steps,
                "stage_us": {k_: round(v_, 2) for k_, v_ in cus.items()},
                "attention_tflops": round(4.0 * C * seg_n2 / cus["segment_attention_unpack"] / 1e6, 2)}
            cp2 = ContainerForwardPass(B, side, side, C, H, wl.dtype, 49, (3, 3), wl.tau, wl.bias, fused_unpack=False)
            c2 = cp2.stages(x, w, qkv)

            def c2step():
                for _, fn in c2:
                    fn()

            for _ in range(5):
                c2step()
            torch.cuda.synchronize()
            c2dt = timed(c2step, args.steps, torch)
            result["container_local"]["separate_unpack"] = {
                "outputs_equal": bool(torch.equal(cp2.y, cp.y)), "ms_per_step": 1e3 * c2dt / args.steps,
                "launches": [n_ for n_, _ in c2]}

        # four-stage hierarchy (batch 16, 56^2 .. 7^2 tokens, C 96 .. 768): 12 launches, eager and as one hipGraph
        from paper_2410_23608_amd.pipeline import HierarchyPass
        hb = workloads.generate_hierarchy(args.seed)
        hcfg = [(b_["workload"].B, *b_["workload"].grid, b_["workload"].C, b_["workload"].H, b_["workload"].dtype,
                 b_["workload"].tau, b_["bias"]) for b_ in hb]
        hp = HierarchyPass(hcfg)
        hdt_ = [b_["workload"].dtype for b_ in hb]
        hx = [up(b_["x"], d_) for b_, d_ in zip(hb, hdt_)]
        hw = [up(b_["w"], d_) for b_, d_ in zip(hb, hdt_)]
        hq = [up(b_["qkv"], d_) for b_, d_ in zip(hb, hdt_)]
        hstages = hp.stages(hx, hw, hq)

        def hstep():
            for _, fn in hstages:
                fn()

        for _ in range(5):
            hstep()
        torch.cuda.synchronize()
        hT = [int(p_.total.item()) for p_ in hp.passes]
        hdt = timed(hstep, args.steps, torch)
        hres = {"stages": [b_["workload"].name for b_ in hb], "launches": len(hstages), "selected_tokens": hT,
                "tokens": [c_[0] * c_[1] * c_[2] for c_ in hcfg], "ms_per_chain": 1e3 * hdt / args.steps,
                "value": sum(hT) * args.steps / hdt, "unit": "selected tokens/s",
                "stage_us": {nme: round(back_to_back_us(fn, args.steps, torch), 2) for nme, fn in hstages}}
        try:
            def make_hstep():
                st_ = hp.stages(hx, hw, hq)
                return lambda: [fn() for _, fn in st_]
            ghdt = graph_replay_s(make_hstep, args.steps, torch)
            hres["graph_replay_ms_per_chain"] = 1e3 * ghdt / args.steps
        except Exception as ex:
            hres["graph_replay_error"] = str(ex)[:200]
        # the same hierarchy forward + backward (20 calls)
        from paper_2410_23608_amd.pipeline import HierarchyTrainPass
        htp = HierarchyTrainPass(hcfg)
        hqk = [up(b_["qkv"][:, :, :2 * b_["workload"].C], b_["workload"].dtype) for b_ in hb]
        hlab = [torch.from_numpy(b_["labels"]).cuda() for b_ in hb]
        hdy = [up(b_["dy"], b_["workload"].dtype) for b_ in hb]
        htstages = htp.stages(hx, hw, hqk, hlab, hdy)

        def htstep():
            for _, fn in htstages:
                fn()

        for _ in range(5):
            htstep()
        torch.cuda.synchronize()
        htT = [int(p_.total.item()) for p_ in htp.passes]
        htdt = timed(htstep, args.steps, torch)
        hres["fwd_bwd"] = {"launches": len(htstages), "selected_tokens": htT, "ms_per_chain": 1e3 * htdt / args.steps,
                           "value": sum(htT) * args.steps / htdt, "unit": "selected tokens/s"}
        htpc = HierarchyTrainPass(hcfg, concurrent=True)
        htcstages = htpc.stages(hx, hw, hqk, hlab, hdy)

        def htcstep():
            for _, fn in htcstages:
                fn()

        for _ in range(5):
            htcstep()
        torch.cuda.synchronize()
        htcdt = timed(htcstep, args.steps, torch)
        hres["fwd_bwd"]["stream_per_stage"] = {
            "ms_per_chain": 1e3 * htcdt / args.steps, "value": sum(htT) * args.steps / htcdt,
            "gradients_equal_one_stream": bool(all(torch.equal(a_.dx, b_.dx) and torch.equal(a_.dw, b_.dw)
                                                   for a_, b_ in zip(htpc.passes, htp.passes)))}
        result["hierarchy"] = hres

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_oracle_baseline(wl, bun, args.cpu_seconds)
        result["cpu_baseline"]["gpu_over_cpu"] = round(value / result["cpu_baseline"]["value"], 1)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
