"""Turns rocprofv3 CSV output of bench.py runs into the short text summaries under profiles/ and
into profiles/hbm_traffic_table.txt, the table bench.py reads its `roofline.traffic` from.

    python -m paper_2410_23608_amd.profiling kernels <dir> --workload det --chain forward_gathered --command "..."
    python -m paper_2410_23608_amd.profiling traffic <fetch dir> <write dir> --workload det --chain forward_gathered --command "..."
    python -m paper_2410_23608_amd.profiling pipes <dir> --workload det --chain forward_gathered --command "..." [--flops F]

<dir> is the -d directory of a `rocprofv3 ... --output-format csv -d <dir> -o p -- python3 bench.py --only ...`
run (kernel-trace for `kernels`, one --pmc counter set for the others).  A chain names the calls of one
step; every libspa kernel of the run is attributed to the call that launches it by its name, and for
the multi-stage hierarchy to its stage by its grid size (finest stage = largest grid).
"""
from __future__ import annotations

import argparse
import csv
import glob
import os
import re
import statistics
from collections import defaultdict

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
TABLE = os.path.join(PROFILES, "hbm_traffic_table.txt")
PRE = "cd /tmp && export TMPDIR=/tmp && "

# call of the chain <- substring of the kernel name (first match wins); a call may launch two kernels
CHAINS = {
    "forward_fused": [("gate_select_kernel", "gate_select_index"), ("attn_fwd", "gathered_attention_unpack")],
    "forward_selected": [("gate_select_kernel", "gate_select"), ("attn_fwd", "selected_attention_unpack")],
    "forward_gathered": [("gate_select_kernel", "gate_select"), ("pack_kernel", "pack_indices"),
                         ("attn_fwd", "gathered_attention_unpack")],
    "forward_packed": [("gate_select_kernel", "gate_select"), ("pack_kernel", "pack"),
                       ("attn_fwd", "packed_attention_unpack")],
    "train": [("gate_select_kernel", "gate_select"), ("pack_kernel", "pack_qk_rg"), ("attn_fwd", "packed_attention_unpack"),
              ("attn_bwd", "packed_attention_bwd_tokens"), ("gate_bwd", "gate_bwd")],
}
CHAINS["hierarchy"] = CHAINS["train"]
# a whole bench.py run (every configuration and the extras): calls named by kind only
CHAINS["all"] = [("gate_select_kernel", "gate"), ("count_selected", "gate"), ("pack_kernel", "pack"), ("unpack_kernel", "unpack"),
                 ("gather_rows", "unpack / pack backward"), ("attn_fwd", "attention forward"), ("attn_bwd", "attention backward"),
                 ("gate_bwd", "gate backward"), ("linear_bwd", "projection backward"), ("linear", "projection"),
                 ("container_segments", "container segments"), ("maxpool", "max-pool"), ("ceiling", "yardstick")]


def template_args(mangled: str) -> str:
    """'DF16bLi16ELb0E' -> 'bf16, 16, false' (the few forms libspa's kernel templates use)."""
    out, i = [], 0
    while i < len(mangled):
        if mangled.startswith("DF16b", i):
            out.append("bf16")
            i += 5
        elif mangled[i] == "f":
            out.append("float")
            i += 1
        elif mangled[i] == "L" and (m := re.match(r"L([ib])(n?\d+)E", mangled[i:])):
            v = m.group(2).replace("n", "-")
            out.append(v if m.group(1) == "i" else ("true" if v != "0" else "false"))
            i += m.end()
        else:
            return mangled
    return ", ".join(out)


def short(name: str) -> str:
    m = re.match(r"_ZN3spa\d+([a-z_0-9]+?_kernel)I(.*?)E+v", name)      # names the profiler left mangled
    if m:
        args = m.group(2)                      # (the pattern's E+ may have eaten the last literal's closing E)
        return m.group(1) + "<" + template_args(args if re.search(r"L[ib]n?\d+$", args) is None else args + "E") + ">"
    name = re.sub(r"\(.*", "", name).replace("void ", "").replace("spa::", "")
    return name.strip()


def is_spa(name: str) -> bool:
    return "spa::" in name or "_ZN3spa" in name


def read_csv(d: str, suffix: str):
    paths = sorted(glob.glob(os.path.join(d, "**", f"*{suffix}"), recursive=True))
    if not paths:
        raise SystemExit(f"no *{suffix} under {d}")
    rows = []
    for p in paths:
        rows += list(csv.DictReader(open(p)))
    return rows


def grid_of(r) -> int:
    if "Grid_Size" in r and r["Grid_Size"]:
        return int(r["Grid_Size"])
    g = 1
    for k in ("Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"):
        g *= int(r.get(k) or 1)
    return g


def call_of(name: str, chain: str):
    if chain == "hierarchy":       # the run also holds the forward-only chain, whose stages use other attention forms
        if "attn_fwd_bf16_wave_mask" in name:
            return "selected_attention_unpack"
        if re.search(r"attn_fwd_bf16_\w+_kernel(<[^>]*true>|I\w*Lb1EEE)", name):
            return "gathered_attention_unpack"
    for sub, call in CHAINS[chain]:
        if sub in name:
            return call
    return None


def stage_labels(groups, chain):
    """hierarchy: (call, grid) groups -> 's<k>.call' with k by descending grid among the groups whose
    kernel shares a name; other chains: the call itself."""
    if chain != "hierarchy":
        return {g: g[1] for g in groups}
    by_family = defaultdict(list)                 # instances of one kernel template differ by stage (lanes per token)
    for g in groups:
        by_family[(g[1], g[0].split("<")[0])].append(g)
    labels = {}
    for (_, family), gs in by_family.items():
        # a stage = a distinct grid size; the gate backward picks its instance (tokens per workgroup) by the
        # stage's C and two of them launch the same grid, so there the instance tells the stages apart
        key = lambda g: (-g[2], g[0] if family == "gate_bwd_kernel" else "")
        ranks = sorted({key(g) for g in gs})
        # kernels of the long-segment forms serve the two finest stages, the short forms the two coarsest
        first = 3 if (("wave" in family or "fused" in family) and len(ranks) <= 2) else 1     # (wave: lpt64 and mask kernels)
        for g in gs:
            labels[g] = f"s{first + ranks.index(key(g))}.{g[1]}"
    return labels


def cmd_kernels(a):
    rows = [r for r in read_csv(a.dir, "kernel_trace.csv") if is_spa(r["Kernel_Name"])]
    groups = defaultdict(list)
    for r in rows:
        groups[(short(r["Kernel_Name"]), call_of(r["Kernel_Name"], a.chain) or "-", grid_of(r))].append(
            (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    labels = stage_labels(list(groups), a.chain)
    out = [f"# rocprofv3 kernel trace: {a.title or a.chain + ', ' + a.workload}, one stream (every kernel runs alone)", "",
           "Command (MI355X box):", "", f"    {PRE}{a.command}", "",
           "libspa kernels of that run, by kernel and grid size (the run holds the warm-up, the timed steps, the "
           "event-instrumented steps and the back-to-back launches of bench.py):" if a.chain != "all" else
           "libspa kernels of that run, by kernel and grid size.  The run holds every configuration and the extras; a "
           "kernel's launches are partly overlapped with the launches of other batches in flight (the timed regions of "
           "the forward and training steps) and partly alone (the per-kernel timing passes), so min and median "
           "describe the launch alone and avg / max the launches under overlap:", "",
           "| call | kernel | grid (threads) | launches | avg us | median us | min us | max us |", "|---|---|---|---|---|---|---|---|"]
    if a.chain == "all":
        out[0] = f"# rocprofv3 kernel trace: {a.title or 'a whole bench.py run'} (the 60 kernel / grid pairs with the most GPU time)"
    for g in sorted(groups, key=lambda g: -sum(groups[g])):
        d = groups[g]
        out.append(f"| {labels[g]} | {g[0]} | {g[2]} | {len(d)} | {statistics.mean(d):.2f} | {statistics.median(d):.2f} | "
                   f"{min(d):.2f} | {max(d):.2f} |")
    if a.note:
        out += ["", a.note]
    write(f"kernels_{a.workload}.md", out[:10 + 60] if a.chain == "all" else out)


def counters(d: str):
    """(kernel name, grid) -> counter -> list of per-dispatch values; plus the calibration copies."""
    vals = defaultdict(lambda: defaultdict(list))
    for r in read_csv(d, "counter_collection.csv"):
        vals[(r["Kernel_Name"], grid_of(r))][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return vals


def calibration(vals, counter):
    known = 256 * 1024.0        # KiB moved each way by the plain 256 MiB device copy of --calibration-copy
    big = sorted(v for (k, _), c in vals.items() if "copyBuffer" in k for v in c.get(counter, []) if v > known / 8)[-3:]
    if not big:
        raise SystemExit(f"no calibration copy with {counter} in the run (bench.py --calibration-copy)")
    return known / (sum(big) / len(big)), sum(big) / len(big)


def cmd_traffic(a):
    f, w = counters(a.fetch_dir), counters(a.write_dir)
    sf, rf = calibration(f, "FETCH_SIZE")
    sw, rw = calibration(w, "WRITE_SIZE")
    groups = {}
    for (k, grid), c in f.items():
        if not is_spa(k) or "FETCH_SIZE" not in c:
            continue
        wv = w.get((k, grid), {}).get("WRITE_SIZE", [0.0])
        fa = statistics.mean(c["FETCH_SIZE"]) * sf * 1024
        wa = statistics.mean(wv) * sw * 1024
        groups[(short(k), call_of(k, a.chain) or "-", grid)] = (len(c["FETCH_SIZE"]), fa, wa)
    labels = stage_labels(list(groups), a.chain)
    out = [f"# rocprofv3 HBM traffic counters: {a.title or a.chain + ', ' + a.workload}", "",
           "Commands (MI355X box), one counter per run:", "",
           f"    {PRE}{a.command.replace('COUNTER', 'FETCH_SIZE')}", f"    {PRE}{a.command.replace('COUNTER', 'WRITE_SIZE')}", "",
           f"Plain 256 MiB device copy in the same runs: FETCH_SIZE reads {rf:.0f}, WRITE_SIZE reads {rw:.0f} for 262144 KiB "
           f"each way -> scale factors {sf:.3f} and {sw:.3f}.", "",
           "| call | kernel | grid (threads) | launches | fetch MB | write MB | total MB per launch |", "|---|---|---|---|---|---|---|"]
    per_call = defaultdict(float)
    for g in sorted(groups, key=lambda g: -(groups[g][1] + groups[g][2])):
        n, fa, wa = groups[g]
        out.append(f"| {labels[g]} | {g[0]} | {g[2]} | {n} | {fa / 1e6:.2f} | {wa / 1e6:.2f} | {(fa + wa) / 1e6:.2f} |")
        if g[1] != "-":
            per_call[labels[g]] += fa + wa
    write(f"hbm_traffic_{a.workload}.md", out)
    # the table bench.py reads: the rows of this workload are replaced
    keep = []
    if os.path.exists(TABLE):
        keep = [ln.rstrip("\n") for ln in open(TABLE) if ln.startswith("#") or (ln.split() and ln.split()[0] != a.workload)]
    if not keep:
        keep = ["# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, copy-calibrated), seed 0: workload call bytes",
                "# written by `python -m paper_2410_23608_amd.profiling traffic`; sources: profiles/hbm_traffic_<workload>.md"]
    keep += [f"{a.workload} {call} {v:.0f}" for call, v in sorted(per_call.items())]
    with open(TABLE, "w") as fo:
        fo.write("\n".join(keep) + "\n")
    print(f"updated {TABLE}")


def cmd_pipes(a):
    vals = counters(a.dir)
    out = [f"# rocprofv3 counters: busy cycles of the matrix and vector pipes, {a.title or a.chain + ', ' + a.workload}", "",
           "Command (MI355X box), one run:", "", f"    {PRE}{a.command}", "",
           "Averages per launch.  Counters are sums over the chip (8 XCDs, 256 compute units, 1024 SIMDs).  cycles = "
           "`GRBM_GUI_ACTIVE / 8` = cycles the", "launch was on the GPU; matrix pipe busy = `SQ_VALU_MFMA_BUSY_CYCLES / "
           "(cycles x 1024)`; vector ALU busy = `4 x SQ_ACTIVE_INST_VALU / (cycles x 1024)`", "(the counter ticks once per "
           "four cycles of an issued vector instruction); waiting = `SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES`; executed MFMA flop "
           "= `512 x SQ_INSTS_VALU_MFMA_MOPS_BF16`.", "",
           "| call | kernel | grid | launches | cycles | MFMA busy | VALU busy | waves waiting | VALU instr per MFMA | "
           "executed MFMA GFLOP |", "|---|---|---|---|---|---|---|---|---|---|"]
    groups = {}
    for (k, grid), c in vals.items():
        if is_spa(k) and "GRBM_GUI_ACTIVE" in c:
            groups[(short(k), call_of(k, a.chain) or "-", grid)] = c
    labels = stage_labels(list(groups), a.chain)
    m = lambda c, n: statistics.mean(c[n]) if c.get(n) else float("nan")
    for g in sorted(groups, key=lambda g: -m(groups[g], "GRBM_GUI_ACTIVE")):
        c = groups[g]
        cyc = m(c, "GRBM_GUI_ACTIVE") / 8
        mf = m(c, "SQ_INSTS_MFMA")
        out.append(f"| {labels[g]} | {g[0]} | {g[2]} | {len(c['GRBM_GUI_ACTIVE'])} | {cyc:.0f} | "
                   f"{100 * m(c, 'SQ_VALU_MFMA_BUSY_CYCLES') / (cyc * 1024):.1f} % | "
                   f"{100 * 4 * m(c, 'SQ_ACTIVE_INST_VALU') / (cyc * 1024):.1f} % | "
                   f"{100 * m(c, 'SQ_WAIT_INST_ANY') / m(c, 'SQ_WAVE_CYCLES'):.1f} % | "
                   f"{(m(c, 'SQ_INSTS_VALU') - mf) / mf if mf and mf == mf and mf > 0 else float('nan'):.1f} | "
                   f"{512 * m(c, 'SQ_INSTS_VALU_MFMA_MOPS_BF16') / 1e9:.2f} |")
    if a.note:
        out += ["", a.note]
    write(f"pipe_utilisation_{a.workload}.md", out)


def write(name, lines):
    os.makedirs(PROFILES, exist_ok=True)
    path = os.path.join(PROFILES, name)
    with open(path, "w") as fo:
        fo.write("\n".join(lines) + "\n")
    print(f"wrote {path}")


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    for name in ("kernels", "traffic", "pipes"):
        p = sub.add_parser(name)
        if name == "traffic":
            p.add_argument("fetch_dir")
            p.add_argument("write_dir")
        else:
            p.add_argument("dir")
        p.add_argument("--workload", required=True)
        p.add_argument("--chain", required=True, choices=sorted(CHAINS))
        p.add_argument("--command", required=True, help="the rocprofv3 command that made the data (COUNTER = the counter)")
        p.add_argument("--title", default="")
        p.add_argument("--note", default="")
    a = ap.parse_args()
    {"kernels": cmd_kernels, "traffic": cmd_traffic, "pipes": cmd_pipes}[a.what](a)


if __name__ == "__main__":
    main()
