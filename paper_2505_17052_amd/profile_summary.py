"""Turns rocprofv3 CSV output of a bench.py run into the short text summaries kept under profiles/.

    python3 -m paper_2505_17052_amd.profile_summary kernel-stats --dir D --workload W --cmd "..." [--bench-json J] --out F
    python3 -m paper_2505_17052_amd.profile_summary counters     --dir D --workload W --cmd "..." --out F
    python3 -m paper_2505_17052_amd.profile_summary traffic      --fetch-dir D1 --write-dir D2 --workload W --cmd "..." --out F

kernel-stats: per-kernel calls / total / average / min / max from a --kernel-trace run (the *_kernel_trace.csv).
counters:     per-kernel averages of every counter of a --pmc run (the *_counter_collection.csv), plus the matrix-pipe
              utilisation when SQ_VALU_MFMA_BUSY_CYCLES and GRBM_GUI_ACTIVE are among them.
traffic:      HBM bytes per launch of the gate/up GEMM from a FETCH_SIZE run and a WRITE_SIZE run (bench.py
              --calibration-copy adds plain 1 GiB device copies whose known size scales the counters); ends with the
              machine-readable line 'sev-traffic ...' that bench.py reads, stamped with the hash of the kernel sources.
Only formats data that the profiler wrote; it measures nothing itself.
"""
import argparse
import collections
import csv
import glob
import json
import os
import sys

EPI_NAMES = {"0": "QKV projection (rotary + cache append)", "1": "gate/up projection + SwiGLU", "2": "LM head + arg-max",
             "3": "O / down projection (residual + next norm operand)"}


def _find(d, suffix):
    hits = sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    if not hits:
        sys.exit(f"no *{suffix} under {d}")
    return hits[0]


def short_name(name):
    """Kernel name without its argument list; template arguments kept."""
    n = name.replace("void ", "")
    cut = n.find("(")
    return n[:cut] if cut > 0 else n


def is_gate_up(name):
    s = short_name(name)
    if not s.startswith("gemm_bf16_kernel<"):
        return False
    args = [a.strip() for a in s[s.index("<") + 1:s.rindex(">")].split(",")]
    return len(args) >= 3 and args[2] == "1"


def header(title, workload, cmd):
    line = f"{title}, workload {workload}"
    return f"{line}\n{'=' * len(line)}\n\nCommand (from the repository root $REPO on one MI355X; library built beforehand with __graft_entry__.build()):\n\n  {cmd}\n\n"


def kernel_stats(a):
    rows = list(csv.DictReader(open(_find(a.dir, "kernel_trace.csv"))))
    agg = collections.defaultdict(list)
    for r in rows:
        agg[short_name(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in agg.values())
    out = [header("Kernel-time summary of a whole bench.py run", a.workload, a.cmd)]
    if a.bench_json:
        bj = json.loads(open(a.bench_json).read().strip().splitlines()[-1])
        out.append(f"bench.py's JSON line from the same run: ms_per_step {bj['ms_per_step']:.3f}, {bj['value']:.0f} {bj['unit']}, rows per step "
                   f"{bj['config']['rows_per_step']}, steps {bj['steps']} + warm-up {bj['warmup']} (+ the same number of event-timed steps and 5 per-class "
                   f"steps; the run also holds the cache fill and, for chain workloads, the single-token rounds that make the drafts).\n"
                   f"Event-timed gate/up launch: {bj['roofline']['avg_launch_ms'] * 1e3:.2f} us (HIP events; about {bj['roofline']['empty_event_pair_ms'] * 1e3:.1f} us "
                   f"above the kernel's own duration below).\n\n")
    out.append(f"{'kernel':72s} {'calls':>7s} {'total ms':>9s} {'avg us':>8s} {'med us':>8s} {'min us':>8s} {'max us':>8s} {'%':>6s}\n")
    for name, v in sorted(agg.items(), key=lambda kv: -sum(kv[1]))[:a.top]:
        s = sorted(v)
        out.append(f"{name[:72]:72s} {len(v):7d} {sum(v) / 1e3:9.2f} {sum(v) / len(v):8.2f} {s[len(s) // 2]:8.2f} {s[0]:8.2f} {s[-1]:8.2f} {100 * sum(v) / total:6.2f}\n")
    out.append("\ngemm_bf16_kernel<MT, NT, EPI, PF>: row tiles per block, column tiles per wave, epilogue, prefetch depth.  EPI: " +
               "; ".join(f"{k} = {v}" for k, v in EPI_NAMES.items()) +
               ".\ngemm_fixup_kernel<EPI> sums the split-K slices and runs the same epilogue; attn_merge_kernel combines the KV chunks.\n")
    open(a.out, "w").write("".join(out))


def _counter_rows(d):
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_find(d, "counter_collection.csv"))):
        per[short_name(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return per


def counters(a):
    per = _counter_rows(a.dir)
    names = sorted({c for v in per.values() for c in v})
    out = [header("Hardware counters per dispatch (averages)", a.workload, a.cmd)]
    out.append(f"{'kernel':64s} {'n':>6s} " + " ".join(f"{c[:24]:>24s}" for c in names) + "\n")
    rows = sorted(per.items(), key=lambda kv: -sum(sum(x) for x in kv[1].values()))[:a.top]
    for k, v in rows:
        n = max(len(x) for x in v.values())
        out.append(f"{k[:64]:64s} {n:6d} " + " ".join(f"{(sum(v[c]) / len(v[c]) if v.get(c) else float('nan')):24.1f}" for c in names) + "\n")
    if "SQ_VALU_MFMA_BUSY_CYCLES" in names and "GRBM_GUI_ACTIVE" in names:
        out.append("\nMatrix-pipe utilisation.  SQ_VALU_MFMA_BUSY_CYCLES is summed over the chip's 1024 SIMDs (32 cycles per 32x32x16 MFMA issued);\n"
                   "GRBM_GUI_ACTIVE is summed over the 8 XCDs, so a dispatch lasts GRBM_GUI_ACTIVE / 8 cycles.  busy = MFMA busy / (duration x 1024).\n"
                   "Every activation is multiplied as two bf16 planes: the useful bf16 FLOP rate is half of the pipe utilisation.\n\n")
        out.append(f"{'kernel':64s} {'MFMA busy cyc':>14s} {'duration cyc':>13s} {'pipe busy':>10s} {'useful':>8s}\n")
        for k, v in rows:
            if not v.get("SQ_VALU_MFMA_BUSY_CYCLES") or not v.get("GRBM_GUI_ACTIVE"):
                continue
            busy = sum(v["SQ_VALU_MFMA_BUSY_CYCLES"]) / len(v["SQ_VALU_MFMA_BUSY_CYCLES"])
            dur = sum(v["GRBM_GUI_ACTIVE"]) / len(v["GRBM_GUI_ACTIVE"]) / 8.0
            if busy > 0 and dur > 0:
                out.append(f"{k[:64]:64s} {busy:14.0f} {dur:13.0f} {100 * busy / (dur * 1024):9.1f}% {50 * busy / (dur * 1024):7.1f}%\n")
    if "TCP_TCC_READ_REQ_sum" in names:
        out.append("\nA read request from a compute unit's L1 to the L2 carries 128 bytes: TCP_TCC_READ_REQ_sum x 128 B is what a launch moves from the L2s\n"
                   "into the compute units.\n\n")
        out.append(f"{'kernel':64s} {'MB into the compute units':>26s} {'L2 hit rate':>12s}\n")
        for k, v in rows:
            if v.get("TCP_TCC_READ_REQ_sum"):
                req = sum(v["TCP_TCC_READ_REQ_sum"]) / len(v["TCP_TCC_READ_REQ_sum"])
                hit = sum(v.get("TCC_HIT_sum", [0])) / max(len(v.get("TCC_HIT_sum", [0])), 1)
                miss = sum(v.get("TCC_MISS_sum", [0])) / max(len(v.get("TCC_MISS_sum", [0])), 1)
                rate = f"{100 * hit / (hit + miss):11.1f}%" if hit + miss > 0 else f"{'-':>12s}"
                out.append(f"{k[:64]:64s} {req * 128 / 1e6:26.1f} {rate}\n")
    open(a.out, "w").write("".join(out))


def traffic(a):
    from bench import kernel_source_hash
    f, w = _counter_rows(a.fetch_dir), _counter_rows(a.write_dir)

    def pick(per, pred, counter, fn):
        vals = [x for k, v in per.items() if pred(k) for x in v.get(counter, [])]
        return (fn(vals), len(vals), min(vals), max(vals)) if vals else (float("nan"), 0, 0, 0)
    mean = lambda v: sum(v) / len(v)
    copy_f = pick(f, lambda k: "copyBuffer" in k, "FETCH_SIZE", max)[0]
    copy_w = pick(w, lambda k: "copyBuffer" in k, "WRITE_SIZE", max)[0]
    ff, fw = 1048576.0 / copy_f, 1048576.0 / copy_w
    # the gate/up kernel of the timed steps: the instance with the most dispatches
    gu_names = sorted((k for k in f if is_gate_up(k)), key=lambda k: -len(f[k].get("FETCH_SIZE", [])))
    gu = gu_names[0]
    guf = pick(f, lambda k: k == gu, "FETCH_SIZE", mean)
    guw = pick(w, lambda k: k == gu, "WRITE_SIZE", mean)
    att_f = pick(f, lambda k: k.startswith("attn_bf16_kernel"), "FETCH_SIZE", mean)
    att_w = pick(w, lambda k: k.startswith("attn_bf16_kernel"), "WRITE_SIZE", mean)
    fetched, written = guf[0] * ff * 1024, guw[0] * fw * 1024
    out = [header(f"HBM traffic of the gate/up GEMM ({gu})", a.workload, a.cmd)]
    out.append("--calibration-copy adds three plain device-to-device copies of 1 GiB (1 048 576 KiB read, the same written; they run as\n"
               "__amd_rocclr_copyBuffer) to the same process.  Counter values per dispatch (KiB as reported), from the *_counter_collection.csv:\n\n")
    out.append(f"  {'kernel':50s} {'FETCH_SIZE':>12s} {'WRITE_SIZE':>12s}\n")
    out.append(f"  {'copy of 1 GiB (calibration)':50s} {copy_f:12.1f} {copy_w:12.1f}\n")
    out.append(f"  {(gu + f' (n={guf[1]})')[:50]:50s} {guf[0]:12.1f} {guw[0]:12.1f}    (fetch min {guf[2]:.1f}, max {guf[3]:.1f})\n")
    out.append(f"  {f'attn_bf16_kernel (n={att_f[1]})':50s} {att_f[0]:12.1f} {att_w[0]:12.1f}\n\n")
    out.append(f"Scale factors from the copy: FETCH_SIZE reads {1 / ff:.4f} of the bytes fetched (factor {ff:.3f}), WRITE_SIZE reads {1 / fw:.4f} of the\n"
               f"bytes written (factor {fw:.3f}).\n\nGate/up GEMM per launch:\n"
               f"  fetched  {guf[0]:10.1f} KiB x {ff:.3f} = {fetched / 1e6:7.1f} MB\n  written  {guw[0]:10.1f} KiB x {fw:.3f} = {written / 1e6:7.2f} MB\n"
               f"  traffic  {(fetched + written) / 1e6:.1f} MB against {a.algorithmic_mb:.1f} MB algorithmic (both weight matrices, bf16, once)\n\n"
               f"Attention per launch: {att_f[0] * ff * 1024 / 1e6:.1f} MB fetched, {att_w[0] * fw * 1024 / 1e6:.1f} MB written.\n\n"
               f"sev-traffic kernel=gemm_gate_up_swiglu workload={a.workload} fetch_KiB={guf[0]:.1f} write_KiB={guw[0]:.1f} fetch_factor={ff:.4f} "
               f"write_factor={fw:.4f} source_sha={kernel_source_hash()}\n")
    open(a.out, "w").write("".join(out))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    for name in ("kernel-stats", "counters", "traffic"):
        p = sub.add_parser(name)
        p.add_argument("--workload", required=True)
        p.add_argument("--cmd", required=True, help="the full profiling command, quoted verbatim in the summary")
        p.add_argument("--out", required=True)
        p.add_argument("--top", type=int, default=22)
        if name == "traffic":
            p.add_argument("--fetch-dir", required=True)
            p.add_argument("--write-dir", required=True)
            p.add_argument("--algorithmic-mb", type=float, default=234.9)
        else:
            p.add_argument("--dir", required=True)
        if name == "kernel-stats":
            p.add_argument("--bench-json")
    a = ap.parse_args()
    {"kernel-stats": kernel_stats, "counters": counters, "traffic": traffic}[a.what](a)


if __name__ == "__main__":
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    main()
