"""Turns the CSV output of the rocprofv3 runs of bench.py into the short summaries kept under
profiles/: `layer_step_<workload>.md` (kernel times, memory counters, matrix-core counters) and
`traffic_<workload>.txt` (bytes per launch of every kernel, which bench.py reads for
`roofline.traffic`).

    python -m paper_2408_00232_amd.profsum --workload share --dir gpurun_out/prof_share

expects under --dir one folder per run, named as in `commands()` below: kt (kernel trace), FETCH_SIZE,
WRITE_SIZE, TCC_HIT_sum, SQ_VALU_MFMA_BUSY_CYCLES (optional). Raw output stays where it is.
`--sq` summarises one more run (SQ_WAVE_CYCLES: eight wave-level counters) into `sq_counters_<workload>.md`.
"""
import argparse
import collections
import csv
import os
import subprocess

from . import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MFMA_COUNTERS = {"f32": "SQ_INSTS_VALU_MFMA_MOPS_F32", "bf16": "SQ_INSTS_VALU_MFMA_MOPS_BF16"}
COUNTER_RUNS = ["FETCH_SIZE", "WRITE_SIZE", "TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum",
                "SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE SQ_INSTS_VALU_MFMA_MOPS_F32 SQ_INSTS_VALU_MFMA_MOPS_BF16"]


def commands(workload, order, d):
    """The rocprofv3 command lines whose output this module summarises (run from the repository root)."""
    common = f"python3 bench.py --workload {workload} --order {order} --no-cpu-baseline --no-optimised --no-rho-sweep --epochs 0"
    out = [f"rocprofv3 --kernel-trace --stats --output-format csv -d {d}/kt -o {workload} -- {common} --steps 3 --warmup 2"]
    for c in COUNTER_RUNS:
        out.append(f"rocprofv3 --pmc {c} --output-format csv -d {d}/{c.split()[0]} -o {workload} -- "
                   f"{common} --steps 2 --warmup 1 --copy-calibration")
    return out


SQ_COUNTERS = ("SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_ACTIVE_INST_ANY SQ_ACTIVE_INST_LDS SQ_LDS_BANK_CONFLICT "
               "SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES")


def sq_command(workload, order, d):
    """The rocprofv3 run behind `sq_counters_<workload>.md` (eight SQ counters: one pass)."""
    return (f"rocprofv3 --pmc {SQ_COUNTERS} --output-format csv -d {d}/SQ_WAVE_CYCLES -o {workload} -- "
            f"python3 bench.py --workload {workload} --order {order} --no-cpu-baseline --no-optimised --no-rho-sweep "
            f"--epochs 0 --steps 2 --warmup 1")


def summarise_sq(workload, order, d, out_dir):
    """Wave-level counters per kernel: residency, how the waves' time splits, LDS activity."""
    S = counters(d, "SQ_WAVE_CYCLES", workload)
    sha = build.sources_sha()
    L = [f"# rocprofv3 SQ counters: workload `{workload}`, order `{order}` (one MI355X)\n",
         f"Library sources `{sha}` (paper_2408_00232_amd.build.sources_sha).\n",
         "Command (from the repository root, `export TMPDIR=/tmp`; summary by "
         f"`python -m paper_2408_00232_amd.profsum --sq --workload {workload} --order {order} --dir {d}`):\n",
         "```", sq_command(workload, order, d), "```\n",
         "Per-launch averages. SQ_BUSY_CYCLES is summed over the 32 shader engines (kernel cycles = value / 32); "
         "SQ_WAVE_CYCLES, SQ_WAIT_* and SQ_ACTIVE_* are summed over wavefronts in units of 4 cycles; waves / SIMD = "
         "4 x SQ_WAVE_CYCLES / kernel cycles / 1024 SIMDs; MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (1024 x kernel "
         "cycles).\n",
         "| kernel | launches | kernel Mcycles | waves / SIMD | MFMA busy % | wait-any % of wave time | wait-issue % | "
         "LDS active (M quad-cycles) | LDS bank conflict (M) |", "|---|---:|---:|---:|---:|---:|---:|---:|---:|"]
    for k, c in S.items():
        if "cdf::" not in k:
            continue
        av = {n: mean(v) for n, v in c.items()}
        cyc = av["SQ_BUSY_CYCLES"] / 32
        wave = max(av["SQ_WAVE_CYCLES"], 1.0)
        L.append("| `%s` | %d | %.2f | %.2f | %.1f | %.1f | %.1f | %.1f | %.1f |" % (
            k, len(c["SQ_BUSY_CYCLES"]), cyc / 1e6, 4 * av["SQ_WAVE_CYCLES"] / max(cyc, 1.0) / 1024,
            100 * av["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024 * max(cyc, 1.0)), 100 * av["SQ_WAIT_ANY"] / wave,
            100 * av["SQ_WAIT_INST_ANY"] / wave, av["SQ_ACTIVE_INST_LDS"] / 1e6, av["SQ_LDS_BANK_CONFLICT"] / 1e6))
    os.makedirs(out_dir, exist_ok=True)
    path = os.path.join(out_dir, f"sq_counters_{workload}.md")
    with open(path, "w") as fh:
        fh.write("\n".join(L) + "\n")
    return path


def short(name):
    return name.replace("void ", "").split("(")[0]


def base(name):
    return short(name).replace("cdf::", "").split("<")[0]


def counters(d, tag, workload):
    path = os.path.join(d, tag, f"{workload}_counter_collection.csv")
    a = collections.defaultdict(lambda: collections.defaultdict(list))
    if not os.path.exists(path):
        return a
    for r in csv.DictReader(open(path)):
        a[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return a


def mean(xs):
    return sum(xs) / len(xs)


def summarise(workload, order, d, out_dir):
    try:
        commit = subprocess.check_output(["git", "rev-parse", "--short", "HEAD"], cwd=ROOT, text=True).strip()
    except Exception:
        commit = "unknown"
    sha = build.sources_sha()
    L = [f"# rocprofv3 summary: whole layer step, workload `{workload}`, order `{order}` (one MI355X)\n",
         f"Library sources `{sha}` (paper_2408_00232_amd.build.sources_sha), on top of commit `{commit}`.\n",
         "Commands (from the repository root, `export TMPDIR=/tmp`; summary by "
         f"`python -m paper_2408_00232_amd.profsum --workload {workload} --order {order} --dir {d}`):\n", "```"]
    L += commands(workload, order, d) + ["```\n"]

    rows = list(csv.DictReader(open(os.path.join(d, "kt", f"{workload}_kernel_stats.csv"))))
    L += ["## Kernel time (`--kernel-trace --stats`, library kernels only; warm-up, timed and per-layer passes together)\n",
          "| kernel | calls | avg ms | min ms | max ms | total ms |", "|---|---:|---:|---:|---:|---:|"]
    comb = collections.OrderedDict()
    for r in rows:
        if "cdf::" in r["Name"] or r["Name"].startswith("copy_kernel"):
            L.append("| `%s` | %s | %.3f | %.3f | %.3f | %.1f |" % (
                short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e6, float(r["MinNs"]) / 1e6,
                float(r["MaxNs"]) / 1e6, float(r["TotalDurationNs"]) / 1e6))
        if "cdf::" in r["Name"]:
            c = comb.setdefault(base(r["Name"]), [0, 0.0, 0])
            c[0] += int(r["Calls"])
            c[1] += float(r["TotalDurationNs"])
            c[2] += 1
    L.append("\nTemplate instances of one kernel taken together (what bench.py's per-kernel events average over): " +
             "; ".join("`%s` %d calls, avg %.3f ms" % (b, c[0], c[1] / c[0] / 1e6) for b, c in comb.items()) + ".")

    F, Wr, T = counters(d, "FETCH_SIZE", workload), counters(d, "WRITE_SIZE", workload), counters(d, "TCC_HIT_sum", workload)
    ck = [k for k in F if k.startswith("copy_kernel")]
    fs = ws = 1.0
    if ck and ck[0] in Wr:
        fs = 1048576.0 / mean(F[ck[0]]["FETCH_SIZE"])
        ws = 1048576.0 / mean(Wr[ck[0]]["WRITE_SIZE"])
        L += ["\n## Memory counters (`--pmc`, one counter set per run)\n",
              f"Calibration: the library's plain copy kernel moved 1 GiB (1048576 KiB each way); the counters read "
              f"FETCH_SIZE = {mean(F[ck[0]]['FETCH_SIZE']):.0f} KiB and WRITE_SIZE = {mean(Wr[ck[0]]['WRITE_SIZE']):.0f} KiB, "
              f"so readings are scaled by {fs:.3f} (fetch) and {ws:.3f} (write). These counters sit between the L2 and "
              f"the fabric: they count L2 misses and write-backs, in front of the memory-side cache.\n"]
    L += ["| kernel | launches | fetch GB / launch | write GB / launch | L2 hit rate |", "|---|---:|---:|---:|---:|"]
    per = collections.OrderedDict()
    for k in F:
        if "cdf::" not in k:
            continue
        f = [x * 1024 * fs for x in F[k]["FETCH_SIZE"]]
        w = [x * 1024 * ws for x in Wr[k]["WRITE_SIZE"]] if k in Wr else []
        hit = sum(T[k]["TCC_HIT_sum"]) / max(sum(T[k]["TCC_REQ_sum"]), 1) if k in T else float("nan")
        L.append("| `%s` | %d | %.3f | %.3f | %.2f |" % (k, len(f), mean(f) / 1e9, (mean(w) if w else 0) / 1e9, hit))
        c = per.setdefault(base(k), [[], []])
        c[0] += f
        c[1] += w
    for k in F:
        if base(k) in ("spmm_kernel", "spmm_sliced_kernel"):
            v = [x * 1024 * fs / 1e9 for x in F[k]["FETCH_SIZE"]]
            L.append("\n`%s` fetch GB of its first launches, in launch order: %s" % (k, ", ".join("%.2f" % x for x in v[:6])))

    M = counters(d, "SQ_VALU_MFMA_BUSY_CYCLES", workload)
    if M:
        L += ["\n## Matrix-core utilisation of the dense kernels\n",
              "MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x cycles), cycles = GRBM_GUI_ACTIVE / 8 (the counter is "
              "summed over the 8 XCDs); executed flops = SQ_INSTS_VALU_MFMA_MOPS_{F32,BF16} x 512.\n",
              "| kernel | launches | MFMA busy % | executed GFLOP / launch (fp32 + bf16 instructions) | cycles / launch |",
              "|---|---:|---:|---:|---:|"]
        for k, c in M.items():
            if "gemm" not in k:
                continue
            av = {n: mean(v) for n, v in c.items()}
            cyc = av["GRBM_GUI_ACTIVE"] / 8
            gf = sum(av.get(n, 0.0) for n in MFMA_COUNTERS.values()) * 512 / 1e9
            L.append("| `%s` | %d | %.1f | %.1f | %.3g |" % (
                k, len(c["GRBM_GUI_ACTIVE"]), 100 * av["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024 * cyc), gf, cyc))
    os.makedirs(out_dir, exist_ok=True)
    with open(os.path.join(out_dir, f"layer_step_{workload}.md"), "w") as fh:
        fh.write("\n".join(L) + "\n")
    with open(os.path.join(out_dir, f"traffic_{workload}.txt"), "w") as fh:
        fh.write(f"# bytes per launch at the L2 <-> fabric interface from the two --pmc runs summarised in "
                 f"layer_step_{workload}.md\n")
        fh.write(f"# workload={workload} order={order} kernels_sha={sha} commit={commit}\n")
        fh.write(f"# kernel = fetch_bytes write_bytes, all template instances of a kernel together, averaged over "
                 f"their launches (scaled by the copy-kernel calibration: fetch x{fs:.3f}, write x{ws:.3f})\n")
        for b, (f, w) in per.items():
            fh.write(f"{b} = {mean(f):.0f} {(mean(w) if w else 0):.0f}\n")
    return os.path.join(out_dir, f"layer_step_{workload}.md")


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="share")
    ap.add_argument("--order", default="aggregate")
    ap.add_argument("--dir", required=True, help="folder that holds the rocprofv3 output folders")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    ap.add_argument("--print-commands", action="store_true")
    ap.add_argument("--sq", action="store_true", help="summarise the SQ counter run (sq_counters_<workload>.md) instead")
    args = ap.parse_args(argv)
    if args.print_commands:
        print("\n".join(commands(args.workload, args.order, args.dir) + [sq_command(args.workload, args.order, args.dir)]))
        return
    if args.sq:
        print(open(summarise_sq(args.workload, args.order, args.dir, args.out)).read())
        return
    print(open(summarise(args.workload, args.order, args.dir, args.out)).read())


if __name__ == "__main__":
    main()
