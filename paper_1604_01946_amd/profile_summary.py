"""Turns the CSV output of rocprofv3 runs of bench.py into the short summaries kept under profiles/.

    python -m paper_1604_01946_amd.profile_summary stats   <dir> <prefix> <out.md>  [--title ...]
    python -m paper_1604_01946_amd.profile_summary traffic <fetch dir> <write dir> <out stem> --workload cfg3
    python -m paper_1604_01946_amd.profile_summary pmc     <out.md> <dir> [<dir> ...] [--title ...]

`stats`    reads <dir>/<prefix>_kernel_stats.csv (rocprofv3 --kernel-trace --stats) and <dir>/bench.json (the bench
           line the same command printed) and writes a markdown table of per-kernel durations next to the phases
           that bench.py timed with HIP events in that run.
`traffic`  reads the pmc_counter_collection.csv of one FETCH_SIZE pass and one WRITE_SIZE pass, scales both by
           what the same counters read for the 1 GiB device copy that `bench.py --copy-calibration` makes first,
           and writes <out stem>.md (a table) and <out stem>.json (bytes per launch per kernel; bench.py's
           `roofline.traffic` is read from that file and is null when it does not name the kernel being timed).
`pmc`      reads the pmc_counter_collection.csv of any number of counter passes (one rocprofv3 --pmc run each) and
           writes one markdown table, kernels down, counters across, averaged over the launches of each kernel.
Nothing here touches the GPU: it only reads CSV files.
"""
import argparse
import collections
import csv
import json
import os
import re
import sys

COPY_KERNEL = "__amd_rocclr_copyBuffer"
COPY_BYTES = 1 << 30


def short_name(full):
    n = full.replace("lstm::(anonymous namespace)::", "").replace("lstm::", "").replace("void ", "")
    return n.split("(")[0].strip()


def base_name(full):
    return re.sub(r"<.*", "", short_name(full))


def load_counters(path):
    """{counter: {kernel: [value per dispatch]}} from one pmc_counter_collection.csv."""
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(path) as f:
        for r in csv.DictReader(f):
            out[r["Counter_Name"]][short_name(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return out


def find_csv(d, suffix):
    for root, _, files in os.walk(d):
        for f in files:
            if f.endswith(suffix):
                return os.path.join(root, f)
    raise FileNotFoundError(f"no *{suffix} under {d}")


def bench_line(d):
    p = os.path.join(d, "bench.json")
    if not os.path.exists(p):
        return None
    lines = [l for l in open(p).read().strip().splitlines() if l.startswith("{")]
    return json.loads(lines[-1]) if lines else None


def cmd_stats(a):
    rows = list(csv.DictReader(open(find_csv(a.dir, f"{a.prefix}_kernel_stats.csv"))))
    b = bench_line(a.dir)
    L = [f"# {a.title or 'Kernel statistics'}\n"]
    if a.command:
        L += ["Command (run on the MI355X box, the program itself after `--`):\n", "    cd /tmp && export TMPDIR=/tmp", f"    {a.command}\n"]
    L.append("Kernel statistics over every pass of the run (warm-up, timed and phase-timing passes; nanoseconds):\n")
    L.append("| kernel | calls | total ns | average ns | % |\n|---|---|---|---|---|")
    for r in rows:
        if float(r["Percentage"]) < 0.05:
            continue
        n = r["Name"].replace("lstm::(anonymous namespace)::", "").replace("void ", "")
        L.append(f"| `{n[:90]}` | {r['Calls']} | {r['TotalDurationNs']} | {float(r['AverageNs']):.0f} | {float(r['Percentage']):.2f} |")
    if b:
        L.append("\nThe same run's bench line (HIP-event phase times inside bench.py, ms per pass; FLOPs as the library counts them for the products each phase really carried):\n")
        L.append("| phase | kernel | ms | GFLOP | TFLOP/s |\n|---|---|---|---|---|")
        for k, v in b["phases"].items():
            L.append(f"| {k} | {v.get('kernel', '')} | {v['ms']:.4f} | {v.get('gflop', '')} | {v.get('tflops', '')} |")
        L.append(f"\nWhole pass: {b['ms_per_step']} ms = {b['value']} {b['unit']}.  roofline: {json.dumps(b['roofline'])}\n")
    open(a.out, "w").write("\n".join(L) + "\n")
    print("wrote", a.out)


def cmd_traffic(a):
    f = load_counters(find_csv(a.fetch, "counter_collection.csv"))["FETCH_SIZE"]
    w = load_counters(find_csv(a.write, "counter_collection.csv"))["WRITE_SIZE"]
    avg = lambda d, k: (sum(d[k]) / len(d[k])) if d.get(k) else 0.0
    if COPY_KERNEL not in f or COPY_KERNEL not in w:
        sys.exit("no calibration copy in the runs: use bench.py --copy-calibration")
    # counters are in KiB; the copy read 1 GiB and wrote 1 GiB (the runtime's small staging copies run under the same
    # kernel name: the calibration copy is the largest dispatch)
    cf, cw = max(f[COPY_KERNEL]), max(w[COPY_KERNEL])
    kf = COPY_BYTES / 1024.0 / cf
    kw = COPY_BYTES / 1024.0 / cw
    kernels = {}
    rows = ["| kernel | launches | FETCH_SIZE avg (KiB, raw) | read MiB per launch | WRITE_SIZE avg (KiB, raw) | written MiB per launch |",
            "|---|---|---|---|---|---|"]
    for k in sorted(set(f) | set(w)):
        rd, wr = avg(f, k) * kf * 1024.0, avg(w, k) * kw * 1024.0
        rows.append(f"| {k[:70]} | {max(len(f.get(k, [])), len(w.get(k, [])))} | {avg(f, k):.1f} | {rd / 2**20:.1f} | {avg(w, k):.1f} | {wr / 2**20:.1f} |")
        b = base_name(k)
        if b.startswith("at::") or b.startswith("__amd"):
            continue
        e = kernels.setdefault(b, {"read_bytes": 0, "write_bytes": 0, "launches": 0, "instances": []})
        # several instances of one template (or launch shapes of one kernel): keep the one that moves the most
        if rd + wr > e["read_bytes"] + e["write_bytes"]:
            e.update(read_bytes=int(rd), write_bytes=int(wr), launches=len(f.get(k, [])))
        e["instances"].append(k)
    md = [f"# HBM traffic per launch from rocprofv3 counters: {a.workload}\n"]
    if a.command:
        md += ["Commands (two passes, one counter each, run on the MI355X box):\n", "    cd /tmp && export TMPDIR=/tmp"]
        md += [f"    {a.command.replace('COUNTER', c)}" for c in ("FETCH_SIZE", "WRITE_SIZE")]
        md.append("")
    md.append(f"Calibration: `--copy-calibration` makes one 1 GiB device-to-device copy (`{COPY_KERNEL}`).  The counters read "
              f"FETCH_SIZE = {cf:.1f} KiB and WRITE_SIZE = {cw:.1f} KiB for it, so read bytes = "
              f"FETCH_SIZE x {kf:.3f} KiB and written bytes = WRITE_SIZE x {kw:.3f} KiB.\n")
    md += rows
    if a.notes and os.path.exists(a.notes):
        md += ["", open(a.notes).read().rstrip()]
    open(a.out + ".md", "w").write("\n".join(md) + "\n")
    json.dump({"workload": a.workload, "fetch_factor": kf, "write_factor": kw, "kernels": kernels},
              open(a.out + ".json", "w"), indent=1, sort_keys=True)
    print("wrote", a.out + ".md", a.out + ".json")


def cmd_pmc(a):
    table = collections.defaultdict(dict)
    counters = []
    for d in a.dirs:
        for c, per in load_counters(find_csv(d, "counter_collection.csv")).items():
            if c not in counters:
                counters.append(c)
            for k, v in per.items():
                table[k][c] = (sum(v) / len(v), len(v))
    L = [f"# {a.title or 'Hardware counters per launch'}\n"]
    if a.command:
        L += ["Command (one run per group of counters, run on the MI355X box; COUNTERS = the group):\n", "    cd /tmp && export TMPDIR=/tmp", f"    {a.command}\n"]
    L.append("Average over the launches of each kernel:\n")
    L.append("| kernel | launches | " + " | ".join(counters) + " |\n|---|---|" + "---|" * len(counters))
    for k in sorted(table):
        if k.startswith("at::") or (a.only and not any(o in k for o in a.only)):
            continue
        n = max(v[1] for v in table[k].values())
        L.append(f"| `{k[:60]}` | {n} | " + " | ".join(f"{table[k][c][0]:.4g}" if c in table[k] else "" for c in counters) + " |")
    if a.notes and os.path.exists(a.notes):
        L += ["", open(a.notes).read().rstrip()]
    open(a.out, "w").write("\n".join(L) + "\n")
    print("wrote", a.out)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="mode", required=True)
    s = sub.add_parser("stats")
    s.add_argument("dir"); s.add_argument("prefix"); s.add_argument("out")
    s.add_argument("--title"); s.add_argument("--command")
    s.set_defaults(fn=cmd_stats)
    t = sub.add_parser("traffic")
    t.add_argument("fetch"); t.add_argument("write"); t.add_argument("out")
    t.add_argument("--workload", required=True); t.add_argument("--command"); t.add_argument("--notes")
    t.set_defaults(fn=cmd_traffic)
    p = sub.add_parser("pmc")
    p.add_argument("out"); p.add_argument("dirs", nargs="+")
    p.add_argument("--title"); p.add_argument("--command"); p.add_argument("--notes"); p.add_argument("--only", nargs="*")
    p.set_defaults(fn=cmd_pmc)
    a = ap.parse_args()
    a.fn(a)


if __name__ == "__main__":
    main()
