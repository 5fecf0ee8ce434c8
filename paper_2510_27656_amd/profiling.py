"""Turns rocprofv3 output of a bench.py run into the short summaries kept under
profiles/ (text only), and into profiles/hbm_traffic.json, which bench.py reads
for `roofline.traffic`.  Every stored figure carries the build id of the library
it was measured with (fl_moe_build_id), so a figure measured with other kernels
than the ones being timed is recognised as stale.

    python -m paper_2510_27656_amd.profiling kernel-trace <kt_kernel_stats.csv> <bench log> <out.md> \\
        --title "workload dsv3_decode" --command "rocprofv3 --kernel-trace ... -- python3 bench.py ..."
    python -m paper_2510_27656_amd.profiling traffic <workload> <fetch csv> <write csv> <counters log> \\
        [--tag stream_ordered] [--flags "--stream-ordered"]
    python -m paper_2510_27656_amd.profiling counters <counter csv> <out.md> --title ... --command ...
    python -m paper_2510_27656_amd.profiling timeline <kernel_trace.csv> <bench log> <out.md> --title ... --command ...

The counter CSVs are `*_counter_collection.csv` of `rocprofv3 --pmc ... --output-format csv`;
the logs are the stdout of the profiled bench.py (its JSON line is read from them).
"""
import argparse
import collections
import csv
import json
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")


def _json_line(path):
    last = None
    for line in open(path):
        if line.startswith("{"):
            last = json.loads(line)
    if last is None:
        raise SystemExit(f"no JSON line in {path}")
    return last


def _short(name):
    return name.split("(")[0].replace("void ", "")


def _counter_rows(path, wanted=None):
    """{kernel name: {counter: [value per dispatch]}}"""
    rows = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        if wanted is None or r["Counter_Name"] in wanted:
            rows[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return rows


def kernel_label(name):
    """bench.py's name of a kernel from its demangled name (the two fabric launches are
    told apart by their PHASE template argument)."""
    short = _short(name).replace("flmoe::", "")
    key = short.split("<")[0]
    if key == "fabric_copy_kernel":
        return "fabric_copy_kernel(dispatch)" if re.search(r"<(true|false), 0[,>]", name) \
            else "fabric_copy_kernel(combine)"
    if key == "fabric_private_kernel":
        return "fabric_copy_kernel(dispatch, private slots)"
    return key


def kernel_trace(stats_csv, bench_log, out_md, title, command):
    rows = [r for r in csv.DictReader(open(stats_csv)) if "flmoe" in r["Name"]]
    out = [f"# rocprofv3 kernel trace, {title}\n",
           "Command (run from /tmp with TMPDIR=/tmp on the MI355X box):\n", f"    {command}\n",
           "Per-kernel statistics (kt_kernel_stats.csv), times in microseconds:\n",
           "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    for r in rows:
        out.append(f"| {_short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | "
                   f"{float(r['MinNs']) / 1e3:.1f} | {float(r['MaxNs']) / 1e3:.1f} | {r['Percentage']} |")
    j = _json_line(bench_log)
    if "kernel_us" in j:
        out.append("\nThe same run's own HIP-event timings (bench.py, per launch, us): " + json.dumps(j["kernel_us"]))
    out.append(f"\nbench line of that run: value {j['value']} GB/s, {j['ms_per_step']} ms/step (profiler attached); "
               f"library build id {j.get('library_build_id', 'not recorded')}.")
    open(out_md, "w").write("\n".join(out) + "\n")
    print("\n".join(out))


def traffic(workload, fetch_csv, write_csv, counters_log, tag="", flags=""):
    f = _counter_rows(fetch_csv, {"FETCH_SIZE"})
    w = _counter_rows(write_csv, {"WRITE_SIZE"})
    alg = _json_line(counters_log)
    copyname = [n for n in f if "plain_copy" in n][0]
    copy_kib = alg["copy_bytes"] / 1024
    fc, wc = f[copyname]["FETCH_SIZE"], w[copyname]["WRITE_SIZE"]
    ff, wf = copy_kib / (sum(fc) / len(fc)), copy_kib / (sum(wc) / len(wc))
    key = workload + (f"_{tag}" if tag else "")
    fl = f" --workload {workload}" if workload != "dsv3_decode" else ""
    fl += f" {flags}" if flags else ""
    out = [f"# HBM traffic from rocprofv3 --pmc, workload {workload}{' (' + tag + ')' if tag else ''}\n",
           "Commands (each from /tmp with TMPDIR=/tmp; one counter per run):\n",
           f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o fetch -- python3 /root/repo/bench.py{fl} --counters",
           f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out> -o write -- python3 /root/repo/bench.py{fl} --counters",
           f"    python -m paper_2510_27656_amd.profiling traffic {workload} <fetch csv> <write csv> <log of the first run>\n",
           f"Library build id: {alg.get('library_build_id', 'not recorded')}.\n",
           f"Calibration: plain_copy_kernel of {alg['copy_bytes']} bytes reads FETCH_SIZE = {sum(fc) / len(fc):.0f} KiB and "
           f"WRITE_SIZE = {sum(wc) / len(wc):.0f} KiB, so the scale factors are {ff:.4f} (fetch) and {wf:.4f} (write).\n",
           "Figures are per launch; a call that moves several GB is issued as several launches over rank groups "
           f"(launches per step = dispatches / {alg.get('steps', 3)} steps), and the algorithmic bytes of a step are "
           "divided likewise.\n",
           "| kernel | dispatches | fetch KiB (raw avg) | write KiB (raw avg) | scaled traffic MB | algorithmic MB | traffic / algorithmic |",
           "|---|---|---|---|---|---|---|"]
    kernels = {}
    for name in f:
        if "flmoe" not in name or "plain_copy" in name:
            continue
        label = kernel_label(name)
        if label not in alg["algorithmic_bytes"]:
            continue
        fv, wv = f[name]["FETCH_SIZE"], w[name]["WRITE_SIZE"]
        per_step = len(fv) / alg.get("steps", 3)
        algb = alg["algorithmic_bytes"][label] / per_step
        t = (sum(fv) / len(fv) * ff + sum(wv) / len(wv) * wf) * 1024
        kernels[label] = int(t)
        out.append(f"| {label} | {len(fv)} | {sum(fv) / len(fv):.0f} | {sum(wv) / len(wv):.0f} | {t / 1e6:.1f} | "
                   f"{algb / 1e6:.1f} | {t / algb:.3f} |")
    open(os.path.join(PROFILES, f"hbm_traffic_{key}.md"), "w").write("\n".join(out) + "\n")
    p = os.path.join(PROFILES, "hbm_traffic.json")
    allt = json.load(open(p)) if os.path.exists(p) else {}
    allt[key] = {"library_build_id": alg.get("library_build_id"), "kernels": kernels}
    json.dump(allt, open(p, "w"), indent=1)
    print("\n".join(out))


def stored_traffic(workload, kernel, build_id, tag=""):
    """(bytes or None, note or None) for bench.py's roofline.traffic."""
    p = os.path.join(PROFILES, "hbm_traffic.json")
    if not os.path.exists(p):
        return None, "profiles/hbm_traffic.json is missing"
    entry = json.load(open(p)).get(workload + (f"_{tag}" if tag else ""))
    if not isinstance(entry, dict) or "kernels" not in entry:
        return None, "no counter run stored for this workload"
    if entry.get("library_build_id") != build_id:
        return None, (f"stored counters were measured with library build {entry.get('library_build_id')}, "
                      f"this run times build {build_id}: re-run the two --pmc passes")
    return entry["kernels"].get(kernel), None


def counters(counter_csv, out_md, title, command, per_kernel_note=""):
    """Per-kernel averages of whatever counters one --pmc pass collected."""
    rows = _counter_rows(counter_csv)
    names = sorted({c for k in rows.values() for c in k})
    out = [f"# rocprofv3 counters, {title}\n", "Command (run from /tmp with TMPDIR=/tmp on the MI355X box):\n",
           f"    {command}\n", "Average per dispatch:\n",
           "| kernel | dispatches | " + " | ".join(names) + " |", "|---|---|" + "---|" * len(names)]
    for k, cs in rows.items():
        if "flmoe" not in k:
            continue
        n = max(len(v) for v in cs.values())
        vals = [f"{sum(cs[c]) / len(cs[c]):.4g}" if cs.get(c) else "-" for c in names]
        out.append(f"| {_short(k).replace('flmoe::', '')} | {n} | " + " | ".join(vals) + " |")
    if per_kernel_note:
        out.append("\n" + per_kernel_note)
    open(out_md, "w").write("\n".join(out) + "\n")
    print("\n".join(out))


def timeline(trace_csv, bench_log, out_md, title, command, foreign=False):
    """One step of a two-stream run as a table of kernel start and end times per queue, and
    how often, over all traced steps, a receive-side kernel (gate or polling receive kernel)
    was already running when the send kernels it waits for started.
    foreign: also list the kernels that are not the library's (a caller's own work on another
    stream), by the first 40 characters of their names; the waiting statistic is left out then."""
    rows = [r for r in csv.DictReader(open(trace_csv)) if foreign or "flmoe" in r["Kernel_Name"]]
    rows = [r for r in rows if "plain_copy" not in r["Kernel_Name"] and "elementwise" not in r["Kernel_Name"]
            and "distribution" not in r["Kernel_Name"]]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    starts = [i for i, r in enumerate(rows) if "route_layout" in r["Kernel_Name"]]
    steps = [rows[a:b] for a, b in zip(starts, starts[1:] + [len(rows)])]
    if foreign:                       # the steps that ran together with the caller's kernels
        steps = [st for st in steps if any("flmoe" not in r["Kernel_Name"] for r in st)]
        usual = collections.Counter(len(st) for st in steps).most_common(1)[0][0]
        steps = [st for st in steps if len(st) == usual]
    else:
        steps = [st for st in steps if len(st) == len(steps[len(steps) // 2])]   # whole steps only
    mid = steps[len(steps) // 2]
    t0 = int(mid[0]["Start_Timestamp"])
    queues = ("the stream with the shuffle calls, and the stream with the caller's own kernels" if foreign else
              "the stream with the layout and the receive calls, and the stream with the send calls")
    out = [f"# {title}\n", "Command (from /tmp with TMPDIR=/tmp on the MI355X box):\n", f"    {command}\n",
           f"Timeline of one step from the kernel trace (us since the step's first kernel; the queues are {queues}):\n",
           "| kernel | queue | start | end |", "|---|---|---|---|"]
    for r in mid:
        name = _short(r["Kernel_Name"]) if "flmoe" in r["Kernel_Name"] else "(caller) " + r["Kernel_Name"][:40]
        out.append(f"| {name} | {r['Queue_Id']} | {(int(r['Start_Timestamp']) - t0) / 1e3:.1f} | "
                   f"{(int(r['End_Timestamp']) - t0) / 1e3:.1f} |")
    if foreign:
        j = _json_line(bench_log)
        out.append(f"\nbench line of that run (profiler attached): {json.dumps(j.get('interleaved_caller_work'))}; "
                   f"library build id {j.get('library_build_id', 'not recorded')}.")
        open(out_md, "w").write("\n".join(out) + "\n")
        print("\n".join(out))
        return

    def span(step, pred):
        ks = [r for r in step if pred(r["Kernel_Name"])]
        return (min(int(r["Start_Timestamp"]) for r in ks), max(int(r["End_Timestamp"]) for r in ks)) if ks else None
    early = late = 0
    for st in steps:
        waiter = span(st, lambda n: "arrival_gate" in n or "dispatch_unpack_kernel<true" in n)
        sender = span(st, lambda n: "fabric_copy_kernel" in n and ", 0," in n)
        if waiter and sender:
            early += waiter[0] < sender[0]
            late += waiter[1] > sender[0]
    out.append(f"\nIn {early} of {len(steps)} traced steps the first waiting receive-side kernel of the dispatch "
               f"(gate kernel, or the polling unpack kernel) started before the dispatch fabric kernel did, and in "
               f"{late} it was still running when that kernel started: the receivers were waiting on the counters, "
               "not on stream order.")
    j = _json_line(bench_log)
    out.append(f"\nStep time of that run (profiler attached): {j['ms_per_step'] * 1e3:.0f} us; library build id "
               f"{j.get('library_build_id', 'not recorded')}.")
    open(out_md, "w").write("\n".join(out) + "\n")
    print("\n".join(out))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("kernel-trace")
    a.add_argument("stats_csv"); a.add_argument("bench_log"); a.add_argument("out_md")
    a.add_argument("--title", required=True); a.add_argument("--command", required=True)
    b = sub.add_parser("traffic")
    b.add_argument("workload"); b.add_argument("fetch_csv"); b.add_argument("write_csv")
    b.add_argument("counters_log"); b.add_argument("--tag", default=""); b.add_argument("--flags", default="")
    c = sub.add_parser("counters")
    c.add_argument("counter_csv"); c.add_argument("out_md")
    c.add_argument("--title", required=True); c.add_argument("--command", required=True)
    c.add_argument("--note", default="")
    t = sub.add_parser("timeline")
    t.add_argument("trace_csv"); t.add_argument("bench_log"); t.add_argument("out_md")
    t.add_argument("--title", required=True); t.add_argument("--command", required=True)
    t.add_argument("--foreign", action="store_true")
    args = ap.parse_args()
    if args.cmd == "timeline":
        timeline(args.trace_csv, args.bench_log, args.out_md, args.title, args.command, args.foreign)
    elif args.cmd == "kernel-trace":
        kernel_trace(args.stats_csv, args.bench_log, args.out_md, args.title, args.command)
    elif args.cmd == "traffic":
        traffic(args.workload, args.fetch_csv, args.write_csv, args.counters_log, args.tag, args.flags)
    else:
        counters(args.counter_csv, args.out_md, args.title, args.command, args.note)


if __name__ == "__main__":
    main()
