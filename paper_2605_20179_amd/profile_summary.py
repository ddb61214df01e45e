"""Measurement tooling, not part of the hot path (nothing in the library, the binding, the tests or bench.py imports
it): it lives in the package only so that the commands quoted under profiles/ can name it with `python -m`.

Summarise a rocprofv3 --kernel-trace CSV of a bench.py run: per kernel, launches and
mean/min/max duration over (a) every launch and (b) the launches of bench.py's timed region
(launch numbers warmup .. warmup+steps-1 of each step kernel).

usage: python -m paper_2605_20179_amd.profile_summary <kernel_trace.csv> --warmup W --steps K
       python -m paper_2605_20179_amd.profile_summary <counter_collection.csv> --pmc --warmup W --steps K"""
import argparse
import csv
import collections


def short(name: str) -> str:
    name = name.replace("tide::(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0].replace(", ", ",")          # no blanks inside a name: the summaries are column text


def pmc(path: str, warmup: int, steps: int) -> None:
    """Per kernel and counter: mean over all dispatches and over the timed-region dispatches."""
    rows = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(path) as f:
        for r in csv.DictReader(f):
            rows[short(r["Kernel_Name"])][r["Counter_Name"]].append((int(r["Dispatch_Id"]), float(r["Counter_Value"])))
    print("%-40s %-14s %8s %16s | %8s %16s" % ("kernel", "counter", "launches", "mean(all)", "timed", "mean(timed)"))
    for k, d in sorted(rows.items()):
        for c, v in sorted(d.items()):
            v.sort()
            x = [val for _, val in v]
            t = x[warmup:warmup + steps] if len(x) >= warmup + steps else []
            print("%-40s %-14s %8d %16.1f | %8d %16s" % (k[:40], c, len(x), sum(x) / len(x), len(t),
                                                           "%.1f" % (sum(t) / len(t)) if t else "-"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("trace")
    ap.add_argument("--warmup", type=int, required=True)
    ap.add_argument("--steps", type=int, required=True)
    ap.add_argument("--pmc", action="store_true", help="the file is a rocprofv3 --pmc counter_collection CSV")
    a = ap.parse_args()
    if a.pmc:
        pmc(a.trace, a.warmup, a.steps)
        return
    rows = collections.defaultdict(list)
    with open(a.trace) as f:
        for r in csv.DictReader(f):
            rows[short(r["Kernel_Name"])].append((int(r["Start_Timestamp"]), int(r["End_Timestamp"])))
    print("%-34s %8s %12s | %8s %12s %10s %10s" % ("kernel", "launches", "mean_us(all)", "timed", "mean_us", "min_us", "max_us"))
    for k, v in sorted(rows.items(), key=lambda kv: -sum(e - s for s, e in kv[1])):
        v.sort()
        d = [(e - s) / 1e3 for s, e in v]
        t = d[a.warmup:a.warmup + a.steps] if len(d) >= a.warmup + a.steps else []
        line = "%-34s %8d %12.2f | " % (k[:34], len(d), sum(d) / len(d))
        line += "%8d %12.2f %10.2f %10.2f" % (len(t), sum(t) / len(t), min(t), max(t)) if t else "%8s" % "-"
        print(line)


if __name__ == "__main__":
    main()
