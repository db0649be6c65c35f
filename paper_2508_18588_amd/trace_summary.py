"""Per-step kernel table from a rocprofv3 kernel trace of a program that drives the library.

    python -m paper_2508_18588_amd.trace_summary <..._kernel_trace.csv> <n_steps> [skip_last]

A step starts at each launch of the draft scan kernel (the first kernel of hs_draft).  The table covers the last
n_steps steps of the trace (optionally skipping the last skip_last ones): launches per step, average duration
(End - Start) and milliseconds per step for every kernel, largest first.
"""
import collections
import csv
import sys


def summarise(path: str, n_steps: int, skip: int = 0) -> str:
    rows = list(csv.DictReader(open(path)))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    starts = [i for i, r in enumerate(rows) if "draft_scan" in r["Kernel_Name"]]
    if len(starts) < n_steps + skip:
        raise SystemExit(f"trace holds {len(starts)} steps, {n_steps + skip} asked for")
    first = starts[-(n_steps + skip)]
    last = starts[-skip] if skip else len(rows)
    agg = collections.defaultdict(lambda: [0, 0])
    for r in rows[first:last]:
        name = r["Kernel_Name"].replace("void ", "").replace("(anonymous namespace)::", "").split("(")[0]
        if name.startswith("_Z"):       # a name the profiler's demangler did not take (e.g. _Float16 arguments)
            import re
            m = re.search(r"_GLOBAL__N_1\d+([A-Za-z_]+?)I(?:Li(\d+)E)+", name)
            if m:
                name = m.group(1) + "<" + ", ".join(re.findall(r"Li(\d+)E", name.split(m.group(1), 1)[1].split("EEv")[0])) + ">"
        agg[name][0] += 1
        agg[name][1] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    total = sum(v[1] for v in agg.values())
    span = int(rows[last - 1]["End_Timestamp"]) - int(rows[first]["Start_Timestamp"])
    out = [f"{n_steps} steps: kernel time {total / 1e6 / n_steps:.3f} ms/step, wall span {span / 1e6 / n_steps:.3f} ms/step"]
    for name, (calls, ns) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        out.append(f"{name[:60]:60s} calls/step {calls / n_steps:7.1f}  avg {ns / calls / 1e3:9.1f} us  "
                   f"ms/step {ns / 1e6 / n_steps:8.3f}")
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) < 3:
        raise SystemExit(__doc__)
    print(summarise(sys.argv[1], int(sys.argv[2]), int(sys.argv[3]) if len(sys.argv) > 3 else 0))
