"""Turn rocprofv3 result databases (rocpd sqlite, the default output of ROCm 7) into short text summaries.

    python3 -m paper_2107_06419_amd.rocprof_summary trace_results.db [more.db ...]
    python3 -m paper_2107_06419_amd.rocprof_summary --traffic fetch_results.db write_results.db --copy-mib 1024

The first form prints per-kernel call counts and average durations, and per-kernel averages of any
counters the run collected.  The second form converts FETCH_SIZE / WRITE_SIZE (KiB per dispatch) into
HBM bytes per launch, scaling each counter by what it reads for the plain device-to-device copy of
`--copy-mib` MiB that profile_driver.py issues last, and prints a JSON object.
"""
import argparse
import json
import re
import sqlite3
import sys


def demangle_simple(name: str) -> str:
    """Names the profiler leaves mangled (its demangler gives up on some bf16 signatures): nested name plus
    integer / bool template arguments is all that this library's kernels use."""
    m = re.match(r"_ZN((?:\d+[A-Za-z_]\w*?)+?)(I(?:L[ibjm]n?\d+E)+E)?E", name)
    if not m:
        return name
    parts, rest = [], m.group(1)
    while rest:
        n = int(re.match(r"\d+", rest).group(0))
        k = len(str(n))
        parts.append(rest[k:k + n])
        rest = rest[k + n:]
    out = "::".join(parts)
    if m.group(2):
        args = []
        for kind, neg, val in re.findall(r"L([ibjm])(n?)(\d+)E", m.group(2)):
            args.append(("true" if val == "1" else "false") if kind == "b" else ("-" if neg else "") + val)
        out += "<" + ", ".join(args) + ">"
    return out


def short(name: str) -> str:
    if name.startswith("_ZN"):
        name = demangle_simple(name)
    name = re.sub(r"\(.*", "", name).replace("void ", "")
    return name[:72]


def kernel_stats(cur):
    return list(cur.execute("select name,total_calls,total_duration,average,percentage from top_kernels"))


def counter_stats(cur):
    try:
        return list(cur.execute("select kernel_name,counter_name,count(*),avg(value),min(value),max(value) "
                                "from counters_collection group by kernel_name,counter_name"))
    except sqlite3.Error:
        return []


def summarise(path: str) -> None:
    cur = sqlite3.connect(path).cursor()
    print(f"## {path}")
    rows = kernel_stats(cur)
    if rows:
        print(f"{'kernel':74s} {'calls':>6s} {'avg_us':>12s} {'total_us':>13s} {'pct':>6s}")
        for n, c, t, a, p in rows[:10]:
            print(f"{short(n):74s} {c:6d} {a:12.2f} {t:13.2f} {p:6.2f}")
    rows = counter_stats(cur)
    if rows:
        print(f"{'kernel':74s} {'counter':>28s} {'n':>3s} {'avg':>18s} {'min':>18s} {'max':>18s}")
        for n, c, k, a, mi, ma in rows:
            print(f"{short(n):74s} {c:>28s} {k:3d} {a:18.2f} {mi:18.2f} {ma:18.2f}")


def traffic(fetch_db: str, write_db: str, copy_mib: int) -> dict:
    out = {"copy_mib": copy_mib, "kernels": {}}
    per = {}
    for key, path in (("FETCH_SIZE", fetch_db), ("WRITE_SIZE", write_db)):
        cur = sqlite3.connect(path).cursor()
        vals = {short(n): a for n, c, k, a, mi, ma in counter_stats(cur) if c == key}
        copy = [v for n, v in vals.items() if "copyBuffer" in n]
        if not copy:
            raise SystemExit(f"{path}: no copy kernel found for calibration")
        scale = copy_mib * 1024.0 / copy[0]  # true KiB moved per counted KiB
        out[f"{key}_scale"] = scale
        for n, v in vals.items():
            per.setdefault(n, {})[key] = v * scale * 1024.0
    for n, d in per.items():
        if "flat::" in n:
            out["kernels"][n] = {"fetch_bytes": d.get("FETCH_SIZE"), "write_bytes": d.get("WRITE_SIZE")}
    fused = [d for n, d in out["kernels"].items() if "fwd_bf16_kernel" in n]
    unf = [d for n, d in out["kernels"].items() if "fwd_" not in n]
    if fused:
        out["fused_bytes_per_launch"] = sum((fused[0]["fetch_bytes"] or 0, fused[0]["write_bytes"] or 0))
    if unf:
        out["unfused_bytes_per_launch"] = sum((d["fetch_bytes"] or 0) + (d["write_bytes"] or 0) for d in unf)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("dbs", nargs="+")
    ap.add_argument("--traffic", action="store_true", help="dbs = FETCH_SIZE run, WRITE_SIZE run")
    ap.add_argument("--copy-mib", type=int, default=1024)
    args = ap.parse_args()
    if args.traffic:
        if len(args.dbs) != 2:
            ap.error("--traffic needs exactly two databases")
        print(json.dumps(traffic(args.dbs[0], args.dbs[1], args.copy_mib), indent=1))
        return 0
    for p in args.dbs:
        summarise(p)
    return 0


if __name__ == "__main__":
    sys.exit(main())
