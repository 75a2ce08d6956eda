"""Turn rocprofv3 output (CSV) into the short text summaries kept under profiles/.

    python -m paper_2406_08128_amd.profile_summary stats   <dir>/..._kernel_stats.csv  --command "<full command>" --title "..."
    python -m paper_2406_08128_amd.profile_summary traffic --fetch <csv> --write <csv> --kernel bf16_bwd_sweep_kernel \
                                                            --copy-mib 1024 --command "..." --title "..."
    python -m paper_2406_08128_amd.profile_summary counters <..._counter_collection.csv>... --command "..." --title "..."
    python -m paper_2406_08128_amd.profile_summary stats-multi --section NAME CSV [--section NAME CSV ...] --command "..." --title "..."

Every summary starts with the commit and the hash of the kernel sources it was taken on (bench.py quotes a summary's
figures only while that hash is the tree's), the title and the command, and prints kernel names with their template
arguments.  Lines of the form `key: value` at the end are what bench.py reads back.
"""
import argparse
import collections
import csv
import re
import subprocess
import sys

from .binding import kernel_sources_sha256

ROOT = __import__("os").path.dirname(__import__("os").path.dirname(__import__("os").path.abspath(__file__)))


def demangle(name: str) -> str:
    """Kernel name with its template arguments, without namespace and parameter list."""
    n = name
    m = re.match(r"_ZN5chela(\d+)", n)
    if m:
        # (c++filt does not know the bfloat16 parameter type: the name and its integer / bool template arguments are
        # read off the mangled form directly)
        start = m.end()
        ident = n[start:start + int(m.group(1))]
        rest = n[start + int(m.group(1)):]
        args = []
        if rest.startswith("I"):
            rest = rest[1:]
            while True:
                a = re.match(r"L([ib])(\d+)E", rest)
                if a:
                    args.append(a.group(2) if a.group(1) == "i" else ("true" if a.group(2) == "1" else "false"))
                    rest = rest[a.end():]
                    continue
                t = re.match(r"DF16b|f", rest)           # type arguments: bfloat16, float
                if not t:
                    break
                args.append("bf16" if t.group(0) == "DF16b" else "float")
                rest = rest[t.end():]
        return ident + ("<%s>" % ", ".join(args) if args else "")
    if n.startswith("_Z"):
        try:
            n = subprocess.run(["c++filt", n], stdout=subprocess.PIPE, text=True, check=True).stdout.strip()
        except (OSError, subprocess.CalledProcessError):
            pass
    n = re.sub(r"^void ", "", n)
    n = n.replace("chela::", "")
    n = n.replace("bool _Accum", "bf16")      # (how rocprofv3's own demangler prints the bfloat16 type)
    depth, out = 0, []
    for ch in n:                       # cut the parameter list: the first '(' outside template brackets
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            break
        out.append(ch)
    return "".join(out).strip()


def header(title: str, command: str) -> str:
    try:
        commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "HEAD"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL,
                                text=True, check=True).stdout.strip()
        dirty = subprocess.run(["git", "-C", ROOT, "status", "--porcelain", "--", "paper_2406_08128_amd/csrc", "bench.py"],
                               stdout=subprocess.PIPE, text=True).stdout.strip()
        if dirty:
            commit += " + uncommitted changes (the hash below says which sources)"
    except (OSError, subprocess.CalledProcessError):
        commit = "unknown"
    return ("%s\n\ncommit: %s\nkernel_sources_sha256: %s\ncommand: %s\n"
            % (title, commit, kernel_sources_sha256(), command))


def cmd_stats(a):
    print(header(a.title, a.command))
    print("Source: %s (the library's kernels only)\n" % a.csv)
    print(_stats_table(a.csv))
    print()
    for r in csv.DictReader(open(a.csv)):
        if "chela" in r["Name"]:
            print("avg_ns[%s]: %.0f" % (demangle(r["Name"]).split("<")[0], float(r["AverageNs"])))
    if a.note:
        print("\n" + a.note)


def _stats_table(path):
    rows = []
    for r in csv.DictReader(open(path)):
        if "chela" not in r["Name"]:
            continue
        rows.append((demangle(r["Name"]), int(r["Calls"]), int(r["TotalDurationNs"]), float(r["AverageNs"]),
                     int(r["MinNs"]), int(r["MaxNs"])))
    tot = sum(x[2] for x in rows) or 1
    out = ["%-62s %6s %12s %10s %7s %9s %9s" % ("kernel", "calls", "total_ns", "avg_ns", "share", "min_ns", "max_ns")]
    for x in sorted(rows, key=lambda x: -x[2]):
        out.append("%-62s %6d %12d %10.0f %6.1f%% %9d %9d" % (x[0], x[1], x[2], x[3], 100.0 * x[2] / tot, x[4], x[5]))
    return "\n".join(out)


def cmd_stats_multi(a):
    """Several runs of one command pattern in one summary: --section "ARGS or name" CSV, repeated."""
    print(header(a.title, a.command))
    for name, path in a.section:
        print("== %s   (%s)" % (name, path))
        print(_stats_table(path))
        print()
    if a.note:
        print(a.note)


def _means(*paths):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in paths:
        for r in csv.DictReader(open(path)):
            if "chela" not in r["Kernel_Name"]:
                continue
            agg[demangle(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in agg.items()}


def cmd_traffic(a):
    f, w = _means(a.fetch), _means(a.write)
    print(header(a.title, a.command))
    print("FETCH_SIZE and WRITE_SIZE in KiB per dispatch, mean over the dispatches of each kernel:\n")
    print("%-62s %14s %14s" % ("kernel", "FETCH_SIZE", "WRITE_SIZE"))
    names = sorted(set(f) | set(w))
    for k in names:
        print("%-62s %14.1f %14.1f" % (k, f.get(k, {}).get("FETCH_SIZE", float("nan")), w.get(k, {}).get("WRITE_SIZE", float("nan"))))
    copy = [k for k in names if k.startswith("copy_probe_kernel")]
    if not copy:
        sys.exit("no copy_probe_kernel dispatches in the counter files: run bench.py with --copy-probe-mib")
    kib = a.copy_mib * 1024.0
    sf, sw = kib / f[copy[0]]["FETCH_SIZE"], kib / w[copy[0]]["WRITE_SIZE"]
    print("\nCalibration: the copy kernel reads and writes %d MiB per launch -> FETCH_SIZE scale %.4f, WRITE_SIZE scale %.4f"
          % (a.copy_mib, sf, sw))
    dom = [k for k in names if k.startswith(a.kernel)]
    if not dom:
        sys.exit("kernel %s not found" % a.kernel)
    total_all = 0.0
    print()
    for k in names:
        if k.startswith("copy_probe") or k.startswith("stream_probe") or k.startswith("mfma_probe"):
            continue
        rd, wr = f[k]["FETCH_SIZE"] * sf * 1024.0, w[k]["WRITE_SIZE"] * sw * 1024.0
        print("%-62s read %8.1f MB  write %8.1f MB per launch" % (k, rd / 1e6, wr / 1e6))
    rd, wr = f[dom[0]]["FETCH_SIZE"] * sf * 1024.0, w[dom[0]]["WRITE_SIZE"] * sw * 1024.0
    if a.note:
        print("\n" + a.note)
    print("\ntraffic_kernel: %s" % dom[0])
    print("traffic_bytes_per_launch: %d" % round(rd + wr))


def cmd_counters(a):
    m = _means(*a.csv)
    cols = sorted({c for d in m.values() for c in d})
    print(header(a.title, a.command))
    if len(cols) > 5:      # many counters: one kernel per block, one counter per line
        for k in sorted(m):
            print("Mean per dispatch of %s:" % k)
            for c in cols:
                if c in m[k]:
                    print("  %-28s %18.0f" % (c, m[k][c]))
            print()
    else:
        print("Mean per dispatch:\n")
        print("%-62s " % "kernel" + " ".join("%28s" % c for c in cols))
        for k in sorted(m):
            print("%-62s " % k + " ".join("%28.4e" % m[k].get(c, float("nan")) for c in cols))
    if a.kernel:
        dom = [k for k in sorted(m) if k.startswith(a.kernel)]
        if dom and "SQ_INSTS_VALU_MFMA_MOPS_BF16" in m[dom[0]]:
            d = m[dom[0]]
            flop = d["SQ_INSTS_VALU_MFMA_MOPS_BF16"] * 512.0            # one MOPS unit is 512 FLOP
            print("\nmfma_kernel: %s" % dom[0])
            print("mfma_flop_per_launch: %.6e" % flop)
            if "SQ_VALU_MFMA_BUSY_CYCLES" in d and "GRBM_GUI_ACTIVE" in d:
                # GRBM_GUI_ACTIVE is summed over the 8 XCDs; 1024 SIMDs in all
                busy = d["SQ_VALU_MFMA_BUSY_CYCLES"] / (d["GRBM_GUI_ACTIVE"] / 8.0 * 1024.0)
                print("mfma_busy_frac: %.4f" % busy)
    if a.note:
        print("\n" + a.note)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    for name in ("stats", "stats-multi", "traffic", "counters"):
        p = sub.add_parser(name)
        p.add_argument("--title", required=True)
        p.add_argument("--command", required=True)
        p.add_argument("--note", default="")
        if name == "stats":
            p.add_argument("csv")
        elif name == "stats-multi":
            p.add_argument("--section", nargs=2, action="append", required=True, metavar=("NAME", "CSV"))
        elif name == "counters":
            p.add_argument("csv", nargs="+")
            p.add_argument("--kernel", default="")
        else:
            p.add_argument("--fetch", required=True)
            p.add_argument("--write", required=True)
            p.add_argument("--kernel", required=True)
            p.add_argument("--copy-mib", type=int, default=1024)
    a = ap.parse_args()
    {"stats": cmd_stats, "stats-multi": cmd_stats_multi, "traffic": cmd_traffic, "counters": cmd_counters}[a.what](a)


if __name__ == "__main__":
    main()
