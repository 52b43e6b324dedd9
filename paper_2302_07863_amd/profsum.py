"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2302_07863_amd.profsum stats  <kernel_stats.csv>
  python -m paper_2302_07863_amd.profsum pmc    <fetch counter_collection.csv> <write counter_collection.csv>
  python -m paper_2302_07863_amd.profsum counters <counter_collection.csv>
  python -m paper_2302_07863_amd.profsum passes <kernel_trace.csv> [passes]

`passes` lists, per kernel instantiation and launch size, the launches of the last `passes` (default 10) decoder passes
of a `bench.py --profile-run --profile-rows T` run (a pass ends with the policy kernel).
`stats` groups the template instantiations of one kernel under one name and prints calls,
total and mean duration.  `pmc` scales FETCH_SIZE / WRITE_SIZE per dispatch by what the same
counters read for bild::probe_copy_kernel, a plain copy of known size (1 GiB read, 1 GiB written).
"""
from __future__ import annotations

import collections
import csv
import re
import sys

PROBE_BYTES = 1 << 30


# The decode GEMM is one device function behind four launch wrappers (any row count, exactly one row, two to
# four rows, input still in key-split attention partials); they are summed under one name.  The encoder / prefill
# wrapper (row blocks, bild::gemm_rows_kernel) works in another regime and stays separate.
_DECODE_GEMM = ("bild::gemm_kernel", "bild::gemm_row_kernel", "bild::gemm_few_kernel", "bild::gemm_merge_kernel",
                "bild::gemm_pre_kernel", "bild::gemm_merge_nx_kernel", "bild::gemm_part_row_kernel", "bild::gemm_part_few_kernel")


def _group(name: str) -> str:
    name = name.split("(")[0].replace("void ", "").strip()
    base = re.sub(r"<.*>$", "", name)
    if base in _DECODE_GEMM:
        return "bild::gemm_kernel<*>"
    return base + "<*>" if "<" in name else name


def stats(path: str) -> str:
    agg = collections.defaultdict(lambda: [0, 0])
    for r in csv.DictReader(open(path)):
        g = agg[_group(r["Name"])]
        g[0] += int(r["Calls"])
        g[1] += int(r["TotalDurationNs"])
    total = sum(v[1] for v in agg.values())
    lines = [f"{'kernel':34s} {'calls':>8s} {'total_ms':>10s} {'mean_us':>9s} {'share':>7s}"]
    for k, (n, t) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        lines.append(f"{k:34s} {n:8d} {t / 1e6:10.2f} {t / n / 1e3:9.2f} {100.0 * t / total:6.1f}%")
    g = agg.get("bild::gemm_kernel<*>")
    if g:
        lines.append(f"gemm_mean_us={g[1] / g[0] / 1e3:.3f}")
    return "\n".join(lines)


def _pmc(path: str):
    agg = collections.defaultdict(lambda: [0, 0.0])
    for r in csv.DictReader(open(path)):
        g = agg[_group(r["Kernel_Name"])]
        g[0] += 1
        g[1] += float(r["Counter_Value"])
    return agg


def pmc(fetch_path: str, write_path: str) -> str:
    f, w = _pmc(fetch_path), _pmc(write_path)
    probe = "bild::probe_copy_kernel"
    sf = PROBE_BYTES / (f[probe][1] / f[probe][0])
    sw = PROBE_BYTES / (w[probe][1] / w[probe][0])
    lines = [f"scale: FETCH_SIZE count = {sf:.1f} B, WRITE_SIZE count = {sw:.1f} B "
             f"(from {probe}: {PROBE_BYTES} B read and written per launch)",
             f"{'kernel':34s} {'dispatches':>10s} {'fetch_B/launch':>15s} {'write_B/launch':>15s}"]
    for k in sorted(f, key=lambda k: -f[k][1]):
        n = f[k][0]
        fb = f[k][1] / n * sf
        wb = (w[k][1] / w[k][0] * sw) if k in w else 0.0
        lines.append(f"{k:34s} {n:10d} {fb:15.0f} {wb:15.0f}")
        if k.startswith("bild::gemm_kernel"):
            lines.append(f"traffic_bytes_per_launch={fb + wb:.0f}")
    return "\n".join(lines)


def counters(path: str) -> str:
    """Sums every counter of a --pmc run per kernel group: one line per group with dispatches and, per counter, the
    mean value per dispatch."""
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    disp = collections.defaultdict(set)
    for r in csv.DictReader(open(path)):
        g = _group(r["Kernel_Name"])
        agg[g][r["Counter_Name"]] += float(r["Counter_Value"])
        disp[g].add(r["Dispatch_Id"])
    names = sorted({c for v in agg.values() for c in v})
    lines = [f"{'kernel':34s} {'dispatches':>10s} " + " ".join(f"{c:>24s}" for c in names)]
    for g in sorted(agg, key=lambda k: -len(disp[k])):
        n = len(disp[g])
        lines.append(f"{g:34s} {n:10d} " + " ".join(f"{agg[g].get(c, 0.0) / n:24.1f}" for c in names))
    return "\n".join(lines)


def verify(path: str) -> str:
    """Counter run of `bench.py --workload verify`: the dispatch list is cut at every run of bild::probe_empty_kernel
    (the benchmark launches one before each row count 1, 4, 8, 16, 32); per segment and kernel group the mean of
    every counter over the dispatches.  MfmaUtil is the profiler's derived counter: matrix-core busy cycles over
    (GPU active cycles x SIMDs), in percent."""
    rows = list(csv.DictReader(open(path)))
    by_disp = collections.OrderedDict()
    for r in sorted(rows, key=lambda r: int(r["Dispatch_Id"])):
        d = by_disp.setdefault(int(r["Dispatch_Id"]), dict(kernel=_group(r["Kernel_Name"]), c={}))
        d["c"][r["Counter_Name"]] = float(r["Counter_Value"])
    segs, cur, in_sep = [], None, False
    for d in by_disp.values():
        if d["kernel"] == "bild::probe_empty_kernel":
            if not in_sep:
                cur = collections.defaultdict(list)
                segs.append(cur)
            in_sep = True
            continue
        in_sep = False
        if cur is not None:
            cur[d["kernel"]].append(d["c"])
    t_values = (1, 4, 8, 16, 32)
    lines = []
    for i, seg in enumerate(segs[:len(t_values)]):
        T = t_values[i]
        lines.append(f"rows T={T}")
        for k, ds in sorted(seg.items(), key=lambda kv: -len(kv[1])):
            names = sorted({c for d in ds for c in d})
            means = {c: sum(d.get(c, 0.0) for d in ds) / len(ds) for c in names}
            lines.append(f"  {k:34s} dispatches {len(ds):6d}  " + "  ".join(f"{c}={means[c]:.4g}" for c in names))
            if k == "bild::gemm_kernel<*>" and "MfmaUtil" in means:
                lines.append(f"mfma_util_T{T}={means['MfmaUtil'] / 100.0:.5f}")
    return "\n".join(lines)


def passes(path: str, count: int = 10) -> str:
    rows = sorted(csv.DictReader(open(path)), key=lambda r: int(r["Start_Timestamp"]))
    fin = [i for i, r in enumerate(rows) if "finish" in r["Kernel_Name"]]
    if not fin:
        return "no policy kernel in the trace: not a run of decoder passes"
    lo = fin[-count - 1] + 1 if len(fin) > count else 0
    sel = rows[lo:fin[-1] + 1]
    agg = collections.defaultdict(list)
    for r in sel:
        name = re.sub(r"\(.*$", "", r["Kernel_Name"].replace("void ", ""))
        agg[(name, int(r["Grid_Size_X"]) // max(int(r["Workgroup_Size_X"]), 1) * max(int(r.get("Grid_Size_Y", 1) or 1), 1),
             r["Workgroup_Size_X"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    n_pass = min(count, len(fin))
    busy = sum(sum(v) for v in agg.values())
    lines = [f"passes={n_pass} launches_per_pass={len(sel) / n_pass:.0f} kernel_busy_us_per_pass={busy / n_pass:.1f}",
             f"{'kernel (template arguments as compiled)':60s} {'workgroups':>10s} {'threads':>7s} {'per_pass':>8s} {'mean_us':>8s} {'us_per_pass':>11s}"]
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        lines.append(f"{k[0][:60]:60s} {k[1]:10d} {k[2]:>7s} {len(v) / n_pass:8.1f} {sum(v) / len(v):8.2f} {sum(v) / n_pass:11.1f}")
    return "\n".join(lines)


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "passes":
        print(passes(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 10))
    elif len(sys.argv) >= 3 and sys.argv[1] == "verify":
        print(verify(sys.argv[2]))
    elif len(sys.argv) >= 3 and sys.argv[1] == "stats":
        print(stats(sys.argv[2]))
    elif len(sys.argv) >= 3 and sys.argv[1] == "counters":
        print(counters(sys.argv[2]))
    elif len(sys.argv) >= 4 and sys.argv[1] == "pmc":
        print(pmc(sys.argv[2], sys.argv[3]))
    else:
        print(__doc__)
        sys.exit(2)
