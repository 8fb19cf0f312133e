"""Turn rocprofv3 CSV output of a bench.py run into the short text summaries kept under profiles/.

    python -m paper_2502_02770_amd.rocprof_summary trace  <dir-with-*_kernel_trace.csv>  "<title>" "<command>" > profiles/<name>.md
    python -m paper_2502_02770_amd.rocprof_summary traffic <fetch-dir> <write-dir> "<title>" "<command>" > profiles/<name>.md

`trace`   one table row per kernel: calls, median / average / min / max duration in ns
          (rocprofv3 --kernel-trace --stats --output-format csv).
`traffic` one row per (kernel, grid): median FETCH_SIZE and WRITE_SIZE in KiB per dispatch from two
          --pmc runs, with the calibration factors taken from the plain copy kernel that
          `bench.py --calib-copy` runs in the same process (it reads and writes 256 MiB).

bench.py reads both tables back (`read_trace_table`, `read_traffic_table`) to put the profiled
duration and the HBM traffic of its dominant kernel beside the live figure.
"""
import collections
import csv
import glob
import os
import re
import sys

CALIB_BYTES = 256 << 20          # bench.py --calib-copy: torch.add over 256 MiB of uint8 (reads and writes that much)


def short_name(k):
    """Kernel name without namespaces / argument lists: `page_score_kernel<4, true>`."""
    if "CUDAFunctorOnSelf_add<unsigned char>" in k:
        return "torch_add_u8"                    # bench.py --calib-copy
    if "at::native" in k or "elementwise" in k:
        return "torch_elementwise"
    m = re.search(r"(\w+_kernel(?:<[^>]*>)?)", k)
    return m.group(1) if m else k[:60]


def _one(pattern, d):
    f = sorted(glob.glob(os.path.join(d, "**", pattern), recursive=True))
    if not f:
        raise SystemExit("no %s under %s" % (pattern, d))
    return f[0]


def trace_rows(d):
    dur = collections.defaultdict(list)
    grid = {}
    for r in csv.DictReader(open(_one("*kernel_trace.csv", d))):
        k = short_name(r["Kernel_Name"])
        dur[k].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
        grid[k] = "%sx%s" % (r.get("Grid_Size_X", r.get("Grid_Size", "?")), r.get("Grid_Size_Y", "1"))
    rows = []
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        if k.startswith("torch_") or "rocclr" in k or "Cijk" in k:
            continue
        v = sorted(v)
        rows.append((k, grid[k], len(v), v[len(v) // 2], sum(v) // len(v), v[0], v[-1]))
    return rows


def write_trace(d, title, command, out=sys.stdout):
    out.write("# %s\n\nCommand (from /tmp on the MI355X box, TMPDIR=/tmp):\n\n    %s\n\n" % (title, command))
    out.write("Durations in ns, from the kernel trace's start and end timestamps.\n\n")
    out.write("| Kernel | Grid (threads) | Calls | Median | Average | Min | Max |\n|---|---|---|---|---|---|---|\n")
    for r in trace_rows(d):
        out.write("| `%s` | %s | %d | %d | %d | %d | %d |\n" % r)


def counter_rows(d):
    a = collections.defaultdict(list)
    for r in csv.DictReader(open(_one("*counter_collection.csv", d))):
        a[(short_name(r["Kernel_Name"]), r["Grid_Size"])].append(float(r["Counter_Value"]))
    return {k: sorted(v)[len(v) // 2] for k, v in a.items()}, {k: len(v) for k, v in a.items()}


def write_traffic(dfetch, dwrite, title, command, out=sys.stdout):
    fe, nfe = counter_rows(dfetch)
    wr, _ = counter_rows(dwrite)
    cal = [k for k in fe if k[0] == "torch_add_u8" and int(k[1]) * 16 == CALIB_BYTES and k in wr]
    if not cal:
        raise SystemExit("no calibration copy (run bench.py with --calib-copy)")
    ffac = CALIB_BYTES / 1024.0 / fe[cal[0]]
    wfac = CALIB_BYTES / 1024.0 / wr[cal[0]]
    out.write("# %s\n\nCommands (two separate runs, from /tmp on the MI355X box, TMPDIR=/tmp):\n\n" % title)
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        out.write("    " + command.replace("COUNTER", c) + "\n")
    out.write("\nCounter values are KiB per dispatch (median over the dispatches of the kernel at that grid size).\n"
              "Calibration: the plain copy kernel of `--calib-copy` reads 256 MiB and writes 256 MiB; it shows FETCH_SIZE = %.0f KiB and\n"
              "WRITE_SIZE = %.0f KiB, so the counters are scaled by **%.3f** (FETCH_SIZE) and **%.3f** (WRITE_SIZE) to bytes.\n\n"
              % (fe[cal[0]], wr[cal[0]], ffac, wfac))
    out.write("| Kernel | Grid (threads) | Dispatches | FETCH_SIZE KiB | WRITE_SIZE KiB | HBM bytes per dispatch (scaled) |\n|---|---|---|---|---|---|\n")
    for k in sorted(fe, key=lambda k: -fe[k]):
        if k[0].startswith("torch_") or "rocclr" in k[0] or k not in wr:
            continue
        out.write("| `%s` | %s | %d | %.0f | %.0f | %d |\n" % (k[0], k[1], nfe[k], fe[k], wr[k],
                                                              int((fe[k] * ffac + wr[k] * wfac) * 1024)))


def _table(path):
    rows = []
    if not os.path.exists(path):
        return rows
    for line in open(path):
        if line.startswith("| `"):
            rows.append([c.strip().strip("`") for c in line.strip().strip("|").split("|")])
    return rows


def read_trace_table(path):
    """-> {kernel name: {"calls", "median_ns", "avg_ns"}} from a summary written by `trace`."""
    out = {}
    for r in _table(path):
        try:
            out[r[0]] = {"calls": int(r[2]), "median_ns": int(r[3]), "avg_ns": int(r[4])}
        except (IndexError, ValueError):         # a table of another layout
            pass
    return out


def read_traffic_table(path):
    """-> {(kernel name, grid): HBM bytes per dispatch} from a summary written by `traffic`."""
    out = {}
    for r in _table(path):
        try:
            out[(r[0], r[1])] = int(r[5])
        except (IndexError, ValueError):
            pass
    return out


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "trace":
        write_trace(sys.argv[2], sys.argv[3], sys.argv[4])
    elif len(sys.argv) >= 6 and sys.argv[1] == "traffic":
        write_traffic(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5])
    else:
        raise SystemExit(__doc__)
