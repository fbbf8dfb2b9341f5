"""Text summaries of rocprofv3 runs (rocpd sqlite output) for this library's kernels.

  python profile_summary.py kernels  DIR OUT.txt --cmd "..."
  python profile_summary.py counters DIR OUT.txt --cmd "..."
  python profile_summary.py traffic  FETCH_DIR WRITE_DIR OUT.txt
         --copy-bytes N --cmd "..." [--cmd "..."]

`kernels` lists calls / total / average duration per kernel of a --kernel-trace run;
`counters` lists the per-dispatch average of every collected counter per kernel;
`traffic` turns one FETCH_SIZE run and one WRITE_SIZE run into HBM bytes per launch,
scaled by what the same counters read for `calibration_copy_kernel`, whose traffic is
known (N bytes read, N bytes written).  bench.py reads the "traffic_bytes_per_launch"
lines of the file written by `traffic`.
"""
from __future__ import annotations

import argparse
import collections
import sqlite3
from pathlib import Path

COPY_KERNEL = "calibration_copy_kernel"


def _db(path: str) -> sqlite3.Connection:
    p = Path(path)
    if p.is_dir():
        found = sorted(p.rglob("*.db"))
        if not found:
            raise SystemExit(f"no rocpd database under {p}")
        p = found[-1]
    return sqlite3.connect(str(p))


def _short(name: str) -> str:
    for key in ("fwd_worker_kernel<8>", "fwd_worker_kernel<4>", "bwd_worker_kernel<8>",
                "bwd_worker_kernel<4>"):
        if key in name:
            return key
    name = name.split("(")[0]
    return name.split("::")[-1][:60]


def kernel_rows(con):
    q = "select name,total_calls,total_duration,average,percentage from top_kernels"
    return [(n, int(c), float(t), float(a), float(p)) for n, c, t, a, p in con.execute(q)]


def counter_avgs(con):
    q = ("select kernel_name, counter_name, avg(value), count(*) from counters_collection "
         "group by kernel_name, counter_name")
    out = collections.defaultdict(dict)
    for k, n, v, c in con.execute(q):
        out[k][n] = (float(v), int(c))
    return out


def counter_avgs_by_cycle(con, cycles):
    """{kernel: {phase: {counter: (avg, dispatches)}}} for the kernels named in `cycles`
    ({short kernel name: launches per pass}): the i-th dispatch of such a kernel, in dispatch
    order, is launch i % cycle of a pass (a staged schedule launches the worker kernel once per
    phase, always in the same order)."""
    q = ("select kernel_name, dispatch_id, counter_name, value from counters_collection "
         "order by dispatch_id")
    seen, acc = {}, {}
    for k, disp, c, v in con.execute(q):
        name = _short(k)
        if name not in cycles:
            continue
        order = seen.setdefault(name, {})
        if disp not in order:
            order[disp] = len(order)
        ph = order[disp] % cycles[name]
        tot = acc.setdefault(name, {}).setdefault(ph, {}).setdefault(c, [0.0, 0])
        tot[0] += v
        tot[1] += 1
    return {k: {ph: {c: (t[0] / t[1], t[1]) for c, t in d.items()} for ph, d in phs.items()}
            for k, phs in acc.items()}


def _header(f, cmds):
    f.write("commands (MI355X box, from the repo root after `cd /tmp; export TMPDIR=/tmp` "
            "and cd back):\n")
    for c in cmds:
        f.write(f"  {c}\n")
    f.write("\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("mode", choices=["kernels", "counters", "traffic", "phases"])
    ap.add_argument("paths", nargs="+")
    ap.add_argument("--cmd", action="append", default=[])
    ap.add_argument("--copy-bytes", type=int, default=0)
    ap.add_argument("--note", action="append", default=[])
    ap.add_argument("--cycle", action="append", default=[],
                    help="phases mode: kernel=launches per pass, e.g. fwd_worker_kernel=3")
    a = ap.parse_args()
    out = a.paths[-1]
    with open(out, "w") as f:
        _header(f, a.cmd)
        for n in a.note:
            f.write(n + "\n")
        if a.note:
            f.write("\n")
        if a.mode == "kernels":
            f.write("%-64s %6s %12s %12s %7s\n" % ("kernel", "calls", "total_us", "avg_us", "pct"))
            for n, calls, tot, avg, pct in kernel_rows(_db(a.paths[0])):
                f.write("%-64s %6d %12.1f %12.3f %7.2f\n" % (_short(n), calls, tot, avg, pct))
        elif a.mode == "phases":
            cycles = {c.split("=")[0]: int(c.split("=")[1]) for c in a.cycle}
            for k, phs in sorted(counter_avgs_by_cycle(_db(a.paths[0]), cycles).items()):
                for ph, d in sorted(phs.items()):
                    f.write(f"{k} launch {ph} of {cycles[k]}\n")
                    for n, (v, c) in sorted(d.items()):
                        f.write("   %-34s avg/dispatch=%.6g  (dispatches=%d)\n" % (n, v, c))
        elif a.mode == "counters":
            for k, d in sorted(counter_avgs(_db(a.paths[0])).items()):
                f.write(_short(k) + "\n")
                for n, (v, c) in sorted(d.items()):
                    f.write("   %-34s avg/dispatch=%.6g  (dispatches=%d)\n" % (n, v, c))
        else:
            fetch = counter_avgs(_db(a.paths[0]))
            write = counter_avgs(_db(a.paths[1]))
            copy_f = [d["FETCH_SIZE"][0] for k, d in fetch.items() if COPY_KERNEL in k]
            copy_w = [d["WRITE_SIZE"][0] for k, d in write.items() if COPY_KERNEL in k]
            if not copy_f or not copy_w or not a.copy_bytes:
                raise SystemExit("calibration copy kernel not found in both runs, or --copy-bytes missing")
            fs, wsc = a.copy_bytes / copy_f[0], a.copy_bytes / copy_w[0]
            f.write(f"{COPY_KERNEL}: {a.copy_bytes} bytes read and written per launch; counters read "
                    f"FETCH_SIZE={copy_f[0]:.6g} WRITE_SIZE={copy_w[0]:.6g} per dispatch\n")
            f.write(f"scale: bytes per FETCH_SIZE unit = {fs:.2f}, per WRITE_SIZE unit = {wsc:.2f} "
                    "(1024 would be exact KiB)\n\n")
            for k in sorted(fetch):
                if k not in write or COPY_KERNEL in k:
                    continue
                fb = fetch[k]["FETCH_SIZE"][0] * fs
                wb = write[k]["WRITE_SIZE"][0] * wsc
                f.write("%s fetch_bytes_per_launch=%.0f write_bytes_per_launch=%.0f "
                        "traffic_bytes_per_launch=%.0f\n" % (_short(k), fb, wb, fb + wb))
    print(open(out).read())


if __name__ == "__main__":
    main()
