"""Turns rocprofv3 output of bench.py runs into the short summaries kept under profiles/.

    python -m paper_2012_03096_amd.profile_summary trace   RESULTS.db --steps N --title T --command CMD --out profiles/X.md
    python -m paper_2012_03096_amd.profile_summary traffic --workload NAME --steps N --fetch F.csv --write W.csv
                                                           --copy-fetch CF.csv --copy-write CW.csv --copy-mib 256
                                                           --command CMD --out profiles/X.md --json profiles/hbm_traffic.json

`trace`: per-kernel calls, total and average duration from the `kernels` view of a `rocprofv3 --kernel-trace --stats`
run's rocpd database, normalised per step (N = every step the command ran: warm-up and timed ones).
`traffic`: per-kernel HBM bytes per launch from two `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE; CSV output),
each scaled by what the same counter reads for a plain device copy of known size (bench.py --calibrate-copy), written as
a table and merged into the JSON file bench.py reads its `traffic` figures from.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import sqlite3

# kernel name fragment -> the library's kernel kind (pbkd_kernel_kind_name) the bench reports it under
KIND_OF = [
    ("conv_mfma_kernel", "conv_mfma_kernel"), ("conv_split_kernel", "conv_split_kernel"), ("conv_first_kernel", "conv3x3_first"), ("conv_ksplit_finish", "conv_ksplit_finish"),
    ("dw_fwd", "dw3x3_fwd"), ("dw_bwd_finalize", "reduce_partials"), ("dw_bwd", "dw3x3_bwd"), ("dwpw_fwd", "dwpw_fwd"),
    ("bn_bwd_apply", "bn_bwd_apply"), ("head_kernel<0", "head_out"), ("head_kernel<1", "head_loss"), ("head_kernel<2", "head_bwd"),
    ("reduce_update", "sgd_momentum"), ("conv_wgrad_kernel", "conv3x3_wgrad"), ("wgrad_taps_bn_kernel", "conv3x3_wgrad"), ("pw_wgrad_kernel", "pw_wgrad_mfma"),
    ("pw_mfma", "pw_mfma (forward and data gradient)"), ("bn_finalize", "bn_finalize"), ("head_finalize", "reduce_partials"),
]


def kind_of(kernel_name: str) -> str:
    if "pw_wgrad_kernel" in kernel_name and kernel_name.rstrip().split(">")[0].endswith(", 3"):
        return "conv3x3_wgrad"
    for frag, kind in KIND_OF:
        if frag in kernel_name:
            return kind
    return "other"


def short(name: str, n: int = 100) -> str:
    return name.replace("|", "\\|")[:n]


def cmd_trace(a):
    db = sqlite3.connect(a.db)
    rows = db.execute("select name, start, end from kernels order by start").fetchall()
    agg = collections.OrderedDict()
    for name, s, e in rows:
        rec = agg.setdefault(name, [0, 0.0])
        rec[0] += 1
        rec[1] += (e - s) / 1e3
    total = sum(v[1] for v in agg.values())
    md = [f"# {a.title}\n", "Command (from /tmp on the MI355X box, `R` = repository root):\n", f"    {a.command}\n",
          f"{a.steps} steps in all (warm-up and timed).  Durations in microseconds from the `kernels` view of the run's rocpd "
          f"database; {total / a.steps:.1f} us of kernel time per step over the `pbkd::` and helper kernels below.\n"]
    if a.note:
        md.append(a.note + "\n")
    md += ["| kernel | calls | calls/step | total us | avg us | us/step | % |", "|---|---|---|---|---|---|---|"]
    for name, (c, us) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        md.append("| %s | %d | %.2f | %.1f | %.2f | %.2f | %.2f |" % (short(name), c, c / a.steps, us, us / c, us / a.steps, 100 * us / total))
    with open(a.out, "w") as f:
        f.write("\n".join(md) + "\n")
    print("wrote", a.out)


def _pmc(path):
    agg = collections.defaultdict(list)
    with open(path) as f:
        for r in csv.DictReader(f):
            agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in agg.items()}


def cmd_traffic(a):
    copy_bytes = a.copy_mib << 20
    cf = [v for k, v in _pmc(a.copy_fetch).items() if "copy" in k.lower()]
    cw = [v for k, v in _pmc(a.copy_write).items() if "copy" in k.lower()]
    if not cf or not cw:
        raise SystemExit("no copy kernel found in the calibration runs")
    fetch_unit = copy_bytes / cf[0][0]
    write_unit = copy_bytes / cw[0][0]
    fetch, write = _pmc(a.fetch), _pmc(a.write)
    md = [f"# HBM traffic per kernel launch (rocprofv3 --pmc), {a.workload}\n",
          "Commands (each from /tmp on the MI355X box, `R` = repository root; one counter per run):\n"]
    md += ["    " + c for c in a.command]
    md.append("\nCalibration: a device-to-device copy of %d MiB reads FETCH_SIZE = %.0f and WRITE_SIZE = %.0f per dispatch, i.e. one "
              "FETCH_SIZE unit = %.0f bytes and one WRITE_SIZE unit = %.0f bytes on this chip.\n" % (a.copy_mib, cf[0][0], cw[0][0], fetch_unit, write_unit))
    md += ["| kernel | kind | dispatches | read MB / launch | written MB / launch |", "|---|---|---|---|---|"]
    kinds = collections.defaultdict(lambda: [0.0, 0.0, 0])
    for name, (fv, n) in sorted(fetch.items(), key=lambda kv: -kv[1][0] * kv[1][1]):
        if "pbkd::" not in name:
            continue
        wv = write.get(name, (0.0, 0))[0]
        kind = kind_of(name)
        md.append("| %s | %s | %d | %.2f | %.2f |" % (short(name, 90), kind, n, fv * fetch_unit / 1e6, wv * write_unit / 1e6))
        rec = kinds[kind]
        rec[0] += fv * fetch_unit * n
        rec[1] += wv * write_unit * n
        rec[2] += n
    md.append("\nAverages per dispatch over the run (%d steps, one stream).\n" % a.steps)
    with open(a.out, "w") as f:
        f.write("\n".join(md) + "\n")
    data = {"workloads": {}}
    if os.path.exists(a.json):
        with open(a.json) as f:
            data = json.load(f)
    data.setdefault("workloads", {})[a.workload] = {
        "source": os.path.relpath(a.out, os.path.dirname(os.path.abspath(a.json)) or "."),
        "fetch_size_unit_bytes": fetch_unit, "write_size_unit_bytes": write_unit,
        "kernels": {k: {"fetch_bytes_per_launch": round(v[0] / v[2]), "write_bytes_per_launch": round(v[1] / v[2]), "launches": v[2]}
                    for k, v in sorted(kinds.items())}}
    with open(a.json, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", a.out, "and", a.json)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("db")
    t.add_argument("--steps", type=int, required=True)
    t.add_argument("--title", required=True)
    t.add_argument("--command", required=True)
    t.add_argument("--note", default="")
    t.add_argument("--out", required=True)
    t.set_defaults(fn=cmd_trace)
    p = sub.add_parser("traffic")
    p.add_argument("--workload", required=True)
    p.add_argument("--steps", type=int, required=True)
    p.add_argument("--fetch", required=True)
    p.add_argument("--write", required=True)
    p.add_argument("--copy-fetch", required=True)
    p.add_argument("--copy-write", required=True)
    p.add_argument("--copy-mib", type=int, default=256)
    p.add_argument("--command", action="append", default=[])
    p.add_argument("--out", required=True)
    p.add_argument("--json", required=True)
    p.set_defaults(fn=cmd_traffic)
    a = ap.parse_args()
    a.fn(a)


if __name__ == "__main__":
    main()
