"""Turns a rocprofv3 result database (rocpd SQLite) into the short text summaries kept under
profiles/: per-kernel durations from a --kernel-trace run, and per-kernel hardware byte counters
from --pmc FETCH_SIZE / WRITE_SIZE runs, calibrated against a plain copy of known size.

    python profile_summary.py stats  <results.db>
    python profile_summary.py pmc    <fetch.db> <write.db> --copy-mib 1024 \
           --kernel gemm_fused_kernel --launches-per-step 48 --steps 4
    python profile_summary.py counters <run1.db> <run2.db> ...      (one counter per run, any counters)

`source_hash()` identifies the kernel sources (comments and spacing aside) a counter summary belongs
to; bench.py quotes the traffic figure only while the hash still matches.
"""
from __future__ import annotations

import argparse
import hashlib
import os
import re
import sqlite3

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2207_02849_amd")
KERNEL_SOURCES = ["csrc/gemm.hip", "csrc/kernels.hip", "csrc/api.hip", "csrc/internal.h"]


def _code_only(text: str) -> str:
    """Source text without comments and with runs of white space collapsed: what the compiler sees,
    near enough (string literals in these sources hold no comment markers)."""
    text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
    text = re.sub(r"//[^\n]*", " ", text)
    return re.sub(r"\s+", " ", text).strip()


def source_hash() -> str:
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(HERE, rel), "r") as f:
            h.update(_code_only(f.read()).encode())
    return h.hexdigest()[:16]


def _tables(cur):
    tabs = [r[0] for r in cur.execute("select name from sqlite_master where type='table'")]
    pick = lambda key: [t for t in tabs if key in t][0]
    return pick, tabs


def _short(name: str) -> str:
    return re.sub(r"\(.*", "", name)


def kernel_stats(db_path: str):
    cur = sqlite3.connect(db_path).cursor()
    pick, _ = _tables(cur)
    kd, ks = pick("kernel_dispatch"), pick("info_kernel_symbol")
    q = (f"select s.kernel_name, count(*), sum(d.end-d.start), min(d.end-d.start), max(d.end-d.start) "
         f"from {kd} d join {ks} s on d.kernel_id = s.id group by s.kernel_name order by 3 desc")
    return [(_short(n), c, t / 1e3, mn / 1e3, mx / 1e3) for n, c, t, mn, mx in cur.execute(q)]


def print_stats(db_path: str):
    rows = kernel_stats(db_path)
    tot = sum(r[2] for r in rows)
    print(f"{'kernel':96s} {'calls':>7s} {'total_us':>10s} {'avg_us':>9s} {'min_us':>8s} {'max_us':>8s} {'%':>6s}")
    for name, n, t, mn, mx in rows:
        print(f"{name[:96]:96s} {n:7d} {t:10.1f} {t / n:9.2f} {mn:8.2f} {mx:8.2f} {100 * t / tot:6.1f}")
    print(f"total kernel time {tot:.1f} us")


def pmc_totals(db_path: str):
    """{kernel name: (calls, summed counter value in KiB)} for the single counter of a --pmc run."""
    cur = sqlite3.connect(db_path).cursor()
    pick, _ = _tables(cur)
    ev, info, kd, ks = pick("pmc_event"), pick("info_pmc"), pick("kernel_dispatch"), pick("info_kernel_symbol")
    q = (f"select s.kernel_name, i.name, count(distinct d.id), sum(e.value) from {ev} e "
         f"join {info} i on e.pmc_id = i.id join {kd} d on e.event_id = d.event_id "
         f"join {ks} s on d.kernel_id = s.id group by s.kernel_name, i.name")
    out = {}
    for name, counter, calls, val in cur.execute(q):
        out[_short(name)] = (counter, calls, float(val))
    return out


def print_pmc(fetch_db, write_db, copy_mib, kernel_filter, launches_per_step, steps):
    f, w = pmc_totals(fetch_db), pmc_totals(write_db)
    copy_kib = copy_mib * 1024.0
    # the calibration copy is the largest user of the copy kernel in the run
    def scale(tot):
        cands = [(v[2], k) for k, v in tot.items() if "copyBuffer" in k or "copy" in k.lower() and "convert" not in k]
        val, name = max(cands)
        return copy_kib / val, name, val
    sf, fname, fval = scale(f)
    sw, wname, wval = scale(w)
    print(f"source_hash: {source_hash()}")
    print(f"calibration: one plain device copy of {copy_mib} MiB ({fname}): FETCH_SIZE read {fval:.0f} KiB, "
          f"WRITE_SIZE read {wval:.0f} KiB -> scale factors fetch {sf:.3f}, write {sw:.3f}")
    print(f"{'kernel':96s} {'calls':>6s} {'fetch_MiB/call':>15s} {'write_MiB/call':>15s}")
    tot_f = tot_w = 0.0
    tot_calls = 0
    for name in sorted(set(f) | set(w), key=lambda k: -(f.get(k, (0, 0, 0))[2] * sf + w.get(k, (0, 0, 0))[2] * sw)):
        cf = f.get(name, ("", 0, 0.0))
        cw = w.get(name, ("", 0, 0.0))
        calls = max(cf[1], cw[1])
        if calls == 0:
            continue
        print(f"{name[:96]:96s} {calls:6d} {cf[2] * sf / 1024 / calls:15.2f} {cw[2] * sw / 1024 / calls:15.2f}")
        if kernel_filter in name:
            tot_f += cf[2] * sf * 1024
            tot_w += cw[2] * sw * 1024
            tot_calls += calls
    if launches_per_step and steps:
        n = launches_per_step * steps
        print(f"kernel filter '{kernel_filter}': {tot_calls} launches counted, expected {n}")
    if tot_calls:
        print(f"traffic_bytes_per_launch: {(tot_f + tot_w) / tot_calls:.0f}")
        print(f"fetch_bytes_per_launch: {tot_f / tot_calls:.0f}")
        print(f"write_bytes_per_launch: {tot_w / tot_calls:.0f}")


def print_counters(dbs, kernel_filter):
    """One table over several single-counter runs of the same command: per kernel, the launches and
    every counter's value per launch (the sum over the launches divided by their number, so a
    percentage such as MfmaUtil comes out as its mean over the launches)."""
    per = {}
    names = []
    for db in dbs:
        for kern, (counter, calls, val) in pmc_totals(db).items():
            per.setdefault(kern, {})[counter] = (calls, val)
            if counter not in names:
                names.append(counter)
    print(f"source_hash: {source_hash()}")
    print(f"{'kernel':96s} {'calls':>6s} " + " ".join(f"{n[:24]:>24s}" for n in names))
    for kern in sorted(per, key=lambda k: -max(c for c, _ in per[k].values())):
        if kernel_filter and kernel_filter not in kern:
            continue
        calls = max(c for c, _ in per[kern].values())
        cells = []
        for n in names:
            c, v = per[kern].get(n, (0, 0.0))
            cells.append(f"{v / c:24.4g}" if c else f"{'-':>24s}")
        print(f"{kern[:96]:96s} {calls:6d} " + " ".join(cells))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats")
    s.add_argument("db")
    p = sub.add_parser("pmc")
    p.add_argument("fetch_db")
    p.add_argument("write_db")
    p.add_argument("--copy-mib", type=int, required=True)
    p.add_argument("--kernel", default="gemm_fused_kernel")
    p.add_argument("--launches-per-step", type=int, default=0)
    p.add_argument("--steps", type=int, default=0)
    c = sub.add_parser("counters")
    c.add_argument("dbs", nargs="+")
    c.add_argument("--kernel", default="")
    a = ap.parse_args()
    if a.cmd == "stats":
        print_stats(a.db)
    elif a.cmd == "counters":
        print_counters(a.dbs, a.kernel)
    else:
        print_pmc(a.fetch_db, a.write_db, a.copy_mib, a.kernel, a.launches_per_step, a.steps)


if __name__ == "__main__":
    main()
