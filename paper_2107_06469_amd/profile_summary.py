"""Summarises a rocprofv3 kernel trace (rocpd SQLite output) as short text.

    python -m paper_2107_06469_amd.profile_summary <results.db> [--last-seconds S] [--skip-first N]

Prints, per kernel, the number of dispatches, total / average / min / max duration, and for the
whole window the GPU-busy fraction: the union of all kernel intervals divided by the span from the
first kernel start to the last kernel end.  With --window-kernel NAME the window is restricted to
the span between the first and last dispatch whose name contains NAME (e.g. the training kernels),
so set-up work before the timed region does not dilute the figure.
"""
from __future__ import annotations

import argparse
import re
import sqlite3
from collections import defaultdict


def _demangle(name: str) -> str:
    import shutil
    import subprocess
    tool = shutil.which("c++filt") or shutil.which("llvm-cxxfilt") or "/opt/rocm/lib/llvm/bin/llvm-cxxfilt"
    try:
        return subprocess.run([tool, name.replace(".kd", "")], capture_output=True, text=True, timeout=10).stdout.strip() or name
    except Exception:
        return name


_cache = {}


def short(name: str) -> str:
    if name not in _cache:
        _cache[name] = _short(_demangle(name))
    return _cache[name]


def _short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "").replace("void ", "").replace("hydra::", "")
    name = re.sub(r"\(.*$", "", name)
    return name[:96]


def load(db: str):
    c = sqlite3.connect(db)
    rows = c.execute(
        "select s.kernel_name, d.start, d.end, d.stream_id, d.grid_size_x, d.workgroup_size_x "
        "from rocpd_kernel_dispatch d join rocpd_info_kernel_symbol s on d.kernel_id = s.id order by d.start").fetchall()
    return [(short(r[0]), int(r[1]), int(r[2]), r[3], r[4], r[5]) for r in rows]


def busy_fraction(intervals):
    """Union length of [start,end) intervals over the span they cover."""
    if not intervals:
        return 0.0, 0
    intervals = sorted(intervals)
    total, cur_s, cur_e = 0, intervals[0][0], intervals[0][1]
    for s, e in intervals[1:]:
        if s > cur_e:
            total += cur_e - cur_s
            cur_s, cur_e = s, e
        else:
            cur_e = max(cur_e, e)
    total += cur_e - cur_s
    span = max(e for _, e in intervals) - intervals[0][0]
    return total / span, span


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("db")
    ap.add_argument("--window-kernel", default=None, help="restrict the window to dispatches between the first and last "
                                                          "kernel whose name contains this text")
    ap.add_argument("--skip-fraction", type=float, default=0.0,
                    help="drop this leading fraction of the window (warm-up) before computing the figures")
    args = ap.parse_args()
    rows = load(args.db)
    if args.window_kernel:
        idx = [i for i, r in enumerate(rows) if args.window_kernel in r[0]]
        rows = rows[idx[0]: idx[-1] + 1] if idx else []
    if args.skip_fraction > 0 and rows:
        t0, t1 = rows[0][1], max(r[2] for r in rows)
        cut = t0 + args.skip_fraction * (t1 - t0)
        rows = [r for r in rows if r[1] >= cut]
    per = defaultdict(list)
    for name, s, e, *_ in rows:
        per[name].append(e - s)
    frac, span = busy_fraction([(r[1], r[2]) for r in rows])
    print(f"dispatches: {len(rows)}   window: {span / 1e6:.3f} ms   GPU busy (union of kernel intervals / window): {100 * frac:.1f} %")
    tot = sum(sum(v) for v in per.values())
    print(f"sum of kernel durations: {tot / 1e6:.3f} ms  ({tot / max(span, 1):.2f} x window: >1 means kernels overlapped)")
    print(f"{'kernel':<98}{'calls':>7}{'total ms':>11}{'avg us':>10}{'min us':>10}{'max us':>10}{'share':>8}")
    for name, v in sorted(per.items(), key=lambda kv: -sum(kv[1])):
        print(f"{name:<98}{len(v):>7}{sum(v) / 1e6:>11.3f}{sum(v) / len(v) / 1e3:>10.1f}{min(v) / 1e3:>10.1f}"
              f"{max(v) / 1e3:>10.1f}{100 * sum(v) / tot:>7.1f}%")


if __name__ == "__main__":
    main()
