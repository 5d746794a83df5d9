"""Turns rocprofv3 CSV output of a bench.py run into the short text summaries kept under
profiles/.

    python -m paper_2604_12056_amd.profile_summary trace  <dir-with-*_kernel_trace.csv>
    python -m paper_2604_12056_amd.profile_summary traffic <fetch-dir> <write-dir> --copy-bytes N
    python -m paper_2604_12056_amd.profile_summary counters <dir> [<dir> ...]

`trace` prints calls / mean / min / max duration per kernel.  `traffic` reads two counter
runs (FETCH_SIZE in one, WRITE_SIZE in the other; KiB per dispatch), scales each counter by
what it reads for the library's calibration copy kernel of known size, and prints HBM bytes
per launch for every kernel of the library, in the key: value form bench.py reads back.
`counters` prints, for every kernel of the library, the mean per launch of every counter found
in the given counter runs (one table row per kernel and run), plus the derived figures the
matrix-core kernels are judged by: matrix-core busy, vector-ALU busy and both-at-once cycles as
fractions of the kernel's busy cycles."""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os
import re
import sys


def _short(name: str) -> str:
    name = re.sub(r"\(.*", "", name)
    return name.replace("void ", "").strip()


def _find(directory: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit(f"no *{suffix} under {directory}")
    return hits[0]


def trace(directory: str) -> None:
    rows = list(csv.DictReader(open(_find(directory, "_kernel_trace.csv"))))
    dur = collections.defaultdict(list)
    for r in rows:
        dur[_short(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in dur.values())
    print(f"{'kernel':78s} {'calls':>6s} {'mean_us':>9s} {'min_us':>9s} {'max_us':>9s} {'share':>6s}")
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        print(f"{k[:78]:78s} {len(v):6d} {sum(v) / len(v):9.2f} {min(v):9.2f} {max(v):9.2f} {100 * sum(v) / total:5.1f}%")


def _counter(directory: str, counter: str):
    rows = csv.DictReader(open(_find(directory, "_counter_collection.csv")))
    acc = collections.defaultdict(list)
    for r in rows:
        if r["Counter_Name"] == counter:
            acc[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}, {k: len(v) for k, v in acc.items()}


def traffic(fetch_dir: str, write_dir: str, copy_bytes: int) -> None:
    fetch, n = _counter(fetch_dir, "FETCH_SIZE")
    write, _ = _counter(write_dir, "WRITE_SIZE")
    copy = [k for k in fetch if "calibration_copy_kernel" in k]
    if not copy:
        raise SystemExit("the calibration copy kernel is not in the counter run")
    f_scale = copy_bytes / (fetch[copy[0]] * 1024.0)
    w_scale = copy_bytes / (write[copy[0]] * 1024.0)
    print(f"# calibration copy of {copy_bytes} bytes: FETCH_SIZE read {fetch[copy[0]]:.1f} KiB, WRITE_SIZE read "
          f"{write[copy[0]]:.1f} KiB -> scale factors {f_scale:.4f} (fetch), {w_scale:.4f} (write)")
    print(f"{'# kernel':70s} {'launches':>8s} {'fetch_bytes':>14s} {'write_bytes':>14s}")
    for k in sorted(fetch):
        if "losa::" not in k:
            continue
        fb, wb = fetch[k] * 1024.0 * f_scale, write.get(k, 0.0) * 1024.0 * w_scale
        print(f"# {k[:68]:68s} {n[k]:8d} {fb:14.0f} {wb:14.0f}")
    for k in sorted(fetch):
        # the sparse-step attention kernel is the split-pages shape: fourth template argument true
        if re.search(r"attn_mfma_kernel<\d+, \d+, \d+, true\b", k):
            print(f"attn_fetch_bytes_per_launch: {fetch[k] * 1024.0 * f_scale:.0f}")
            print(f"attn_write_bytes_per_launch: {write.get(k, 0.0) * 1024.0 * w_scale:.0f}")
            break


def counters(dirs) -> None:
    """Mean counter values per launch.  The SQ_* cycle counters count per SIMD (MFMA busy, co-execution)
    or per wavefront in units of four cycles (ACTIVE_INST_*, WAVE_CYCLES, WAIT_*), BUSY_CU_CYCLES per
    compute unit; the derived fractions put each on the kernel's own duration in cycles."""
    for d in dirs:
        rows = csv.DictReader(open(_find(d, "_counter_collection.csv")))
        acc = collections.defaultdict(lambda: collections.defaultdict(list))
        for r in rows:
            acc[_short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
        names = sorted({c for v in acc.values() for c in v})
        print(f"# counter run {os.path.basename(os.path.normpath(d))}: " + " ".join(names))
        for k in sorted(acc):
            if "losa::" not in k:
                continue
            v = {c: sum(x) / len(x) for c, x in acc[k].items()}
            n = len(next(iter(acc[k].values())))
            print(f"{k[:84]:84s} launches {n}")
            for c in names:
                if c in v:
                    print(f"    {c:34s} {v[c]:18.1f}")
            cu = v.get("SQ_BUSY_CU_CYCLES")
            if cu:
                # 256 compute units x 4 SIMDs; a kernel that keeps every unit busy for its whole duration has
                # BUSY_CU_CYCLES = 256 x duration in cycles
                dur = cu / 256.0
                if "SQ_VALU_MFMA_BUSY_CYCLES" in v:
                    print(f"    {'matrix-core busy / duration':34s} {v['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024.0 / dur:18.3f}")
                if "SQ_VALU_MFMA_COEXEC_CYCLES" in v:
                    print(f"    {'matrix + vector at once / duration':34s} {v['SQ_VALU_MFMA_COEXEC_CYCLES'] / 1024.0 / dur:18.3f}")
                if "SQ_ACTIVE_INST_VALU" in v:
                    print(f"    {'vector-ALU issue busy / duration':34s} {v['SQ_ACTIVE_INST_VALU'] * 4.0 / 1024.0 / dur:18.3f}")


def main(argv=None) -> None:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("dir")
    f = sub.add_parser("traffic")
    f.add_argument("fetch_dir")
    f.add_argument("write_dir")
    f.add_argument("--copy-bytes", type=int, required=True)
    c = sub.add_parser("counters")
    c.add_argument("dirs", nargs="+")
    a = ap.parse_args(argv)
    if a.cmd == "trace":
        trace(a.dir)
    elif a.cmd == "counters":
        counters(a.dirs)
    else:
        traffic(a.fetch_dir, a.write_dir, a.copy_bytes)


if __name__ == "__main__":
    main()
