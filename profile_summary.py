#!/usr/bin/env python3
"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under
profiles/.  Nothing here runs the GPU: it only reads what rocprofv3 wrote.

  kernel statistics (from `rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o bench -- python3 bench.py ...`):
      python3 profile_summary.py stats DIR --bench-json FILE --out profiles/NAME.txt --cmd "..."
  HBM traffic (two runs, `--pmc FETCH_SIZE` and `--pmc WRITE_SIZE`, same -d/-o convention):
      python3 profile_summary.py traffic FETCH_DIR WRITE_DIR --out profiles/NAME.txt --json profiles/NAME.json --cmd "..."
  any other counters (one run per `--pmc` set):
      python3 profile_summary.py counters DIR [DIR ...] --out profiles/NAME.txt --cmd "..."

Kernels are told apart by name: kv_block_copy<U, NT, W, KIND> with KIND 0 gather (pool ->
records), 1 scatter (records -> pool), 2 fused (pool -> pool); plain_copy_kernel is the
contiguous yardstick whose counter readings calibrate the others.
"""
import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import re

ROOT = os.path.dirname(os.path.abspath(__file__))
KINDS = {"0": "gather", "1": "scatter", "2": "fused", "3": "records"}
OURS = ("kv_block_copy", "plain_copy_kernel", "block_hash_kernel",
        "index_probe_kernel", "index_apply_kernel")


def short(name):
    """Library kernel -> short label, anything else -> None."""
    for k in OURS:
        i = name.find(k + "<") if k == "kv_block_copy" else name.find(k)
        if i < 0:
            continue
        if k == "kv_block_copy":
            m = re.match(r"kv_block_copy<(\d+), (true|false), (\d+)(?:, (?:\(mempool::\(anonymous namespace\)::CopyKind\))?(\d+))?>", name[i:])
            if not m:
                return "kv_block_copy"
            u, nt, w, kind = m.groups()
            return f"kv_block_copy<{u},{nt},{w}> {KINDS.get(kind, '?') if kind is not None else ''}".strip()
        return k
    return None


def one(pattern):
    hits = glob.glob(pattern, recursive=True)
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return hits[0]


def kernel_sha():
    h = hashlib.sha256()
    for f in ("kv_copy.hip", "kv_copy.hpp"):
        with open(os.path.join(ROOT, "paper_2406_17565_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def cmd_stats(a):
    rows = []
    with open(one(os.path.join(a.dirs[0], "**", "*kernel_stats.csv"))) as f:
        for r in csv.DictReader(f):
            s = short(r["Name"])
            if s:
                rows.append((s, int(r["Calls"]), int(r["TotalDurationNs"]), float(r["AverageNs"]),
                             int(r["MinNs"]), int(r["MaxNs"]), r["Percentage"]))
    L = [a.title or "rocprofv3 kernel-trace statistics of bench.py", f"command: {a.cmd}",
         "(run from the repository root on the MI355X box after `cd /tmp && export TMPDIR=/tmp`; only "
         "this library's kernels are listed, torch's fill / RNG kernels of the harness are left out)", "",
         f"{'kernel':<36}{'calls':>7}{'total_ns':>14}{'avg_ns':>13}{'min_ns':>11}{'max_ns':>11}{'pct':>8}"]
    for s, c, tot, avg, mn, mx, pct in sorted(rows, key=lambda r: -r[2]):
        L.append(f"{s:<36}{c:>7}{tot:>14}{avg:>13.1f}{mn:>11}{mx:>11}{pct:>8}")
    if a.bench_json:
        b = json.load(open(a.bench_json))
        rf = b["roofline"]
        if "avg_launch_us" not in rf:          # a side mode of bench.py (host tier, ...): quote its line as it is
            L += ["", "bench.py's line in the same run: " + json.dumps({k: v for k, v in b.items() if k != "config"})]
            write(a.out, L)
            return
        L += ["", f"bench.py's own HIP-event timing in the same run: {rf['kernel']} avg {rf['avg_launch_us']} us over "
                  f"{rf['launches']} timed launches (the trace also counts warm-up launches and the extra legs);",
              f"algorithmic bytes per launch {rf['alg_bytes_per_launch']} => {rf['achieved']} GB/s = "
              f"{rf['frac'] * 100:.1f} % of {rf['peak']:.0f} GB/s; per kind {rf.get('per_kind_GBs')}; plain contiguous copy "
              f"on the same box {rf.get('plain_copy_ceiling_GBs')} GB/s.",
              f"value {b['value']} {b['unit']}, {b['ms_per_step']} ms/step under the profiler."]
        for key in ("fused", "roofline_hash", "per_request"):
            if b.get(key):
                L.append(f"{key}: {json.dumps(b[key])}")
    write(a.out, L)


def read_counters(d):
    """{kernel label: {counter: [(value, grid, wg_size), ...]}} of one --pmc run directory."""
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(one(os.path.join(d, "**", "*counter_collection.csv"))) as f:
        for r in csv.DictReader(f):
            s = short(r["Kernel_Name"])
            if s:
                out[s][r["Counter_Name"]].append((float(r["Counter_Value"]), int(r["Grid_Size"]),
                                                  int(r["Workgroup_Size"])))
    return out


def moved_kib(label, grid, wg):
    """KiB read (= KiB written) by one launch, from its grid: one wave-item moves U KiB."""
    if label.startswith("plain_copy_kernel"):
        return grid * 16 / 1024
    m = re.match(r"kv_block_copy<(\d+),", label)
    return (grid // 64) * int(m.group(1)) if m else None


def cmd_traffic(a):
    fetch, wr = read_counters(a.dirs[0]), read_counters(a.dirs[1])
    cal_f = [(v, moved_kib("plain_copy_kernel", g, w)) for v, g, w in fetch["plain_copy_kernel"]["FETCH_SIZE"]]
    cal_w = [(v, moved_kib("plain_copy_kernel", g, w)) for v, g, w in wr["plain_copy_kernel"]["WRITE_SIZE"]]
    fs = sum(k for _, k in cal_f) / sum(v for v, _ in cal_f)      # KiB per count
    ws = sum(k for _, k in cal_w) / sum(v for v, _ in cal_w)
    L = [a.title or "HBM traffic of kv_block_copy from rocprofv3 counters, bench.py",
         f"commands (one counter per run): {a.cmd}", "",
         f"calibration: plain_copy_kernel moves {cal_f[0][1]:.0f} KiB each way per launch; FETCH_SIZE reads "
         f"{cal_f[0][0]:.1f} => {fs:.4f} KiB per count; WRITE_SIZE reads {cal_w[0][0]:.1f} => {ws:.4f} KiB per count", "",
         f"{'kernel':<34}{'launches':>9}{'alg_KiB each way':>18}{'fetch_KiB':>14}{'write_KiB':>14}{'traffic/alg':>13}"]
    res = {}
    for label in sorted(fetch):
        if not label.startswith("kv_block_copy"):
            continue
        fv, wv = fetch[label]["FETCH_SIZE"], wr[label]["WRITE_SIZE"]
        n = min(len(fv), len(wv))
        alg = sum(moved_kib(label, g, w) for _, g, w in fv[:n])
        fk, wk = sum(v for v, _, _ in fv[:n]) * fs, sum(v for v, _, _ in wv[:n]) * ws
        ratio = (fk + wk) / (2 * alg)
        res[label] = round(ratio, 4)
        L.append(f"{label:<34}{n:>9}{alg:>18.0f}{fk:>14.0f}{wk:>14.0f}{ratio:>13.4f}")
    L += ["", "traffic/alg = (HBM bytes fetched + written) / (bytes the table says must be read + written); 1.0 = every "
              "byte read once and written once.  alg_KiB counts whole wave-items, an upper bound of the table bytes by < 0.01 %."]
    write(a.out, L)
    if a.json:
        lab = [k for k in res if not k.endswith("records")]
        json.dump({"traffic_per_algorithmic_byte": {k.split("> ")[-1]: v for k, v in res.items()},
                   "fetch_scale_KiB_per_count": round(fs, 4), "write_scale_KiB_per_count": round(ws, 4),
                   "kernel_source_sha": kernel_sha(), "kernels": lab}, open(a.json, "w"))


def cmd_counters(a):
    merged = collections.defaultdict(dict)
    launches = {}
    for d in a.dirs:
        for label, ctrs in read_counters(d).items():
            for c, vals in ctrs.items():
                kib = [moved_kib(label, g, w) for _, g, w in vals]
                tot = sum(v for v, _, _ in vals)
                merged[label][c] = (tot / len(vals), tot / sum(kib) * 1024 if all(kib) and sum(kib) else None)
                launches[label] = len(vals)
    names = sorted({c for v in merged.values() for c in v})
    labels = [k for k in sorted(merged) if k.startswith(("kv_block_copy", "plain_copy"))] or sorted(merged)
    L = [a.title or "rocprofv3 hardware counters of bench.py, per kernel", f"commands (one run per counter set): {a.cmd}", "",
         "mean per launch, and in brackets per MiB the launch reads (= writes):", "",
         f"{'counter':<44}" + "".join(f"{k.replace('kv_block_copy', 'kvc'):>30}" for k in labels)]
    L.append(f"{'launches':<44}" + "".join(f"{launches[k]:>30}" for k in labels))
    for c in names:
        cells = []
        for k in labels:
            v = merged[k].get(c)
            cells.append("-" if v is None else f"{v[0]:.4g} [{v[1]:.4g}]" if v[1] is not None else f"{v[0]:.4g}")
        L.append(f"{c:<44}" + "".join(f"{x:>30}" for x in cells))
    write(a.out, L)


def write(path, lines):
    text = "\n".join(lines) + "\n"
    if path:
        with open(path, "w") as f:
            f.write(text)
    print(text)


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("mode", choices=["stats", "traffic", "counters"])
    ap.add_argument("dirs", nargs="+")
    ap.add_argument("--bench-json")
    ap.add_argument("--out")
    ap.add_argument("--json")
    ap.add_argument("--title")
    ap.add_argument("--cmd", default="(not recorded)")
    a = ap.parse_args()
    {"stats": cmd_stats, "traffic": cmd_traffic, "counters": cmd_counters}[a.mode](a)
