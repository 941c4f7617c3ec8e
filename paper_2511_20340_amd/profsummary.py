"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2511_20340_amd.profsummary stats  <*_kernel_stats.csv>        [--cmd "..."] [--top 16]
  python -m paper_2511_20340_amd.profsummary pmc    <*_counter_collection.csv>  --counter FETCH_SIZE
         --calib-kernel <name substring> --calib-bytes <bytes one calibration dispatch moves> [--cmd "..."]

`pmc` prints, per kernel, the mean counter value per dispatch and the bytes it corresponds to after
scaling by the calibration kernel (a plain copy of known size measured in the same run).
"""
import argparse
import collections
import csv
import re


# kernel classes as bench.py names them -> pattern over the kernel names
CLASSES = {"linear": r"gemm_(ring|f32)_kernel", "attention": r"attn_(bf16|f32)_kernel", "argmax": r"argmax_partial",
           "rmsnorm": r"rmsnorm_kernel", "rope_kv_append": r"rope_kv_kernel"}


def short(name):
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"^void ", "", name)
    name = re.sub(r"\(.*$", "", name)
    return name[:90]


def stats(path, top, cmd):
    rows = list(csv.DictReader(open(path)))
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    out = []
    if cmd:
        out.append(f"command: `{cmd}`\n")
    out.append("| kernel | calls | avg us | min us | max us | total ms | % of GPU time |")
    out.append("|---|---|---|---|---|---|---|")
    for r in rows[:top]:
        out.append("| %s | %s | %.1f | %.1f | %.1f | %.2f | %.1f |" % (
            short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
            float(r["MaxNs"]) / 1e3, float(r["TotalDurationNs"]) / 1e6, 100 * float(r["TotalDurationNs"]) / total))
    return "\n".join(out)


def pmc(path, counter, calib_kernel, calib_bytes, cmd):
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            per[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    calib = [v for k, vs in per.items() if calib_kernel in k for v in vs]
    if not calib:
        raise SystemExit(f"no dispatch of a kernel matching {calib_kernel!r} in {path}")
    calib_mean = sum(calib) / len(calib)
    scale = calib_bytes / calib_mean
    out = []
    if cmd:
        out.append(f"command: `{cmd}`\n")
    out.append(f"counter {counter}; calibration: {len(calib)} dispatches of `{calib_kernel}` moving {calib_bytes} "
               f"bytes each read {calib_mean:.1f} -> {scale:.2f} bytes per count\n")
    out.append("| kernel | dispatches | mean count | bytes per dispatch (scaled) |")
    out.append("|---|---|---|---|")
    for k, vs in sorted(per.items(), key=lambda kv: -sum(kv[1])):
        m = sum(vs) / len(vs)
        out.append("| %s | %d | %.1f | %.4g |" % (k, len(vs), m, m * scale))
    out = out[:40]
    # per kernel class, what bench.py reads back as roofline.traffic (dispatch-weighted mean)
    out.append("")
    for cls, pat in CLASSES.items():
        vs = [v for k, vals in per.items() if re.search(pat, k) for v in vals]
        if vs:
            out.append(f"traffic_per_launch {cls} {counter}: {sum(vs) / len(vs) * scale:.6g} bytes "
                       f"(mean of {len(vs)} dispatches)")
    return "\n".join(out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("mode", choices=["stats", "pmc"])
    ap.add_argument("csv")
    ap.add_argument("--cmd", default="")
    ap.add_argument("--top", type=int, default=16)
    ap.add_argument("--counter", default="FETCH_SIZE")
    ap.add_argument("--calib-kernel", default="")
    ap.add_argument("--calib-bytes", type=float, default=0)
    a = ap.parse_args()
    print(stats(a.csv, a.top, a.cmd) if a.mode == "stats" else
          pmc(a.csv, a.counter, a.calib_kernel, a.calib_bytes, a.cmd))


if __name__ == "__main__":
    main()
