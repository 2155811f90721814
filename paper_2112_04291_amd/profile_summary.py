"""Turns rocprofv3 CSV output of `bench.py` runs into the short summaries kept under profiles/.

    python3 -m paper_2112_04291_amd.profile_summary trace   <dir> <out.md> "<what was run>" "<command>"
    python3 -m paper_2112_04291_amd.profile_summary traffic <fetch dir> <write dir> <out.md> <n_values> "<what>" "<command>"
    python3 -m paper_2112_04291_amd.profile_summary sq      <dir> <out.md> "<what>" "<command>"

`trace`   : <dir> holds the output of `rocprofv3 --kernel-trace --stats --output-format csv`.
`traffic` : the two directories hold `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of
            `bench.py --calibrate`, whose first large dispatch is a plain elementwise kernel over the
            value array (out = -in: n_values * 4 bytes read and as many written).  Both counters report
            KiB per dispatch; each is scaled by (known KiB of that kernel) / (what the counter read
            for it).
`sq`      : <dir> holds a `rocprofv3 --pmc SQ_...` run; per kernel the average of every counter per launch.
"""
import collections
import csv
import glob
import re
import sys


def _rows(d, suffix):
    files = glob.glob(d + "/**/*" + suffix, recursive=True)
    if not files:
        raise SystemExit(f"no *{suffix} under {d}")
    return list(csv.DictReader(open(files[0])))


_DECODE_MODES = {"0": "k_decode", "1": "k_decode (aggregate)", "2": "k_decode (Adam)"}


def _short(name):
    name = name.split("(")[0].replace("void ", "").replace("fsgd::", "").strip()
    m = re.match(r"k_decode<(\d)[^>]*>", name)
    if m:          # what the launch does with the pairs: store / add to a dense vector / Adam step
        return _DECODE_MODES.get(m.group(1), "k_decode")
    if name.startswith(("k_encode_values<", "k_pack_keys<")):     # the instantiation for calls with a tau above 128
        arg = name.split("<", 1)[1].rstrip(">").replace("(bool)", "").strip()
        return name.split("<")[0] + (" (16-bit codes)" if arg in ("true", "1") else "")
    return name.split("<")[0] if name.startswith("k_") else name[:60]


def trace(d, out, what, command):
    rows = _rows(d, "kernel_trace.csv")
    st = collections.defaultdict(list)
    meta = {}
    seen = set()
    for r in sorted(rows, key=lambda r: int(r["Start_Timestamp"])):
        k = _short(r["Kernel_Name"])
        if k.startswith("k_") and k not in seen:   # a kernel's first launch in the process can include loading its code
            seen.add(k)
            continue
        st[k].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
        meta[k] = (r.get("VGPR_Count", ""), r.get("LDS_Block_Size", ""), r.get("Grid_Size_X", r.get("Grid_Size", "")),
                   r.get("Workgroup_Size_X", r.get("Workgroup_Size", "")))
    tot = sum(sum(v) for v in st.values())
    with open(out, "w") as f:
        f.write(f"# rocprofv3 kernel trace: {what}\n\n")
        f.write(f"Command: `{command}`\n\n")
        f.write("Durations in microseconds, begin to end of each dispatch; the first launch of each of the library's "
                "kernels in the process is left out (it can include loading the kernel's code).\n\n")
        f.write("| kernel | calls | avg us | min us | max us | % of GPU time | VGPRs | LDS bytes | grid | workgroup |\n")
        f.write("|---|---|---|---|---|---|---|---|---|---|\n")
        for k, v in sorted(st.items(), key=lambda kv: -sum(kv[1])):
            if not k.startswith("k_") and 100.0 * sum(v) / tot < 0.5:
                continue
            m = meta[k]
            f.write(f"| {k} | {len(v)} | {sum(v) / len(v) / 1e3:.1f} | {min(v) / 1e3:.1f} | {max(v) / 1e3:.1f} | "
                    f"{100.0 * sum(v) / tot:.1f} | {m[0]} | {m[1]} | {m[2]} | {m[3]} |\n")


def _counter(d, name):
    """({kernel: [value per dispatch]}, (value, kernel) of the calibration dispatch: the first one, in
    dispatch order, that is not one of the library's kernels and moved a large amount)."""
    per = collections.defaultdict(list)
    rows = [r for r in _rows(d, "counter_collection.csv") if r["Counter_Name"] == name]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    first = None
    for r in rows:
        k, v = _short(r["Kernel_Name"]), float(r["Counter_Value"])
        per[k].append(v)
        if first is None and not k.startswith("k_") and v > 100000.0:
            first = (v, k)
    return per, first or (0.0, "")


def traffic(dfetch, dwrite, out, n_values, what, command):
    known_kib = n_values * 4.0 / 1024.0
    (fetch, fb), (write, wb) = _counter(dfetch, "FETCH_SIZE"), _counter(dwrite, "WRITE_SIZE")
    ff = known_kib / fb[0] if fb[0] > 0 else float("nan")
    wf = known_kib / wb[0] if wb[0] > 0 else float("nan")
    with open(out, "w") as f:
        f.write(f"# HBM traffic per launch: {what}\n\n")
        f.write(f"Commands: `{command.replace('COUNTER', 'FETCH_SIZE')}` and the same with `WRITE_SIZE`.\n\n")
        f.write(f"Calibration: the plain elementwise kernel over the value array ({n_values} x 4 bytes = "
                f"{known_kib:.0f} KiB each way) read FETCH_SIZE = {fb[0]:.0f} and WRITE_SIZE = {wb[0]:.0f} "
                f"(dispatch `{fb[1]}`), so "
                f"the counters are scaled by {ff:.4f} and {wf:.4f}.  Averages over all launches of a kernel in "
                f"the run; the last column is the scaled fetch + write in bytes.\n\n")
        f.write("| kernel | launches | FETCH_SIZE KiB avg | WRITE_SIZE KiB avg | HBM bytes per launch |\n")
        f.write("|---|---|---|---|---|\n")
        for k in sorted(set(fetch) | set(write)):
            if not k.startswith("k_"):
                continue
            fv, wv = fetch.get(k, [0.0]), write.get(k, [0.0])
            fa, wa = sum(fv) / len(fv), sum(wv) / len(wv)
            f.write(f"| {k} | {len(fv)} | {fa:.1f} | {wa:.1f} | {(fa * ff + wa * wf) * 1024.0:.4e} |\n")


def sq(d, out, what, command):
    rows = _rows(d, "counter_collection.csv")
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    names = []
    for r in rows:
        k = _short(r["Kernel_Name"])
        if not k.startswith("k_"):
            continue
        per[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
        if r["Counter_Name"] not in names:
            names.append(r["Counter_Name"])
    with open(out, "w") as f:
        f.write(f"# Shader counters per launch: {what}\n\n")
        f.write(f"Command: `{command}`\n\n")
        f.write("Average per launch of every counter, summed over the whole GPU (instruction counters count wave "
                "instructions; cycle counters are summed over waves or compute units as the counter defines).\n\n")
        f.write("| kernel | launches | " + " | ".join(n.replace("SQ_", "") for n in names) + " |\n")
        f.write("|---|---|" + "---|" * len(names) + "\n")
        for k in sorted(per):
            n_l = max(len(v) for v in per[k].values())
            cells = []
            for n in names:
                v = per[k].get(n, [])
                cells.append(f"{sum(v) / len(v):.4g}" if v else "")
            f.write(f"| {k} | {n_l} | " + " | ".join(cells) + " |\n")


if __name__ == "__main__":
    a = sys.argv
    if len(a) >= 6 and a[1] == "trace":
        trace(a[2], a[3], a[4], a[5])
    elif len(a) >= 8 and a[1] == "traffic":
        traffic(a[2], a[3], a[4], int(a[5]), a[6], a[7])
    elif len(a) >= 6 and a[1] == "sq":
        sq(a[2], a[3], a[4], a[5])
    else:
        raise SystemExit(__doc__)
